// Shared device-side building blocks of libburstattn's gfx950 kernels.
//
// MFMA 32x32x16 bf16 register layouts (lane l: r = l % 32, h = l / 32):
//   A operand (M x K): lane holds A[m = r][k = 8h .. 8h+7]
//   B operand (K x N): lane holds B[k = 8h .. 8h+7][n = r]
//   C/D (M x N), 16 fp32: register v holds C[m = 8*(v/4) + 4h + v%4][n = r]
// The contraction index k may be permuted freely as long as A and B use the same permutation.
// An accumulator tile whose M index is the next contraction index can therefore be fed back as
// an operand after a bf16 pack: registers 8c .. 8c+7 of lane (r, h) hold the eight M rows
//   16c + 8t + 4h + j   (t = 0,1; j = 0..3)
// of column r, and the other operand only has to be read in that same row order.
//
// LDS tiles are row-major [rows][D] bf16 with a row pitch of 2*D + 16 bytes (a multiple of 16 B
// that is an odd number of 16 B units, so 16 lanes reading 16 B from 16 different rows hit 64
// different banks).  Rows are stored permuted inside each group of 16: tile row 16c + 4a + b sits
// at LDS row 16c + 4b + a.  With that, the four rows a transposing read needs per 16-lane group
// (tile rows 8t+4h+0..3) are four LDS rows 4 apart, i.e. 16 banks apart: conflict free.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#ifndef BURST_MFMA_PRIO
#define BURST_MFMA_PRIO 2
#endif

namespace burst {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

enum TileClass : int { TILE_SKIP = 0, TILE_FULL = 1, TILE_PARTIAL = 2 };

// Device copy of the visibility description; positions fit in int32 (checked on the host).
// Each axis (query rows, key rows) is a chunk of nseg pieces of seg_len rows; piece s starts at position
// pos0 + s * period and its rows are pos_stride apart.  The pieces are in increasing position order and do
// not overlap (period > (seg_len - 1) * pos_stride, checked on the host), so the position is a strictly
// increasing function of the local row: every "rows whose position is below x" set is a prefix of the chunk,
// and everything the tile logic needs follows from counting such prefixes (rows_lt).
struct MaskDev {
  int32_t causal;
  int32_t q_nseg, k_nseg;
  int32_t q_seg_len, k_seg_len;
  int32_t q_pos0, k_pos0;
  int32_t q_period, k_period;   // 0 with a single piece
  int32_t pos_stride;
  int32_t window;   // causal only: pos(q) - pos(k) < window as well; kNoWindow = unlimited
  // Block-wise sparse mask over local rows (nullptr: none): byte [q_row / blk_q][k_row / blk_k],
  // row pitch blk_pitch bytes, nonzero = the block pair is open.  blk_q is a multiple of 256 and
  // blk_k of 128 (checked on the host), so every tile of every kernel lies inside one block pair.
  const uint8_t* blk;
  int32_t blk_q, blk_k, blk_pitch;
};
constexpr int kMaxBlockCacheTiles = 4096;   // tiles of the walked axis whose open flags fit the LDS cache

// Open flags of the tiles of one axis against a fixed block of the other, cached in LDS once per
// work-group: flags[t] for tile t of TILE rows.  fixed_row: any row of the fixed block.
template <bool WALK_KEYS, int TILE>
__device__ __forceinline__ void fill_open_flags(const MaskDev& mk, uint8_t* flags, int fixed_row, int rows, int tid, int nthreads) {
  const int n = (rows + TILE - 1) / TILE;
  for (int t = tid; t < n; t += nthreads) {
    const int q_blk = WALK_KEYS ? fixed_row / mk.blk_q : (t * TILE) / mk.blk_q;
    const int k_blk = WALK_KEYS ? (t * TILE) / mk.blk_k : fixed_row / mk.blk_k;
    flags[t] = mk.blk[(int64_t)q_blk * mk.blk_pitch + k_blk];
  }
}
constexpr int32_t kNoWindow = 0x7fffffff;   // no position difference reaches it (positions < 2^31 - 1)

// A [batch, seq, heads, D] tensor; strides in elements.
struct TensorDev {
  void* ptr;
  int64_t sb, ss, sh;
  int32_t is_f32;
};
struct RowvecDev {
  float* ptr;
  int64_t sb, sh;
};

// One axis of the mask.
struct AxisMap {
  int32_t nseg, seg_len, pos0, period, stride;
};
template <bool Q_AXIS>
__host__ __device__ __forceinline__ AxisMap axis_of(const MaskDev& mk) {
  return Q_AXIS ? AxisMap{mk.q_nseg, mk.q_seg_len, mk.q_pos0, mk.q_period, mk.pos_stride}
                : AxisMap{mk.k_nseg, mk.k_seg_len, mk.k_pos0, mk.k_period, mk.pos_stride};
}

// Position of local row `row` (rows past the end of the chunk continue the last piece).
__host__ __device__ __forceinline__ int axis_position(const AxisMap& ax, int row) {
  if (ax.nseg <= 1) return ax.pos0 + row * ax.stride;
  int s = row / ax.seg_len;
  s = s < ax.nseg - 1 ? s : ax.nseg - 1;
  return ax.pos0 + s * ax.period + (row - s * ax.seg_len) * ax.stride;
}

// Number of rows r in [0, rows) whose position is below x (x may carry a window: 64-bit).  The
// divisions run on values clipped to the chunk's position span, which fits 32 bits.
__host__ __device__ __forceinline__ int rows_lt(const AxisMap& ax, long long x, int rows) {
  const long long t = x - ax.pos0;
  if (t <= 0 || rows <= 0) return 0;
  const long long span = (long long)(ax.nseg - 1) * ax.period + (long long)(ax.seg_len - 1) * ax.stride;   // position of the last row - pos0
  if (ax.nseg <= 1) {
    if (t > (long long)(rows - 1) * ax.stride) return rows;
    return (int)(((uint32_t)t + (uint32_t)ax.stride - 1u) / (uint32_t)ax.stride);
  }
  if (t > span) return rows;
  uint32_t p = ((uint32_t)t - 1u) / (uint32_t)ax.period;          // last piece that starts below x
  p = p < (uint32_t)(ax.nseg - 1) ? p : (uint32_t)(ax.nseg - 1);
  const uint32_t rem = (uint32_t)t - p * (uint32_t)ax.period;      // > 0
  uint32_t n = (rem + (uint32_t)ax.stride - 1u) / (uint32_t)ax.stride;
  n = n < (uint32_t)ax.seg_len ? n : (uint32_t)ax.seg_len;
  const int tot = (int)(p * (uint32_t)ax.seg_len + n);
  return tot < rows ? tot : rows;
}

// min / max position over local rows [row0, row1), row1 > row0: positions grow with the row
template <bool Q_AXIS>
__host__ __device__ __forceinline__ void range_minmax(const MaskDev& mk, int row0, int row1, int& lo, int& hi) {
  const AxisMap ax = axis_of<Q_AXIS>(mk);
  lo = axis_position(ax, row0);
  hi = axis_position(ax, row1 - 1);
}

// Class of a block whose query positions span [qlo, qhi] and key positions [klo, khi] under a causal
// mask, from the bounding ranges alone (a mixed verdict is always safe).
__host__ __device__ __forceinline__ int classify_ranges(const MaskDev& mk, int qlo, int qhi, int klo, int khi, bool ragged) {
  if (qhi < klo) return TILE_SKIP;                                   // every key lies after every query
  if ((long long)qlo - khi >= mk.window) return TILE_SKIP;           // every key has left every query's window
  if (qlo >= khi && (long long)qhi - klo < mk.window && !ragged) return TILE_FULL;
  return TILE_PARTIAL;
}

// Classify the block of query rows [q0, q1) against key rows [k0, k1) (both already clipped to the
// chunk).  PARTIAL = needs the per-element predicate: the mask edge crosses the block, or the caller
// says so because the register tile also covers rows beyond the end of a chunk.
__host__ __device__ __forceinline__ int classify(const MaskDev& mk, int q0, int q1, int k0, int k1, bool ragged) {
  if (k1 <= k0 || q1 <= q0) return TILE_SKIP;
  if (!mk.causal) return ragged ? TILE_PARTIAL : TILE_FULL;
  int qlo, qhi, klo, khi;
  range_minmax<true>(mk, q0, q1, qlo, qhi);
  range_minmax<false>(mk, k0, k1, klo, khi);
  return classify_ranges(mk, qlo, qhi, klo, khi, ragged);
}

// Row intervals of one axis against ONE fixed position range [olo, ohi] of the other axis: the rows
// that see / are seen by SOME row of the other side are [some_lo, some_hi), those that see / are seen
// by ALL of them [all_lo, all_hi) (possibly empty).  Positions grow with the row, so each set is one
// interval of rows, whatever the number of pieces.
struct RowIntervals {
  int32_t some_lo, some_hi, all_lo, all_hi;
};
template <bool Q_AXIS>
__host__ __device__ __forceinline__ RowIntervals row_intervals(const MaskDev& mk, int olo, int ohi, int rows, bool other_empty) {
  RowIntervals iv{0, 0, 0, 0};
  if (other_empty || rows <= 0) return iv;   // nothing on the other side: every block is empty
  if (!mk.causal) {
    iv.some_hi = iv.all_hi = rows;
    return iv;
  }
  const AxisMap ax = axis_of<Q_AXIS>(mk);
  const long long w = mk.window;
  if (Q_AXIS) {
    // query position p sees key position k iff k <= p < k + window; keys span [olo, ohi]
    iv.some_lo = rows_lt(ax, olo, rows);                    // first p >= olo
    iv.some_hi = rows_lt(ax, (long long)ohi + w, rows);     // first p >= ohi + window
    iv.all_lo = rows_lt(ax, ohi, rows);                     // first p >= ohi
    iv.all_hi = rows_lt(ax, (long long)olo + w, rows);      // first p >= olo + window
  } else {
    // key position k is seen from query position p iff p - window < k <= p; queries span [olo, ohi]
    iv.some_lo = rows_lt(ax, (long long)olo - w + 1, rows);   // first k > olo - window
    iv.some_hi = rows_lt(ax, (long long)ohi + 1, rows);       // end of k <= ohi
    iv.all_lo = rows_lt(ax, (long long)ohi - w + 1, rows);    // first k > ohi - window
    iv.all_hi = rows_lt(ax, (long long)olo + 1, rows);        // end of k <= olo
  }
  return iv;
}

// The same decisions as classify() for many row blocks of one axis against one fixed position range
// of the other axis, from the row intervals computed once.
template <bool Q_AXIS>
struct BlockClassifier {
  RowIntervals iv;   // (scalar members: the thresholds must stay in registers)

  __host__ __device__ __forceinline__ void init(const MaskDev& mk, int olo, int ohi, int rows, bool other_empty) {
    iv = row_intervals<Q_AXIS>(mk, olo, ohi, rows, other_empty);
  }
  // block of rows [r0, r1), r1 > r0, both inside the chunk
  __host__ __device__ __forceinline__ int operator()(const MaskDev&, int r0, int r1, bool ragged) const {
    // bitwise logic and selects only: this runs once per tile in every wave, and short-circuit
    // operators compile to a chain of scalar branches
    const bool skip = (r1 <= iv.some_lo) | (r0 >= iv.some_hi);
    const bool full = (r0 >= iv.all_lo) & (r1 <= iv.all_hi) & !ragged;
    const int cls = full ? TILE_FULL : TILE_PARTIAL;
    return skip ? TILE_SKIP : cls;
  }
};

// Per-element mask of one 32x32 accumulator tile whose 16 registers of a lane run over rows
// base_row + 4*h + 8*(v/4) + (v%4) of the OTHER side than the lane's own row (base_row: first of the 32
// rows, wave-uniform): KEYS_IN_REGS = true, registers are key rows and the lane owns a query (position
// lane_pos); false, registers are query rows and the lane owns a key.  Invisible entries and rows
// >= n_rows become -inf.  The 32 rows lie in at most two consecutive pieces (a piece has at least 32
// rows whenever there are more than two, checked on the host).  Written with selects only, no
// divergent control flow.
template <bool KEYS_IN_REGS>
__device__ __forceinline__ void mask_tile(f32x16& s, const MaskDev& mk, int base_row, int h, int n_rows, int lane_pos) {
  const AxisMap ax = axis_of<!KEYS_IN_REGS>(mk);
  int split = 0x7fffffff, pos_a = ax.pos0, pos_b = ax.pos0;   // position = pos_a (rows < split) or pos_b, + row * stride
  if (ax.nseg > 1) {
    int s0 = base_row / ax.seg_len;
    s0 = s0 < ax.nseg - 1 ? s0 : ax.nseg - 1;
    pos_a = ax.pos0 + s0 * (ax.period - ax.seg_len * ax.stride);
    pos_b = pos_a + ax.period - ax.seg_len * ax.stride;
    split = s0 < ax.nseg - 1 ? (s0 + 1) * ax.seg_len : 0x7fffffff;
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int row = base_row + 4 * h + 8 * (v >> 2) + (v & 3);
    const int pos = (row >= split ? pos_b : pos_a) + row * ax.stride;
    const int diff = KEYS_IN_REGS ? lane_pos - pos : pos - lane_pos;   // pos(q) - pos(k)
    const bool ordered = (diff >= 0) & (diff < mk.window);
    const bool vis = (row < n_rows) & ((mk.causal == 0) | ordered);
    s[v] = vis ? s[v] : -INFINITY;
  }
}

__device__ __forceinline__ int lds_row(int tile_row) {
  // tile row 16c + 4a + b  ->  LDS row 16c + 4b + a
  return (tile_row & ~15) | ((tile_row & 3) << 2) | ((tile_row >> 2) & 3);
}
// Variant for tiles whose rows are the contraction index of a GEMM whose other operand is read
// row-wise: tile row 16c + 8h + 4t + j -> LDS row 16c + 4j + 2t + h, so that the column-wise operand
// read hands half-wave h the rows 16c + 8h .. 8h+7 in order, the same eight k that lds_rows_operand
// hands it (with lds_row it would be rows 4h..4h+3 and 8+4h..8+4h+3, the accumulator order).
__device__ __forceinline__ int lds_row_k8(int tile_row) {
  return (tile_row & ~15) | ((tile_row & 3) << 2) | (((tile_row >> 2) & 1) << 1) | ((tile_row >> 3) & 1);
}

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Operand with lane = tile row, eight consecutive columns: rows row_base + r (r = lane % 32),
// columns col0 + 8h .. +7 (bf16 elements).
template <int PITCH>
__device__ __forceinline__ bf16x8 lds_rows_operand(const char* tile, int row_base, int col0, int r, int h) {
  const char* p = tile + lds_row(row_base + r) * PITCH + (col0 + 8 * h) * 2;
  return *reinterpret_cast<const bf16x8*>(p);
}

// Operand with lane = tile column, eight rows: column col_base + r, rows
// row16 + 8t + 4h + j (t = 0,1; j = 0..3) of a 16-row group starting at tile row row16
// (a multiple of 16).  Element order 4t + j, matching packed accumulator registers.
template <int PITCH>
__device__ __forceinline__ bf16x8 lds_cols_operand(const char* tile, int row16, int col_base, int lane) {
  typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
  const int i16 = lane & 15, g2 = (lane >> 4) & 1, h = lane >> 5;
  // LDS row of tile row 8t+4h+j is 4j + 2t + h; lanes 4j .. 4j+3 of a 16-lane group supply row j
  const int j = i16 >> 2;
  const char* p = tile + (row16 + 4 * j + h) * PITCH + (col_base + 16 * g2 + 4 * (i16 & 3)) * 2;
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 2 * PITCH));
  typedef __attribute__((ext_vector_type(8))) short s16x8;
  s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, both);
}

// Wait for every outstanding global load of this wave.  Used once, before a tile loop, after the
// loop-invariant register operands were fetched: without it the compiler cannot prove on every
// path that they have landed and re-inserts vmcnt waits inside the loop, which then also wait for
// the tile prefetch issued just before them.
__device__ __forceinline__ void wait_global_loads() { __builtin_amdgcn_s_waitcnt(0x0F70); }   // vmcnt(0)

__device__ __forceinline__ float half_swap(float x) {
  // value held by the lane 32 away
  return __shfl_xor(x, 32, 64);
}

// The tiles of an axis that have any visible pair against the WHOLE other chunk, as up to two runs of
// consecutive tile indices (found by the host; with more runs every tile is launched).  Only these are
// launched: an empty work-group costs a dispatch slot, and many of them in a row starve the other CUs.
struct TileRuns {
  int32_t start[2], len[2];
  __host__ __device__ int total() const { return len[0] + len[1]; }
  __host__ __device__ int tile_of(int i) const { return i < len[0] ? start[0] + i : start[1] + (i - len[0]); }
};

// Tiles of TILE rows along the query axis (Q_AXIS) or the key axis that can hold a pair visible to
// the other side, whose positions span [olo, ohi]: the rows that see / are seen by some row of the other
// side are one interval of rows (row_intervals), hence one run of consecutive tiles.  A tile in the run
// may still turn out empty for a narrower row range; a tile outside it never holds a visible pair.
struct TileRun {
  int32_t start, len;
};
template <bool Q_AXIS, int TILE>
__host__ __device__ __forceinline__ TileRun visible_tiles(const MaskDev& mk, int olo, int ohi, int rows) {
  const RowIntervals iv = row_intervals<Q_AXIS>(mk, olo, ohi, rows, false);
  if (iv.some_lo >= iv.some_hi) return TileRun{0, 0};
  const int first = iv.some_lo / TILE;
  return TileRun{first, (iv.some_hi + TILE - 1) / TILE - first};
}

// Stage a [ROWS x D] bf16 tile: global (row-major, row stride `ss` elements) -> registers -> LDS,
// by THREADS threads.  Split in two so the loads can be issued before the compute they overlap
// with.  The per-lane part of the address is one 32-bit element offset computed once; the
// per-tile and per-pass parts are wave-uniform, so a load costs no vector arithmetic.  Tiles that
// reach past the last row take a slower path that clamps row indices instead.
template <int D, int ROWS, int THREADS = 256, bool K8 = false>   // K8: rows permuted by lds_row_k8
struct TileStager {
  static constexpr int CPR = D / 8;              // 16-byte chunks per row
  static constexpr int RPP = THREADS / CPR;      // rows per pass
  static constexpr int PASSES = ROWS / RPP;
  static constexpr int PITCH = 2 * D + 16;
  static_assert(ROWS % RPP == 0, "tile rows must be a multiple of rows per pass");
  u32x4 regs[PASSES];
  uint32_t lane_off;    // (tid / CPR) * ss + (tid % CPR) * 8, elements
  uint32_t lds_off[PASSES];
  uint32_t src_off[PASSES];   // byte offset of this thread's chunk of pass i from the tile's first row

  // valid_rows < ROWS: load_at() reads the tile's rows beyond valid_rows - 1 as copies of that row,
  // for tiles that reach past the end of a matrix whose extra rows must only be finite.
  __device__ __forceinline__ void init(int64_t ss, int tid, int valid_rows = ROWS) {
    lane_off = (uint32_t)(tid / CPR) * (uint32_t)ss + (uint32_t)(tid % CPR) * 8u;
#pragma unroll
    for (int i = 0; i < PASSES; ++i) {
      lds_off[i] = (K8 ? lds_row_k8(tid / CPR + i * RPP) : lds_row(tid / CPR + i * RPP)) * PITCH + (tid % CPR) * 16;
      src_off[i] = 2u * ((uint32_t)min(tid / CPR + i * RPP, valid_rows - 1) * (uint32_t)ss + (uint32_t)(tid % CPR) * 8u);
    }
  }
  __device__ __forceinline__ void load_pass(const char* tile, int i) { regs[i] = *reinterpret_cast<const u32x4*>(tile + src_off[i]); }
  __device__ __forceinline__ void store_pass(char* tile, int i) const { *reinterpret_cast<u32x4*>(tile + lds_off[i]) = regs[i]; }
  // A tile that lies wholly inside the tensor, given the (wave-uniform) address of its first row:
  // uniform base plus a precomputed 32-bit lane offset, no address arithmetic per load.
  __device__ __forceinline__ void load_at(const char* tile) {
#pragma unroll
    for (int i = 0; i < PASSES; ++i) regs[i] = *reinterpret_cast<const u32x4*>(tile + src_off[i]);
  }
  // base: first row of the tensor slice; row0: first tile row; nrows: rows in the slice (> row0)
  __device__ __forceinline__ void load(const __bf16* base, int64_t ss, int row0, int nrows, int tid) {
    if (row0 + ROWS <= nrows) {
      const __bf16* tile = base + (int64_t)row0 * ss;    // uniform
#pragma unroll
      for (int i = 0; i < PASSES; ++i)
        regs[i] = *reinterpret_cast<const u32x4*>(tile + (int64_t)i * RPP * ss + lane_off);
    } else {
      const int c = tid % CPR, rr = tid / CPR;
#pragma unroll
      for (int i = 0; i < PASSES; ++i) {
        int row = min(row0 + rr + i * RPP, nrows - 1);
        regs[i] = *reinterpret_cast<const u32x4*>(base + (int64_t)row * ss + c * 8);
      }
    }
  }
  __device__ __forceinline__ void store(char* tile) const {
#pragma unroll
    for (int i = 0; i < PASSES; ++i) *reinterpret_cast<u32x4*>(tile + lds_off[i]) = regs[i];
  }
};

// Walk of a query block over the key tiles (BK rows of K and of V) it can see, with the staging
// of the tiles.  The visible tiles are one run of consecutive tiles, so the cursor and the two tile
// addresses move by adding constants and a load needs no address arithmetic.
template <int D, int BK, int NT>
struct KvWalk {
  TileStager<D, BK, NT> stage_k, stage_v;
  int left, k0;           // cursor: tiles left in the run (0: the walk is over), first key row of its tile
  int sk;
  const uint8_t* open;    // LDS flags per key tile from a block-wise sparse mask, or nullptr
  const char *k_base, *v_base, *k_tile, *v_tile;   // row 0 of the head; first row of the cursor's tile
  int64_t k_row, v_row;   // bytes per key row

  // [q_lo, q_hi]: positions spanned by the query rows of the work-group.  The cursor starts on the
  // first tile to visit.
  __device__ __forceinline__ void init(const MaskDev& mk, const TensorDev& k, const TensorDev& v, int b, int hk, int sk_,
                                       int q_lo, int q_hi, int tid, const uint8_t* open_flags) {
    sk = sk_;
    open = open_flags;
    const TileRun run = visible_tiles<false, BK>(mk, q_lo, q_hi, sk);
    left = run.len;
    k0 = run.start * BK;
    k_row = k.ss * 2;
    v_row = v.ss * 2;
    k_base = reinterpret_cast<const char*>((const __bf16*)k.ptr + b * k.sb + hk * k.sh);
    v_base = reinterpret_cast<const char*>((const __bf16*)v.ptr + b * v.sb + hk * v.sh);
    k_tile = k_base + k0 * k_row;
    v_tile = v_base + k0 * v_row;
    stage_k.init(k.ss, tid);
    stage_v.init(v.ss, tid);
    seek();
  }
  __device__ __forceinline__ bool valid() const { return left > 0; }
  __device__ __forceinline__ void issue(int tid) {   // loads of the cursor's tile
    if (k0 + BK <= sk) {
      stage_k.load_at(k_tile);
      stage_v.load_at(v_tile);
    } else {   // last tile of a ragged chunk: row indices clamped per thread
      stage_k.load(reinterpret_cast<const __bf16*>(k_base), k_row >> 1, k0, sk, tid);
      stage_v.load(reinterpret_cast<const __bf16*>(v_base), v_row >> 1, k0, sk, tid);
    }
  }
  __device__ __forceinline__ void step() {
    --left;
    k0 += BK;
    k_tile += BK * k_row;
    v_tile += BK * v_row;
  }
  // skip tiles that the block mask closes
  __device__ __forceinline__ void seek() {
    if (open) {
      while (left > 0 && __builtin_amdgcn_readfirstlane(open[k0 / BK]) == 0) step();
    }
  }
  __device__ __forceinline__ void advance() {
    step();
    seek();
  }
  __device__ __forceinline__ void commit(char* k_lds, char* v_lds) const {
    stage_k.store(k_lds);
    stage_v.store(v_lds);
  }
};

// Scope of a stream of MFMAs: the wave runs at raised issue priority.  A SIMD issues one vector-class
// instruction at a time and picks the oldest ready wave; without this, a co-resident wave in a
// dense vector phase (softmax, dS) keeps winning the issue slot and the matrix pipe idles, although
// an MFMA needs only one slot in eight.
struct MatrixPhase {
  __device__ __forceinline__ MatrixPhase() { __builtin_amdgcn_s_setprio(BURST_MFMA_PRIO); }
  __device__ __forceinline__ ~MatrixPhase() { __builtin_amdgcn_s_setprio(0); }
};

struct NoHook {
  __device__ __forceinline__ void operator()(int) const {}
};

// acc[nb] (+)= A_nb * B for NB row blocks of an LDS tile: A_nb = tile rows row0 + 32*nb .. +31 (all D
// columns, read row-wise), B = DK register operands.  The k-step is the outer loop so consecutive
// MFMAs hit different accumulators, and LDS operands are fetched PRE k-steps ahead of their use;
// the scheduling fences keep the compiler from hoisting more (registers) or less (latency).
// ZERO: the accumulators start from 0 (first MFMA takes the constant, no register clearing).
// hook(ks) runs after the MFMAs of k-step ks, inside the same scheduling region: independent
// vector work placed there issues while the matrix pipe is busy.
template <int PITCH, int NB, int DK, int PRE, bool ZERO = false, class Hook = NoHook>
__device__ __forceinline__ void gemm_rows(const char* tile, int row0, const bf16x8 (&breg)[DK], f32x16 (&acc)[NB],
                                          int r, int h, Hook&& hook = Hook()) {
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  bf16x8 a[DK][NB];
  MatrixPhase prio;
#pragma unroll
  for (int ks = 0; ks < PRE && ks < DK; ++ks)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) a[ks][nb] = lds_rows_operand<PITCH>(tile, row0 + 32 * nb, ks * 16, r, h);
#pragma unroll
  for (int ks = 0; ks < DK; ++ks) {
    if (ks + PRE < DK) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
        a[ks + PRE][nb] = lds_rows_operand<PITCH>(tile, row0 + 32 * nb, (ks + PRE) * 16, r, h);
    }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[nb] = mfma32(a[ks][nb], breg[ks], (ZERO && ks == 0) ? zero : acc[nb]);
    hook(ks);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// Two row-wise GEMMs sharing the row block, interleaved so consecutive MFMAs alternate between the
// two accumulators:  acc0 += rows(tile0) * b0,  acc1 += rows(tile1) * b1.
template <int PITCH, int DK, int PRE, bool ZERO0 = false>   // ZERO0: acc0 starts from zero (not read)
__device__ __forceinline__ void gemm_rows_pair(const char* tile0, const char* tile1, int row0, const bf16x8 (&b0)[DK],
                                               const bf16x8 (&b1)[DK], f32x16& acc0, f32x16& acc1, int r, int h) {
  bf16x8 a0[DK], a1[DK];
  MatrixPhase prio;
#pragma unroll
  for (int ks = 0; ks < PRE && ks < DK; ++ks) {
    a0[ks] = lds_rows_operand<PITCH>(tile0, row0, ks * 16, r, h);
    a1[ks] = lds_rows_operand<PITCH>(tile1, row0, ks * 16, r, h);
  }
#pragma unroll
  for (int ks = 0; ks < DK; ++ks) {
    if (ks + PRE < DK) {
      a0[ks + PRE] = lds_rows_operand<PITCH>(tile0, row0, (ks + PRE) * 16, r, h);
      a1[ks + PRE] = lds_rows_operand<PITCH>(tile1, row0, (ks + PRE) * 16, r, h);
    }
    acc0 = mfma32(a0[ks], b0[ks], (ZERO0 && ks == 0) ? f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f} : acc0);
    acc1 = mfma32(a1[ks], b1[ks], acc1);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// acc[db] += A_db,c * b[c]: A = LDS tile read column-wise (columns 32*db .. +31, rows
// row0 + 16*c .. +15 in packed-accumulator order), b[c] = packed register operands, c < NC.
// One step = one 16-row chunk across all DB accumulators; operands fetched PRE steps ahead.
template <int PITCH, int DB, int NC, int PRE, class Hook = NoHook>
__device__ __forceinline__ void gemm_cols(const char* tile, int row0, const bf16x8 (&b)[NC], f32x16 (&acc)[DB],
                                          int lane, Hook&& hook = Hook()) {
  // operands in use order: i = c * DB + db; fetched AHEAD operands before use
  constexpr int N = NC * DB, AHEAD = PRE;   // PRE counts operands here
  bf16x8 a[N];
  MatrixPhase prio;
#pragma unroll
  for (int i = 0; i < AHEAD && i < N; ++i) a[i] = lds_cols_operand<PITCH>(tile, row0 + 16 * (i / DB), (i % DB) * 32, lane);
#pragma unroll
  for (int i = 0; i < N; ++i) {
    if (i + AHEAD < N)
      a[i + AHEAD] = lds_cols_operand<PITCH>(tile, row0 + 16 * ((i + AHEAD) / DB), ((i + AHEAD) % DB) * 32, lane);
    acc[i % DB] = mfma32(a[i], b[i / DB], acc[i % DB]);
    if (i % DB == DB - 1) hook(i / DB);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// The same product with its first PRE operands fetched by the caller ahead of time (gemm_cols_fetch),
// e.g. before a stretch of vector work, so that the first MFMA does not wait for LDS.
template <int PITCH, int DB, int PRE>
__device__ __forceinline__ void gemm_cols_fetch(const char* tile, int row0, int lane, bf16x8 (&first)[PRE]) {
#pragma unroll
  for (int i = 0; i < PRE; ++i) first[i] = lds_cols_operand<PITCH>(tile, row0 + 16 * (i / DB), (i % DB) * 32, lane);
}
template <int PITCH, int DB, int NC, int PRE, class Hook = NoHook>
__device__ __forceinline__ void gemm_cols_run(const char* tile, int row0, const bf16x8 (&b)[NC], f32x16 (&acc)[DB],
                                              int lane, const bf16x8 (&first)[PRE], Hook&& hook = Hook()) {
  constexpr int N = NC * DB;
  static_assert(PRE <= N, "more operands fetched ahead than the product has");
  bf16x8 a[N];
  MatrixPhase prio;
#pragma unroll
  for (int i = 0; i < PRE; ++i) a[i] = first[i];
#pragma unroll
  for (int i = 0; i < N; ++i) {
    if (i + PRE < N)
      a[i + PRE] = lds_cols_operand<PITCH>(tile, row0 + 16 * ((i + PRE) / DB), ((i + PRE) % DB) * 32, lane);
    acc[i % DB] = mfma32(a[i], b[i / DB], acc[i % DB]);
    if (i % DB == DB - 1) hook(i / DB);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// Streams with one hook per MFMA, for software-pipelined kernels: hook(i) holds the few vector or LDS
// instructions of ANOTHER unit of work that go behind MFMA i, and the scheduling fence after it keeps them
// there, so that a wave's vector work runs in the shadow of matrix work that does not depend on it.
//   acc (+)= rows(tile)[row0 .. row0+31] * b   (ZERO: starts from a literal zero)
template <int PITCH, int DK, int PRE, bool ZERO, class Hook = NoHook>
__device__ __forceinline__ void rows_stream(const char* tile, int row0, const bf16x8 (&b)[DK], f32x16& acc, int r, int h,
                                            Hook&& hook = Hook()) {
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  bf16x8 a[DK];
#pragma unroll
  for (int ks = 0; ks < PRE && ks < DK; ++ks) a[ks] = lds_rows_operand<PITCH>(tile, row0, ks * 16, r, h);
#pragma unroll
  for (int ks = 0; ks < DK; ++ks) {
    if (ks + PRE < DK) a[ks + PRE] = lds_rows_operand<PITCH>(tile, row0, (ks + PRE) * 16, r, h);
    acc = mfma32(a[ks], b[ks], (ZERO && ks == 0) ? zero : acc);
    hook(ks);
    __builtin_amdgcn_sched_barrier(0);
  }
}
//   acc[db] += cols(tile)[db, c] * b[c]  (as gemm_cols), hook(i) behind MFMA i = c * DB + db; b is read when
//   its MFMA is issued, so a hook may still complete b[c] for a later chunk c.
template <int PITCH, int DB, int NC, int PRE, class Hook = NoHook>
__device__ __forceinline__ void cols_stream(const char* tile, int row0, const bf16x8 (&b)[NC], f32x16 (&acc)[DB], int lane,
                                            Hook&& hook = Hook()) {
  constexpr int N = NC * DB;
  bf16x8 a[N];
#pragma unroll
  for (int i = 0; i < PRE && i < N; ++i) a[i] = lds_cols_operand<PITCH>(tile, row0 + 16 * (i / DB), (i % DB) * 32, lane);
#pragma unroll
  for (int i = 0; i < N; ++i) {
    if (i + PRE < N) a[i + PRE] = lds_cols_operand<PITCH>(tile, row0 + 16 * ((i + PRE) / DB), ((i + PRE) % DB) * 32, lane);
    acc[i % DB] = mfma32(a[i], b[i / DB], acc[i % DB]);
    hook(i);
    __builtin_amdgcn_sched_barrier(0);
  }
}

__device__ __forceinline__ bf16x8 pack8(const f32x16& x, int c) {
  bf16x8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = (__bf16)x[8 * c + e];
  return o;
}

// Work-group index -> (kv key = batch*Hkv + kv head, head within group, q tile), such that all work
// on one (batch, kv head) lands on one XCD (work-groups are dealt round-robin to the 8 XCDs, each
// with its own L2) and heavier tiles start first.  Under a causal mask a query tile is heavier the
// higher its rows (HIGH_FIRST), a key tile the lower its rows.  Heavy-first is also what keeps the
// work-groups that share an L2 in step: the ones running together then walk the other axis at the
// same place at the same time, so each tile of it is fetched from HBM once.
struct BlockMap {
  int key, head_in_group, tile;
  bool valid;
};
template <bool HIGH_FIRST>
__device__ __forceinline__ BlockMap map_block(int n, int n_keys, int group, int tiles) {
  const int xcd = n & 7, slot = n >> 3;
  const int per_key = group * tiles;
  BlockMap m;
  int local_key = slot / per_key, rem = slot - local_key * per_key;
  m.key = local_key * 8 + xcd;
  m.head_in_group = rem / tiles;
  const int t = rem - m.head_in_group * tiles;
  m.tile = HIGH_FIRST ? tiles - 1 - t : t;
  m.valid = m.key < n_keys;
  return m;
}
inline int mapped_grid(int n_keys, int group, int tiles) { return 8 * ((n_keys + 7) / 8) * group * tiles; }

}  // namespace burst
