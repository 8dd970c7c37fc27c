// Forward step kernel: O_ij, Lse_cur of a query chunk against one key/value chunk (Eq. 5-6),
// optionally folded into the running (O_i, Lse_i) in the epilogue (forward algorithm).
//
// One work-group = 8 waves = 256 query rows of one (batch, head); wave w owns rows [32w, 32w+32),
// two waves per SIMD.  The key/value chunk streams through LDS in tiles of 64 rows, double buffered,
// one barrier per tile.  Everything is computed transposed so that a lane always owns one query row:
//   S^T = K Q^T   (A = K rows from LDS, B = Q held in registers),
//   P^T = exp2(..) in the accumulator registers, packed to bf16 and fed straight back as the
//   B operand of  O^T = V^T P^T  (A = V columns via transposing LDS reads).
// Row max / row sum / rescale are then per-lane scalars; the two half-waves exchange one value
// per tile.
#include "common.hpp"
#include "kernels.hpp"

namespace burst {

#ifndef BURST_FWD_BQ
#define BURST_FWD_BQ 256
#endif
constexpr int kFwdBQ = BURST_FWD_BQ;   // query rows per work-group: 32 per wave

template <int D, int NW>
__global__ __launch_bounds__(64 * NW, 512 / (64 * NW)) void step_fwd_kernel(FwdParams p) {
  constexpr int BK = 64, KB = BK / 32, DK = D / 16, DB = D / 32, BQ = 32 * NW, NT = 64 * NW;
  constexpr int PITCH = 2 * D + 16;
  constexpr int TILE = BK * PITCH;
  extern __shared__ __attribute__((aligned(16))) char smem[];  // [2 buffers][K tile, V tile]

  const int group = p.q_heads / p.kv_heads;
  const BlockMap bm = map_block<true>(blockIdx.x, p.batch * p.kv_heads, group, p.q_runs.total());
  if (!bm.valid) return;
  const int b = bm.key / p.kv_heads, hk = bm.key - b * p.kv_heads, hq = hk * group + bm.head_in_group;

  const int tid = threadIdx.x, lane = tid & 63, r = lane & 31, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: everything derived from it stays wave-uniform
  const int sq = p.sq, sk = p.sk;
  const MaskDev mk = p.mask;
  const int q_blk0 = p.q_runs.tile_of(bm.tile) * BQ;     // first row of the work-group
  const int q_blk1 = min(q_blk0 + BQ, sq);
  const int q_w0 = q_blk0 + wave * 32;                   // first row of the wave
  const int q_w1 = min(q_w0 + 32, sq);                   // may be <= q_w0: the wave only helps staging

  // Q as the B operand of S^T = K Q^T: lane holds Q[row][16*ks + 8h .. +7]
  bf16x8 qreg[DK];
  const int row = min(q_w0 + r, sq - 1);
  const int qpos = axis_position(axis_of<true>(mk), row);
  {
    const __bf16* src = (const __bf16*)p.q.ptr + b * p.q.sb + hq * p.q.sh + (int64_t)row * p.q.ss + 8 * h;
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8*>(src + ks * 16);
  }

  f32x16 o[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float c = p.scale * kLog2e;

  // Key tiles the work-group can see, and the class of each against this wave's 32 query rows
  int qlo_blk, qhi_blk, qlo_w = 0, qhi_w = 0;
  range_minmax<true>(mk, q_blk0, q_blk1, qlo_blk, qhi_blk);
  if (q_w0 < q_w1) range_minmax<true>(mk, q_w0, q_w1, qlo_w, qhi_w);
  BlockClassifier<false> k_class;
  k_class.init(mk, qlo_w, qhi_w, sk, q_w0 >= q_w1);
  auto tile_class = [&](int k0_) { return k_class(mk, k0_, min(k0_ + BK, sk), k0_ + BK > sk); };   // wave-uniform

  // Open flags of the key tiles against this work-group's query block (block-wise sparse mask)
  uint8_t* open_flags = nullptr;
  if (mk.blk) {
    open_flags = reinterpret_cast<uint8_t*>(smem + 4 * TILE);
    fill_open_flags<true, BK>(mk, open_flags, q_blk0, sk, tid, NT);
    __syncthreads();
  }
  KvWalk<D, BK, NT> walk;
  walk.init(mk, p.k, p.v, b, hk, sk, qlo_blk, qhi_blk, tid, open_flags);
  wait_global_loads();
  int k0 = 0, cls = TILE_SKIP;   // first key row and class of the tile in LDS
  bool have = walk.valid();
  if (have) {
    walk.issue(tid);
    walk.commit(smem, smem + TILE);
    k0 = walk.k0;
    cls = tile_class(k0);
    walk.advance();
  }
  __syncthreads();
  int buf = 0;
  while (have) {
    const bool more = walk.valid();
    int k0n = 0, cls_n = TILE_SKIP;
    if (more) {
      walk.issue(tid);
      k0n = walk.k0;
      cls_n = tile_class(k0n);
      walk.advance();
    }
    const char* kt = smem + buf * 2 * TILE;
    const char* vt = kt + TILE;
    if (cls != TILE_SKIP) {
      f32x16 s[KB];
      gemm_rows<PITCH, KB, DK, kRowsAhead, true>(kt, 0, qreg, s, r, h);
      // the first V operands of the PV product are fetched now, ahead of the softmax arithmetic
      bf16x8 v_first[kColsAhead];
      gemm_cols_fetch<PITCH, DB, kColsAhead>(vt, 0, lane, v_first);
      __builtin_amdgcn_sched_barrier(0);
      if (cls == TILE_PARTIAL) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) mask_tile<true>(s[kb], mk, k0 + kb * 32, h, sk, qpos);
      }
      // largest score among this lane's keys of the tile (the row's other keys sit in the lane 32 away):
      // four short chains instead of one long one
      float mx4[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) mx4[j] = fmaxf(s[0][j], s[0][j + 4]);
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int v = (kb == 0 ? 8 : 0); v < 16; ++v) mx4[v & 3] = fmaxf(mx4[v & 3], s[kb][v]);
      const float mx_own = fmaxf(fmaxf(mx4[0], mx4[1]), fmaxf(mx4[2], mx4[3]));
      // Rescale lazily: keep a stale maximum while no row of the wave has grown by more than
      // 2^kLazyLog2 (any common per-row offset gives the same result; fp32 has the headroom).  A row has
      // grown exactly if one of its two lanes has, and the vote runs over the whole wave, so the two halves
      // of a row exchange their maxima only when a rescale happens: the steady state has no cross-lane
      // traffic (the exchange goes through LDS and costs a round trip the wave cannot fill).
      const bool grow = c * (mx_own - m_run) > kLazyLog2;   // false for -inf - -inf
      if (__any(grow)) {
        const float m_new = fmaxf(m_run, fmaxf(mx_own, half_swap(mx_own)));
        const float alpha = (m_new == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f(c * (m_run - m_new));
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int v = 0; v < 16; ++v) o[db][v] *= alpha;
      }
      const float msub = (m_run == -INFINITY) ? 0.f : c * m_run;
      // P = exp2(c S - c m) as packed bf16 pairs; the row sum is taken in fp32 before rounding (Lse
      // must hold to 1e-3 also for rows with a handful of keys).  The exponentials of key block kb+1
      // are issued between the MFMAs of key block kb's part of the PV product.
      typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
      uint32_t ppw[KB][8];
      auto exp_pairs = [&](int kb, int w0, int nw) {
#pragma unroll
        for (int w = w0; w < w0 + nw; ++w) {
          const float e0 = __builtin_amdgcn_exp2f(c * s[kb][2 * w] - msub);
          const float e1 = __builtin_amdgcn_exp2f(c * s[kb][2 * w + 1] - msub);
          const bf16x2 pr = {(__bf16)e0, (__bf16)e1};
          ppw[kb][w] = __builtin_bit_cast(uint32_t, pr);
          l_run += e0 + e1;
        }
      };
      exp_pairs(0, 0, 8);
      static_assert(KB == 2, "the PV product below is written for two 32-key blocks per tile");
      // one operand stream over both key blocks: pp[2 kb], pp[2 kb + 1] are the two 16-key halves of block kb
      bf16x8 pp[2 * KB];
      auto pack_block = [&](int kb) {
        const u32x4 w_lo = {ppw[kb][0], ppw[kb][1], ppw[kb][2], ppw[kb][3]};
        const u32x4 w_hi = {ppw[kb][4], ppw[kb][5], ppw[kb][6], ppw[kb][7]};
        pp[2 * kb] = __builtin_bit_cast(bf16x8, w_lo);
        pp[2 * kb + 1] = __builtin_bit_cast(bf16x8, w_hi);
      };
      pack_block(0);
      pp[2] = pp[0];   // placeholders until the hooks have produced block 1
      pp[3] = pp[1];
      gemm_cols_run<PITCH, DB, 2 * KB, kColsAhead>(vt, 0, pp, o, lane, v_first, [&](int c2) {
        if (c2 < 2) exp_pairs(1, 4 * c2, 4);
        if (c2 == 1) pack_block(1);
      });
    }
    if (more) walk.commit(smem + (buf ^ 1) * 2 * TILE, smem + (buf ^ 1) * 2 * TILE + TILE);
    __syncthreads();
    buf ^= 1;
    k0 = k0n;
    cls = cls_n;
    have = more;
  }

  // Epilogue: normalise, Lse in natural-log units, optional online-softmax merge.
  const int orow = q_w0 + r;
  const float l_tot = l_run + half_swap(l_run);
  const bool alive = l_tot > 0.f;
  const float inv = alive ? 1.f / l_tot : 0.f;
  const float lse_cur = alive ? (c * m_run + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
  if (orow >= sq) return;
  if (p.o_part.ptr) {
    if (p.o_part.is_f32) {
      float* dst = (float*)p.o_part.ptr + b * p.o_part.sb + (int64_t)orow * p.o_part.ss + hq * p.o_part.sh;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          f32x4 x = {o[db][4 * g] * inv, o[db][4 * g + 1] * inv, o[db][4 * g + 2] * inv, o[db][4 * g + 3] * inv};
          *reinterpret_cast<f32x4*>(dst + db * 32 + 8 * g + 4 * h) = x;
        }
    } else {
      __bf16* dst = (__bf16*)p.o_part.ptr + b * p.o_part.sb + (int64_t)orow * p.o_part.ss + hq * p.o_part.sh;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          bf16x4 x = {(__bf16)(o[db][4 * g] * inv), (__bf16)(o[db][4 * g + 1] * inv), (__bf16)(o[db][4 * g + 2] * inv),
                      (__bf16)(o[db][4 * g + 3] * inv)};
          *reinterpret_cast<bf16x4*>(dst + db * 32 + 8 * g + 4 * h) = x;
        }
    }
    if (h == 0) p.lse_part.ptr[b * p.lse_part.sb + hq * p.lse_part.sh + orow] = lse_cur;
  }
  if (p.o_acc.ptr && alive) {   // a step that saw no key leaves the running state untouched
    float* lse_ptr = p.lse_acc.ptr + b * p.lse_acc.sb + hq * p.lse_acc.sh + orow;
    const float lse_old = *lse_ptr;
    const float mm = fmaxf(lse_old, lse_cur);   // finite: lse_cur is
    const float e_old = __expf(lse_old - mm), e_cur = __expf(lse_cur - mm);
    const float tot = e_old + e_cur;
    const float lse_new = mm + __logf(tot);
    const float w_old = e_old / tot, w_cur_n = e_cur / tot * inv;
    const bool has_old = lse_old != -INFINITY;
    float* dst = (float*)p.o_acc.ptr + b * p.o_acc.sb + (int64_t)orow * p.o_acc.ss + hq * p.o_acc.sh;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float* q4 = dst + db * 32 + 8 * g + 4 * h;
        // a running state that is still (anything, -inf) has weight zero and is not read as a number:
        // the buffer may hold whatever it was allocated with (0 * NaN would poison the row)
        f32x4 old = *reinterpret_cast<const f32x4*>(q4);
        if (!has_old) old = f32x4{0.f, 0.f, 0.f, 0.f};
        f32x4 x = {o[db][4 * g] * w_cur_n + old[0] * w_old, o[db][4 * g + 1] * w_cur_n + old[1] * w_old,
                   o[db][4 * g + 2] * w_cur_n + old[2] * w_old, o[db][4 * g + 3] * w_cur_n + old[3] * w_old};
        *reinterpret_cast<f32x4*>(q4) = x;
      }
    // both half-waves read lse_old above, in lockstep, before this store
    if (h == 0) *lse_ptr = lse_new;
  }
}

// Query rows of a step that no launched work-group covers (their tiles see no key): the step
// result for them is (0, -inf); the running state is left alone.
__global__ __launch_bounds__(256) void fwd_fill_dead_rows_kernel(FwdParams p) {
  const int d4 = p.head_dim / 4;
  const int n_tiles = (p.sq + kFwdBQ - 1) / kFwdBQ;
  const int64_t total = (int64_t)p.batch * p.sq * p.q_heads * d4;
  for (int64_t i = blockIdx.x * 256ll + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int cc = i % d4;
    int64_t rest = i / d4;
    const int hq = rest % p.q_heads;
    rest /= p.q_heads;
    const int row = rest % p.sq;
    const int b = rest / p.sq;
    const int tile = row / kFwdBQ;
    const bool covered = (tile >= p.q_runs.start[0] && tile < p.q_runs.start[0] + p.q_runs.len[0]) ||
                         (tile >= p.q_runs.start[1] && tile < p.q_runs.start[1] + p.q_runs.len[1]);
    if (covered || tile >= n_tiles) continue;
    const int64_t off = b * p.o_part.sb + (int64_t)row * p.o_part.ss + hq * p.o_part.sh + cc * 4;
    if (p.o_part.is_f32) {
      *reinterpret_cast<f32x4*>((float*)p.o_part.ptr + off) = f32x4{0.f, 0.f, 0.f, 0.f};
    } else {
      *reinterpret_cast<bf16x4*>((__bf16*)p.o_part.ptr + off) = bf16x4{(__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f};
    }
    if (cc == 0) p.lse_part.ptr[b * p.lse_part.sb + hq * p.lse_part.sh + row] = -INFINITY;
  }
}

template <int D>
static hipError_t launch_fwd_t(FwdParams p, hipStream_t stream) {
  constexpr int BQ = kFwdBQ;
  constexpr int LDS = 2 * 2 * 64 * (2 * D + 16) + kMaxBlockCacheTiles;
  p.q_runs = nonempty_runs(p.mask, p.sq, p.sk, BQ, true);
  const int n_tiles = (p.sq + BQ - 1) / BQ;
  if (p.o_part.ptr && p.q_runs.total() < n_tiles) {
    const int64_t total = (int64_t)p.batch * p.sq * p.q_heads * (p.head_dim / 4);
    const int64_t blocks = (total + 255) / 256;
    hipLaunchKernelGGL(fwd_fill_dead_rows_kernel, dim3((int)(blocks < 8192 ? blocks : 8192)), dim3(256), 0, stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (p.q_runs.total() == 0) return hipSuccess;
  const int grid = mapped_grid(p.batch * p.kv_heads, p.q_heads / p.kv_heads, p.q_runs.total());
  hipLaunchKernelGGL((step_fwd_kernel<D, kFwdBQ / 32>), dim3(grid), dim3(2 * kFwdBQ), LDS, stream, p);
  return hipGetLastError();
}

// With the fused merge and no separate step result, a key axis longer than two ranges is cut into ranges, one
// launch per range, each folding its part into the running (O, Lse): the same online-softmax merge the ring
// applies from step to step, so the result is the step's up to rounding.  The step result itself (o_part,
// lse_part) cannot be cut this way and is always one launch.
template <int D>
static hipError_t launch_fwd_chunked(const FwdParams& p0, hipStream_t stream) {
  if (!p0.o_acc.ptr || p0.o_part.ptr) return launch_fwd_t<D>(p0, stream);
  const std::vector<RowRange> ranges = chunk_ranges(p0.mask.k_nseg, p0.mask.k_seg_len, p0.sk, p0.mask.blk ? p0.mask.blk_k : 0);
  if (ranges.size() == 1) return launch_fwd_t<D>(p0, stream);
  for (const RowRange& rg : ranges) {
    FwdParams p = p0;
    p.mask = sub_mask<false>(p0.mask, rg.r0, rg.r1);
    p.sk = rg.r1 - rg.r0;
    offset_rows(p.k, rg.r0);
    offset_rows(p.v, rg.r0);
    hipError_t e = launch_fwd_t<D>(p, stream);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_step_fwd(const FwdParams& p, hipStream_t stream) {
  if (p.head_dim == 128) return launch_fwd_chunked<128>(p, stream);
  return launch_fwd_chunked<64>(p, stream);
}

}  // namespace burst
