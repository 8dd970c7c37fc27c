// Sequence-level fusion of the LM head and the loss function (Sec. 3.3, Eq. 9, Alg. 3).
//
// Per sequence tile of B_s tokens, four launches:
//   1. lm_logits_kernel       Logits^T tile = W_head H_i^T on the matrix cores (bf16 in, fp32 out).
//                             Computed transposed so that a lane owns a token: the per-token
//                             (max, sum of exp) over the wave's 128 words is a reduction over the
//                             lane's own registers, as in the attention forward.  The fp32 logits of
//                             the tile go to the workspace (the algorithm keeps them between its two
//                             sweeps over the vocabulary); the partial (max, sum) pairs go to a side array.
//   2. lm_loss_dlogits_kernel one work-group per token: merges the partial pairs into Lse_i, writes
//                             the loss, then streams the token's logits once and writes
//                             grad_scale * (exp(Logits - Lse) - E) as bf16 (HBM-bound).
//   3. lm_dh_kernel           dH_i  = dLogits W_head          (contraction over the vocabulary)
//   4. lm_transpose_h_kernel + lm_dw_kernel
//                             dW^T += H_i^T dLogits           (contraction over the tile's tokens)
// The three GEMMs share one main loop: 256 x 256 output tile per work-group of 8 waves (wave tile
// 128 x 64, 128 accumulator registers), k-tiles of 64 double-buffered in LDS, operands read from LDS
// either row-wise (the matrix is stored with the contraction index contiguous) or column-wise with
// the transposing LDS read (the contraction index is the storage row).  Only H_i, a few MB per
// sequence tile, is ever transposed in memory.  The wave tile is as large as 128 accumulator
// registers allow (0.75 KB of LDS operand reads per MFMA); the loop over the k-tiles has no branches
// and carries the staging of the next k-tile between its MFMAs.
#include <type_traits>

#include "common.hpp"
#include "kernels.hpp"

namespace burst {

namespace {

// Output tile of a work-group: 256 x kLmBN, k-tiles of kLmBK, one wave per 128 x kLmWN sub-tile.
// The defaults (256, 64, 64: eight waves, one work-group per CU) measured fastest; 128 x 128 wave
// tiles at one wave per SIMD and two 256 x 128 work-groups per CU with k-tiles of 32 build from the
// same source and were slower.
#ifndef LM_BN
#define LM_BN 256
#endif
#ifndef LM_BK
#define LM_BK 64
#endif
#ifndef LM_WN
#define LM_WN 64
#endif
constexpr int kLmBM = 256, kLmBN = LM_BN, kLmBK = LM_BK, kLmKS = kLmBK / 16, kLmWN = LM_WN, kLmNB = kLmWN / 32;
constexpr int kLmWaves = (kLmBM / 128) * (kLmBN / kLmWN), kLmThreads = 64 * kLmWaves;
constexpr int kLmPerCU = kLmWN == 128 ? 1 : 512 / kLmThreads;

// One GEMM operand: where its k-tiles come from and how they are staged.  X: extent of the tile
// along the operand's own (non-contracted) index.
//   COLS = false: storage [x][k], k contiguous; the tile is rows x0 .. x0+X-1, columns k0 .. k0+BK-1.
//                 lim = number of valid storage rows; rows beyond are read as the last valid row
//                 (the clamp is folded into the per-thread offsets once).
//   COLS = true : storage [k][x], x contiguous; the tile is rows k0 .. k0+BK-1, columns x0 .. x0+X-1
//                 (always inside the row), its rows permuted in LDS so that the column-wise read
//                 hands out k in the row-wise operand's order.  lim = number of valid k rows: the
//                 k-tiles that reach past it take the slower load with per-row clamping.
template <bool COLS, int X>
struct LmOperand {
  using Stager = std::conditional_t<COLS, TileStager<X, kLmBK, kLmThreads, true>, TileStager<kLmBK, X, kLmThreads>>;
  static constexpr int BYTES = (COLS ? kLmBK : X) * Stager::PITCH;
  static constexpr int PASSES = Stager::PASSES;
  Stager st;
  const __bf16* base;
  const char* tile;     // next k-tile to stage
  int64_t ld, step;
  int lim, k0;

  __device__ __forceinline__ void init(const __bf16* ptr, int64_t ld_, int lim_, int x0, int tid) {
    ld = ld_;
    lim = lim_;
    k0 = 0;
    base = COLS ? ptr + x0 : ptr;
    tile = reinterpret_cast<const char*>(COLS ? ptr + x0 : ptr + (int64_t)x0 * ld);
    step = COLS ? kLmBK * ld * 2 : kLmBK * 2;
    st.init(ld, tid, COLS ? kLmBK : min(X, lim - x0));
  }
  // leading k-tiles that the plain loads can stage
  __device__ __forceinline__ int plain_tiles(int nk) const { return COLS ? min(nk, lim / kLmBK) : nk; }
  __device__ __forceinline__ void load_pass(int i) { st.load_pass(tile, i); }   // plain k-tiles only
  __device__ __forceinline__ void next() {
    tile += step;
    k0 += kLmBK;
  }
  __device__ __forceinline__ void issue(int tid) {   // any k-tile
    if (!COLS || k0 + kLmBK <= lim) st.load_at(tile);
    else st.load(base, ld, k0, lim, tid);
    next();
  }
  __device__ __forceinline__ void commit(char* lds) const { st.store(lds); }
  // fragment for the 16-wide k-step ks of the tile in LDS: lane -> row / column x_off + (lane & 31)
  static __device__ __forceinline__ bf16x8 frag(const char* lds, int x_off, int ks, int lane) {
    if (COLS) return lds_cols_operand<Stager::PITCH>(lds, ks * 16, x_off, lane);
    return lds_rows_operand<Stager::PITCH>(lds, x_off, ks * 16, lane & 31, lane >> 5);
  }
};

template <bool A_COLS, bool B_COLS>
struct LmGemm {
  using OpA = LmOperand<A_COLS, kLmBM>;
  using OpB = LmOperand<B_COLS, kLmBN>;
  static constexpr int STAGE = OpA::BYTES + OpB::BYTES;
  static constexpr int LDS = 2 * STAGE;
  static constexpr int NMFMA = 4 * kLmNB;     // MFMAs per 16-wide k-step

  // The MFMAs of the k-tile in LDS buffer `cur`.  STAGE_NEXT: 0 = nothing else; 1 = the next k-tile
  // is staged into buffer `nxt` with plain loads, one load or LDS write slipped in after every few
  // MFMAs (loads during the first half of the k-steps, LDS writes during the second), so that the
  // waves of a work-group, which the barrier keeps in phase, do not all queue at the memory pipe
  // and then at the LDS write port while the matrix pipe idles; 2 = the next k-tile needs the
  // clamping loads: issued whole before the MFMAs, written whole after them.
  template <int STAGE_NEXT>
  static __device__ __forceinline__ void k_tile(f32x16 (&acc)[4][kLmNB], const char* cur, char* nxt, OpA& a, OpB& b, int wm,
                                                int wn, int tid, int lane) {
    const char* at = cur;
    const char* bt = cur + OpA::BYTES;
    bf16x8 af[2][4], bf[2][kLmNB];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) af[0][mb] = OpA::frag(at, wm * 128 + 32 * mb, 0, lane);
#pragma unroll
    for (int nb = 0; nb < kLmNB; ++nb) bf[0][nb] = OpB::frag(bt, wn * kLmWN + 32 * nb, 0, lane);
    if (STAGE_NEXT == 2) {
      a.issue(tid);
      b.issue(tid);
    }
    constexpr int HALF = kLmKS / 2 > 0 ? kLmKS / 2 : 1;                 // k-steps that carry loads
    constexpr int SLOTS = HALF * NMFMA;                                 // MFMAs that may be followed by a load
    constexpr int NOPS = OpA::PASSES + OpB::PASSES;
    constexpr int EVERY = SLOTS / NOPS > 0 ? SLOTS / NOPS : 1;
#pragma unroll
    for (int ks = 0; ks < kLmKS; ++ks) {
      if (ks + 1 < kLmKS) {
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) af[(ks + 1) & 1][mb] = OpA::frag(at, wm * 128 + 32 * mb, ks + 1, lane);
#pragma unroll
        for (int nb = 0; nb < kLmNB; ++nb) bf[(ks + 1) & 1][nb] = OpB::frag(bt, wn * kLmWN + 32 * nb, ks + 1, lane);
      }
#pragma unroll
      for (int m = 0; m < NMFMA; ++m) {
        const int mb = m / kLmNB, nb = m % kLmNB;
        acc[mb][nb] = mfma32(af[ks & 1][mb], bf[ks & 1][nb], acc[mb][nb]);
        if (STAGE_NEXT == 1) {
          const int slot = (ks % HALF) * NMFMA + m;       // position within its half
          if (slot % EVERY == EVERY - 1 && slot / EVERY < NOPS) {
            const int op = slot / EVERY;
            if (ks < HALF || kLmKS == 1) {
              if (op < OpA::PASSES) a.load_pass(op);
              else b.load_pass(op - OpA::PASSES);
            }
            if (ks >= HALF || kLmKS == 1) {
              if (op < OpA::PASSES) a.st.store_pass(nxt, op);
              else b.st.store_pass(nxt + OpA::BYTES, op - OpA::PASSES);
            }
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if (STAGE_NEXT == 1) {
      a.next();
      b.next();
    }
    if (STAGE_NEXT == 2) {
      a.commit(nxt);
      b.commit(nxt + OpA::BYTES);
    }
  }

  // acc[mb][nb]: rows 32 mb + ... of the wave's 128, columns 32 nb + ... of its kLmWN.  nk >= 1 k-tiles,
  // double-buffered in LDS, one barrier per k-tile.  The loop over the k-tiles that plain loads can
  // stage is free of branches.
  static __device__ __forceinline__ void run(f32x16 (&acc)[4][kLmNB], char* smem, OpA& a, OpB& b, int nk, int wm, int wn,
                                             int tid, int lane) {
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int nb = 0; nb < kLmNB; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.f;
    const int n_plain = min(a.plain_tiles(nk), b.plain_tiles(nk));   // k-tiles 0 .. n_plain-1 are plain
    a.issue(tid);
    b.issue(tid);
    a.commit(smem);
    b.commit(smem + OpA::BYTES);
    __syncthreads();
    int kt = 0, buf = 0;
    for (; kt + 1 < n_plain; ++kt) {        // stages tile kt + 1 < n_plain
      k_tile<1>(acc, smem + buf * STAGE, smem + (buf ^ 1) * STAGE, a, b, wm, wn, tid, lane);
      __syncthreads();
      buf ^= 1;
    }
    for (; kt + 1 < nk; ++kt) {
      k_tile<2>(acc, smem + buf * STAGE, smem + (buf ^ 1) * STAGE, a, b, wm, wn, tid, lane);
      __syncthreads();
      buf ^= 1;
    }
    k_tile<0>(acc, smem + buf * STAGE, nullptr, a, b, wm, wn, tid, lane);
  }
};

// Work-group -> output tile.  Work-group n runs on XCD n mod 8; each XCD takes groups of 4 x 8
// tiles (one per CU), so the 32 work-groups that share an L2 at a time read 4 + 8 operand panels.
__device__ __forceinline__ bool lm_tile(int bid, int TM, int TN, int& tm, int& tn) {
  const int groups_m = (TM + 3) / 4, groups_n = (TN + 7) / 8;
  const int xcd = bid & 7, slot = bid >> 3;
  const int group = (slot >> 5) * 8 + xcd, within = slot & 31;
  if (group >= groups_m * groups_n) return false;
  const int gm = group % groups_m, gn = group / groups_m;
  tm = gm * 4 + (within & 3);
  tn = gn * 8 + (within >> 2);
  return tm < TM && tn < TN;
}
int lm_grid(int TM, int TN) {
  const int groups = ((TM + 3) / 4) * ((TN + 7) / 8);
  return (groups + 7) / 8 * 8 * 32;
}

// (max, sum of exp(x - max)) pairs combine like the log-sum-exp merge of the attention forward.
__device__ __forceinline__ void lm_combine(float& m, float& l, float m2, float l2) {
  const float mm = fmaxf(m, m2);
  l = (mm == -INFINITY) ? 0.f : l * __expf(m - mm) + l2 * __expf(m2 - mm);
  m = mm;
}

// ---------------------------------------------------------------------------------------------
// 1. Logits^T tile (rows: words, columns: tokens of the sequence tile), Alg. 3 forward sweep.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kLmThreads, kLmPerCU) void lm_logits_kernel(LmHeadParams p, int s0, int n_rows, int TM, int TN) {
  using G = LmGemm<false, false>;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  int tm, tn;
  if (!lm_tile(blockIdx.x, TM, TN, tm, tn)) return;
  const int tid = threadIdx.x, lane = tid & 63, r = lane & 31, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), wm = wave & 1, wn = wave >> 1;
  const int m0 = tm * kLmBM, n0 = tn * kLmBN;
  G::OpA a;
  G::OpB b;
  a.init(p.w, p.ld_w, p.vocab, m0, tid);
  b.init(p.h + (int64_t)s0 * p.ld_h, p.ld_h, n_rows, n0, tid);
  f32x16 acc[4][kLmNB];
  G::run(acc, smem, a, b, p.d_model / kLmBK, wm, wn, tid, lane);

  const int word0 = m0 + wm * 128;                 // first word of the wave
#pragma unroll
  for (int nb = 0; nb < kLmNB; ++nb) {
    const int token = n0 + wn * kLmWN + 32 * nb + r;  // < tile_tokens: the tile count covers n_rows only
    float* dst = p.logits + (int64_t)token * p.v_pad + word0 + 4 * h;
    float mx = -INFINITY;
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        f32x4 x = {acc[mb][nb][4 * g], acc[mb][nb][4 * g + 1], acc[mb][nb][4 * g + 2], acc[mb][nb][4 * g + 3]};
        *reinterpret_cast<f32x4*>(dst + 32 * mb + 8 * g) = x;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const bool real = word0 + 32 * mb + 8 * g + 4 * h + j < p.vocab;   // padding words stay out of Lse
          acc[mb][nb][4 * g + j] = real ? x[j] : -INFINITY;
          mx = fmaxf(mx, acc[mb][nb][4 * g + j]);
        }
      }
    mx = fmaxf(mx, half_swap(mx));
    float sum = 0.f;
    if (mx != -INFINITY) {
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) sum += __expf(acc[mb][nb][v] - mx);
    }
    sum += half_swap(sum);
    if (h == 0) p.part[(int64_t)(tm * 2 + wm) * p.tile_tokens + token] = float2{mx, sum};
  }
}

// ---------------------------------------------------------------------------------------------
// 2. Lse_i, loss_i and dLogits of one token per work-group (Alg. 3: the loss line and the first
//    two lines of the backward sweep).  Rows n_rows .. gridDim.x-1 are zero-filled: they pad the
//    contraction of the dW GEMM.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void lm_loss_dlogits_kernel(LmHeadParams p, int s0, int n_rows, int want_grad) {
  __shared__ float red_m[4], red_l[4];
  const int i = blockIdx.x, tid = threadIdx.x;
  __bf16* drow = p.dlogits + (int64_t)i * p.v_pad;
  const bf16x8 zero8 = {(__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f};
  if (i >= n_rows) {
    for (int j = tid * 8; j < p.v_pad; j += 2048) *reinterpret_cast<bf16x8*>(drow + j) = zero8;
    return;
  }
  float m = -INFINITY, l = 0.f;
  const int n_part = p.v_pad / 128;
  for (int pp = tid; pp < n_part; pp += 256) {
    const float2 x = p.part[(int64_t)pp * p.tile_tokens + i];
    lm_combine(m, l, x.x, x.y);
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) lm_combine(m, l, __shfl_xor(m, off), __shfl_xor(l, off));
  if ((tid & 63) == 0) {
    red_m[tid >> 6] = m;
    red_l[tid >> 6] = l;
  }
  __syncthreads();
  m = red_m[0];
  l = red_l[0];
#pragma unroll
  for (int w = 1; w < 4; ++w) lm_combine(m, l, red_m[w], red_l[w]);
  const float lse = m + __logf(l);
  const int64_t y = p.y[s0 + i];
  const bool ok = y >= 0 && y < p.vocab;
  const float* lrow = p.logits + (int64_t)i * p.v_pad;
  if (tid == 0) {
    p.loss[s0 + i] = ok ? lse - lrow[ok ? y : 0] : 0.f;
    if (p.lse) p.lse[s0 + i] = lse;
  }
  if (!want_grad) return;
  if (!ok) {
    for (int j = tid * 8; j < p.v_pad; j += 2048) *reinterpret_cast<bf16x8*>(drow + j) = zero8;
    return;
  }
  const int yi = (int)y;
  const float gs = p.grad_scale;
  for (int j = tid * 8; j < p.v_pad; j += 2048) {
    const f32x4 x0 = *reinterpret_cast<const f32x4*>(lrow + j), x1 = *reinterpret_cast<const f32x4*>(lrow + j + 4);
    bf16x8 out;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float x = e < 4 ? x0[e] : x1[e - 4];
      const float g = gs * (__expf(x - lse) - (j + e == yi ? 1.f : 0.f));
      out[e] = (__bf16)(j + e < p.vocab ? g : 0.f);
    }
    *reinterpret_cast<bf16x8*>(drow + j) = out;
  }
}

// ---------------------------------------------------------------------------------------------
// 3. dH_i = dLogits W_head (rows: tokens, columns: hidden, contraction: words).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kLmThreads, kLmPerCU) void lm_dh_kernel(LmHeadParams p, int s0, int n_rows, int TM, int TN) {
  using G = LmGemm<false, true>;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  int tm, tn;
  if (!lm_tile(blockIdx.x, TM, TN, tm, tn)) return;
  const int tid = threadIdx.x, lane = tid & 63, r = lane & 31, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), wm = wave & 1, wn = wave >> 1;
  const int m0 = tm * kLmBM, n0 = tn * kLmBN;
  G::OpA a;
  G::OpB b;
  a.init(p.dlogits, p.v_pad, p.tile_tokens, m0, tid);
  b.init(p.w, p.ld_w, p.vocab, n0, tid);
  f32x16 acc[4][kLmNB];
  G::run(acc, smem, a, b, (p.vocab + kLmBK - 1) / kLmBK, wm, wn, tid, lane);   // dLogits is zero beyond the vocabulary
#pragma unroll
  for (int mb = 0; mb < 4; ++mb)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = m0 + wm * 128 + 32 * mb + 8 * (v >> 2) + 4 * h + (v & 3);
      if (row >= n_rows) continue;
#pragma unroll
      for (int nb = 0; nb < kLmNB; ++nb) {
        const int64_t off = (int64_t)(s0 + row) * p.ld_dh + n0 + wn * kLmWN + 32 * nb + r;
        if (p.dh_is_f32) ((float*)p.dh)[off] = acc[mb][nb][v];
        else ((__bf16*)p.dh)[off] = (__bf16)acc[mb][nb][v];
      }
    }
}

// ---------------------------------------------------------------------------------------------
// 4. dW (+)= dLogits^T H_i, computed as its transpose dW^T = H_i^T dLogits (rows: hidden,
//    columns: words, contraction: tokens of the tile).  Both factors are stored with the token as
//    the row, and an operand read column-wise costs twice the LDS instructions of a row-wise one;
//    the four-fragment A operand is therefore taken from a transposed copy of H_i (a few MB,
//    written by lm_transpose_h_kernel once per sequence tile), and only the two-fragment B operand
//    (dLogits) uses the transposing read.  A lane then owns a word: it adds four consecutive
//    hidden columns of that word's row of dW at a time.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void lm_transpose_h_kernel(LmHeadParams p, int s0, int n_rows) {
  __shared__ __bf16 tile[64][66];
  const int t0 = blockIdx.x * 64, d0 = blockIdx.y * 64, tid = threadIdx.x;   // 64 tokens x 64 hidden columns
  for (int i = tid; i < 64 * 8; i += 256) {
    const int tok = i >> 3, c8 = (i & 7) * 8;
    bf16x8 x = {(__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f, (__bf16)0.f};
    if (t0 + tok < n_rows) x = *reinterpret_cast<const bf16x8*>(p.h + (int64_t)(s0 + t0 + tok) * p.ld_h + d0 + c8);
#pragma unroll
    for (int e = 0; e < 8; ++e) tile[tok][c8 + e] = x[e];
  }
  __syncthreads();
  for (int i = tid; i < 64 * 8; i += 256) {
    const int dc = i >> 3, t8 = (i & 7) * 8;
    bf16x8 x;
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = tile[t8 + e][dc];
    *reinterpret_cast<bf16x8*>(p.ht + (int64_t)(d0 + dc) * p.tile_tokens + t0 + t8) = x;
  }
}

__global__ __launch_bounds__(kLmThreads, kLmPerCU) void lm_dw_kernel(LmHeadParams p, int s0, int n_rows, int TM, int TN, int accumulate) {
  using G = LmGemm<false, true>;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  int tm, tn;
  if (!lm_tile(blockIdx.x, TM, TN, tm, tn)) return;
  const int tid = threadIdx.x, lane = tid & 63, r = lane & 31, h = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), wm = wave & 1, wn = wave >> 1;
  const int m0 = tm * kLmBM, n0 = tn * kLmBN;      // first hidden column, first word
  G::OpA a;
  G::OpB b;
  a.init(p.ht, p.tile_tokens, p.d_model, m0, tid);
  b.init(p.dlogits, p.v_pad, p.tile_tokens, n0, tid);
  f32x16 acc[4][kLmNB];
  G::run(acc, smem, a, b, (n_rows + kLmBK - 1) / kLmBK, wm, wn, tid, lane);    // both factors are zero beyond n_rows
#pragma unroll
  for (int nb = 0; nb < kLmNB; ++nb) {
    const int word = n0 + wn * kLmWN + 32 * nb + r;
    if (word >= p.vocab) continue;
    float* dst = p.dw + (int64_t)word * p.ld_dw + m0 + wm * 128 + 4 * h;
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        f32x4 x = {acc[mb][nb][4 * g], acc[mb][nb][4 * g + 1], acc[mb][nb][4 * g + 2], acc[mb][nb][4 * g + 3]};
        f32x4* q4 = reinterpret_cast<f32x4*>(dst + 32 * mb + 8 * g);
        if (accumulate) x += *q4;
        *q4 = x;
      }
  }
}

__global__ __launch_bounds__(256) void lm_zero_dw_kernel(LmHeadParams p) {
  const int d4 = p.d_model / 4;
  const int64_t total = (int64_t)p.vocab * d4;
  for (int64_t i = blockIdx.x * 256ll + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256)
    *reinterpret_cast<f32x4*>(p.dw + (i / d4) * p.ld_dw + (i % d4) * 4) = f32x4{0.f, 0.f, 0.f, 0.f};
}

}  // namespace

int64_t lm_head_workspace_bytes(int64_t tile_tokens, int64_t vocab, int64_t d_model) {
  const int64_t v_pad = (vocab + 255) / 256 * 256;
  return tile_tokens * v_pad * 4 + tile_tokens * v_pad * 2 + (v_pad / 128) * tile_tokens * 8 + d_model * tile_tokens * 2;
}

hipError_t launch_lm_head_loss(const LmHeadParams& p, hipStream_t stream) {
  const int want_grad = (p.dh || p.dw) ? 1 : 0;
  const int TD = p.d_model / kLmBN, TV = p.v_pad / kLmBM;   // column tiles of dH / dW, row tiles over the vocabulary
  constexpr int kLdsLogits = LmGemm<false, false>::LDS, kLdsDh = LmGemm<false, true>::LDS, kLdsDw = LmGemm<false, true>::LDS;
  if (p.n_tokens == 0 && p.dw && !p.acc_dw) {
    hipLaunchKernelGGL(lm_zero_dw_kernel, dim3(2048), dim3(256), 0, stream, p);
    return hipGetLastError();
  }
  for (int s0 = 0; s0 < p.n_tokens; s0 += p.tile_tokens) {
    const int n_rows = p.n_tokens - s0 < p.tile_tokens ? p.n_tokens - s0 : p.tile_tokens;
    const int TT = (n_rows + kLmBM - 1) / kLmBM, TTn = (n_rows + kLmBN - 1) / kLmBN, k_rows = (n_rows + 63) / 64 * 64;
    hipLaunchKernelGGL(lm_logits_kernel, dim3(lm_grid(TV, TTn)), dim3(kLmThreads), kLdsLogits, stream, p, s0,
                       n_rows, TV, TTn);
    hipLaunchKernelGGL(lm_loss_dlogits_kernel, dim3(want_grad ? k_rows : n_rows), dim3(256), 0, stream, p, s0, n_rows, want_grad);
    if (p.dh)
      hipLaunchKernelGGL(lm_dh_kernel, dim3(lm_grid(TT, TD)), dim3(kLmThreads), kLdsDh, stream, p, s0, n_rows,
                         TT, TD);
    if (p.dw) {
      hipLaunchKernelGGL(lm_transpose_h_kernel, dim3(k_rows / 64, p.d_model / 64), dim3(256), 0, stream, p, s0, n_rows);
      hipLaunchKernelGGL(lm_dw_kernel, dim3(lm_grid(p.d_model / kLmBM, p.v_pad / kLmBN)), dim3(kLmThreads), kLdsDw, stream, p,
                         s0, n_rows, p.d_model / kLmBM, p.v_pad / kLmBN, (p.acc_dw || s0 > 0) ? 1 : 0);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace burst
