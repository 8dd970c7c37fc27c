// Forward step kernel: O_ij, Lse_cur of a query chunk against one key/value chunk (Eq. 5-6),
// optionally folded into the running (O_i, Lse_i) in the epilogue (forward algorithm lines 6-9).
//
// One work-group = 4 waves = 128*QB query rows of one (batch, head); wave w owns rows
// [32*QB*w, 32*QB*(w+1)).  The key/value chunk streams through LDS in tiles of 64 rows, double
// buffered, one barrier per tile.  Everything is computed transposed so that a lane always owns one
// query row:  S^T = K Q^T  (A = K rows from LDS, B = Q held in registers),  P^T = exp2(..) in the
// accumulator registers, packed to bf16 and fed straight back as the B operand of
// O^T = V^T P^T  (A = V columns via transposing LDS reads).  Row max / row sum / rescale are then
// per-lane scalars; the two half-waves exchange one value per tile.
#include "common.hpp"
#include "kernels.hpp"

namespace burst {

template <int D, int QB>
__global__ __launch_bounds__(256, 2) void step_fwd_kernel(FwdParams p) {
  constexpr int BK = 64, KB = BK / 32, DK = D / 16, DB = D / 32;
  constexpr int BQ = 128 * QB;
  constexpr int PITCH = 2 * D + 16;
  constexpr int TILE = BK * PITCH;
  extern __shared__ __attribute__((aligned(16))) char smem[];  // [2 buffers][K tile, V tile]

  const int group = p.q_heads / p.kv_heads;
  const int q_tiles = (p.sq + BQ - 1) / BQ;
  const BlockMap bm = map_block(blockIdx.x, p.batch * p.kv_heads, group, q_tiles);
  if (!bm.valid) return;
  const int b = bm.key / p.kv_heads, hk = bm.key - b * p.kv_heads, hq = hk * group + bm.head_in_group;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r = lane & 31, h = lane >> 5;
  const int sq = p.sq, sk = p.sk;
  const MaskDev mk = p.mask;
  const int q_blk0 = bm.tile * BQ;                       // first row of the work-group
  const int q_blk1 = min(q_blk0 + BQ, sq);
  const int q_w0 = q_blk0 + wave * 32 * QB;              // first row of the wave
  const int q_w1 = min(q_w0 + 32 * QB, sq);              // may be <= q_w0: the wave only helps staging

  const __bf16* qg = (const __bf16*)p.q.ptr + b * p.q.sb + hq * p.q.sh;
  const __bf16* kg = (const __bf16*)p.k.ptr + b * p.k.sb + hk * p.k.sh;
  const __bf16* vg = (const __bf16*)p.v.ptr + b * p.v.sb + hk * p.v.sh;

  // Q as the B operand of S^T = K Q^T: lane holds Q[row][16*ks + 8h .. +7]
  bf16x8 qreg[QB][DK];
  int qpos[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    int row = min(q_w0 + qb * 32 + r, sq - 1);
    qpos[qb] = seg_position(row, mk.q_nseg, mk.q_seg_len, mk.q_seg_pos, mk.pos_stride);
    const __bf16* src = qg + (int64_t)row * p.q.ss + 8 * h;
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) qreg[qb][ks] = *reinterpret_cast<const bf16x8*>(src + ks * 16);
  }

  f32x16 o[QB][DB];
  float m_run[QB], l_run[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m_run[qb] = -INFINITY;
    l_run[qb] = 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[qb][db][v] = 0.f;
  }
  const float c = p.scale * kLog2e;

  const int n_tiles = (sk + BK - 1) / BK;
  auto next_tile = [&](int t) {
    while (t < n_tiles && classify(mk, q_blk0, q_blk1, t * BK, min(t * BK + BK, sk), false) == TILE_SKIP) ++t;
    return t;
  };

  wait_global_loads();
  TileStager<D, BK> stage_k, stage_v;
  int t = next_tile(0);
  if (t < n_tiles) {
    stage_k.load(kg, p.k.ss, t * BK, sk, tid);
    stage_v.load(vg, p.v.ss, t * BK, sk, tid);
    stage_k.store(smem, tid);
    stage_v.store(smem + TILE, tid);
  }
  __syncthreads();
  int buf = 0;
  while (t < n_tiles) {
    const int tn = next_tile(t + 1);
    if (tn < n_tiles) {
      stage_k.load(kg, p.k.ss, tn * BK, sk, tid);
      stage_v.load(vg, p.v.ss, tn * BK, sk, tid);
    }
    const char* kt = smem + buf * 2 * TILE;
    const char* vt = kt + TILE;
    const int cls = classify(mk, q_w0, q_w1, t * BK, min(t * BK + BK, sk), t * BK + BK > sk);   // wave-uniform
    if (cls != TILE_SKIP) {
      f32x16 s[KB][QB];
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
          for (int v = 0; v < 16; ++v) s[kb][qb][v] = 0.f;
      // k-step outermost: consecutive MFMAs go to different accumulators (a dependent
      // accumulate chain issues at little more than half rate)
#pragma unroll
      for (int ks = 0; ks < DK; ++ks) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
          bf16x8 a = lds_rows_operand<PITCH>(kt, kb * 32, ks * 16, r, h);
#pragma unroll
          for (int qb = 0; qb < QB; ++qb) s[kb][qb] = mfma32(a, qreg[qb][ks], s[kb][qb]);
        }
      }
      if (cls == TILE_PARTIAL) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int qb = 0; qb < QB; ++qb) mask_tile<true>(s[kb][qb], mk, t * BK + kb * 32 + 4 * h, sk, qpos[qb]);
      }
      bf16x8 pp[QB][KB][2];
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        float mx = s[0][qb][0];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[kb][qb][v]);
        mx = fmaxf(mx, half_swap(mx));
        const float m_old = m_run[qb];
        const float m_new = fmaxf(m_old, mx);
        // Rescale lazily: keep a stale maximum while no row of the wave has grown by more than
        // 2^kLazyLog2 (any common per-row offset gives the same result; fp32 has the headroom).
        const bool grow = c * (m_new - m_old) > kLazyLog2;   // false for -inf - -inf
        if (__any(grow)) {
          const float alpha = (m_new == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f(c * (m_old - m_new));
          m_run[qb] = m_new;
          l_run[qb] *= alpha;
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[qb][db][v] *= alpha;
        }
        const float msub = (m_run[qb] == -INFINITY) ? 0.f : c * m_run[qb];
        float sum = 0.f;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            float e = __builtin_amdgcn_exp2f(c * s[kb][qb][v] - msub);
            s[kb][qb][v] = e;
            sum += e;
          }
          pp[qb][kb][0] = pack8(s[kb][qb], 0);
          pp[qb][kb][1] = pack8(s[kb][qb], 1);
        }
        l_run[qb] += sum;
      }
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int kc = 0; kc < 2; ++kc)
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            bf16x8 a = lds_cols_operand<PITCH>(vt, kb * 32 + kc * 16, db * 32, lane);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) o[qb][db] = mfma32(a, pp[qb][kb][kc], o[qb][db]);
          }
    }
    if (tn < n_tiles) {
      char* nk = smem + (buf ^ 1) * 2 * TILE;
      stage_k.store(nk, tid);
      stage_v.store(nk + TILE, tid);
    }
    __syncthreads();
    t = tn;
    buf ^= 1;
  }

  // Epilogue: normalise, Lse in natural-log units, optional online-softmax merge.
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int row = q_w0 + qb * 32 + r;
    const float l_tot = l_run[qb] + half_swap(l_run[qb]);
    const bool alive = l_tot > 0.f;
    const float inv = alive ? 1.f / l_tot : 0.f;
    const float lse_cur = alive ? (c * m_run[qb] + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
    if (row >= sq) continue;
    if (p.o_part.ptr) {
      if (p.o_part.is_f32) {
        float* dst = (float*)p.o_part.ptr + b * p.o_part.sb + (int64_t)row * p.o_part.ss + hq * p.o_part.sh;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            f32x4 x = {o[qb][db][4 * g] * inv, o[qb][db][4 * g + 1] * inv, o[qb][db][4 * g + 2] * inv,
                       o[qb][db][4 * g + 3] * inv};
            *reinterpret_cast<f32x4*>(dst + db * 32 + 8 * g + 4 * h) = x;
          }
      } else {
        __bf16* dst = (__bf16*)p.o_part.ptr + b * p.o_part.sb + (int64_t)row * p.o_part.ss + hq * p.o_part.sh;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            bf16x4 x = {(__bf16)(o[qb][db][4 * g] * inv), (__bf16)(o[qb][db][4 * g + 1] * inv),
                        (__bf16)(o[qb][db][4 * g + 2] * inv), (__bf16)(o[qb][db][4 * g + 3] * inv)};
            *reinterpret_cast<bf16x4*>(dst + db * 32 + 8 * g + 4 * h) = x;
          }
      }
      if (h == 0) p.lse_part.ptr[b * p.lse_part.sb + hq * p.lse_part.sh + row] = lse_cur;
    }
    if (p.o_acc.ptr) {
      float* lse_ptr = p.lse_acc.ptr + b * p.lse_acc.sb + hq * p.lse_acc.sh + row;
      const float lse_old = *lse_ptr;
      const float mm = fmaxf(lse_old, lse_cur);
      float w_old = 1.f, w_cur = 0.f, lse_new = lse_old;
      if (mm != -INFINITY) {
        const float e_old = __expf(lse_old - mm), e_cur = __expf(lse_cur - mm);
        const float tot = e_old + e_cur;
        lse_new = mm + __logf(tot);
        w_old = e_old / tot;
        w_cur = e_cur / tot;
      }
      const float w_cur_n = w_cur * inv;
      float* dst = (float*)p.o_acc.ptr + b * p.o_acc.sb + (int64_t)row * p.o_acc.ss + hq * p.o_acc.sh;
      if (alive) {   // a step that saw no key leaves the running state untouched
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            float* q4 = dst + db * 32 + 8 * g + 4 * h;
            f32x4 old = *reinterpret_cast<const f32x4*>(q4);
            f32x4 x = {o[qb][db][4 * g] * w_cur_n + old[0] * w_old, o[qb][db][4 * g + 1] * w_cur_n + old[1] * w_old,
                       o[qb][db][4 * g + 2] * w_cur_n + old[2] * w_old, o[qb][db][4 * g + 3] * w_cur_n + old[3] * w_old};
            *reinterpret_cast<f32x4*>(q4) = x;
          }
      }
      // both half-waves have read lse_old before either writes: the read above precedes this
      // store in program order and the wave executes in lockstep
      if (h == 0 && alive) *lse_ptr = lse_new;
    }
  }
}

template <int D, int QB>
static hipError_t launch_fwd_t(const FwdParams& p, hipStream_t stream) {
  constexpr int BQ = 128 * QB;
  constexpr int LDS = 2 * 2 * 64 * (2 * D + 16);
  const int q_tiles = (p.sq + BQ - 1) / BQ;
  const int grid = mapped_grid(p.batch * p.kv_heads, p.q_heads / p.kv_heads, q_tiles);
  hipLaunchKernelGGL((step_fwd_kernel<D, QB>), dim3(grid), dim3(256), LDS, stream, p);
  return hipGetLastError();
}

hipError_t launch_step_fwd(const FwdParams& p, hipStream_t stream) {
  if (p.head_dim == 128) return launch_fwd_t<128, 1>(p, stream);
  return launch_fwd_t<64, 1>(p, stream);
}

}  // namespace burst
