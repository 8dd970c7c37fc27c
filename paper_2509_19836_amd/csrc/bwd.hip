// Backward step kernels (Alg. 2, with the softmax scale restored):
//   S = scale Q K^T; P = exp(S - Lse); dV += P^T dO; dP = dO V^T; dS = P o (dP - D);
//   dK += scale dS^T Q; dQ += scale dS K.
//
// Two kernels, each owning its outputs outright (no atomics, results are run-to-run identical):
//
//  * dQ kernel, query-stationary (same orientation as the forward kernel): a lane owns one query
//    row; S^T = K Q^T and dP^T = V dO^T come out with the key index in the accumulator registers,
//    dS^T is packed to bf16 in place and fed back as the B operand of dQ^T = K^T dS^T, whose A
//    operand is the K tile read column-wise (transposing LDS reads) from the same LDS copy that
//    served S^T row-wise.
//
//  * dK/dV kernel, key-stationary: a lane owns one key row; K and V rows live in registers as B
//    operands, S = Q K^T and dP = dO V^T come out with the query index in the accumulator registers,
//    P and dS are packed in place and fed back as B operands of dV^T = dO^T P and dK^T = Q^T dS,
//    whose A operands are the dO and Q tiles read column-wise from the LDS copies that served
//    S and dP row-wise.  With grouped-query attention the work-group walks the query heads of its
//    group, so dK and dV are summed over the group in registers.
#include "common.hpp"
#include "kernels.hpp"

namespace burst {

#ifndef BURST_DQ_KB
#define BURST_DQ_KB 2   // 32-row key blocks per LDS tile of the dQ kernel
#endif
#ifndef BURST_DQ_BQ
#define BURST_DQ_BQ 256
#endif
constexpr int kDqBQ = BURST_DQ_BQ;   // query rows per work-group of the dQ kernel: 32 per wave

// lse in log2 units, with -inf mapped to +inf so that exp2(x - lse2) = 0 for a dead row
__device__ __forceinline__ float lse_to_log2(float lse) { return lse == -INFINITY ? INFINITY : lse * kLog2e; }

__device__ __forceinline__ void zero16(f32x16& x) {
#pragma unroll
  for (int v = 0; v < 16; ++v) x[v] = 0.f;
}

// ---------------------------------------------------------------------------------------------
template <int D, int KB, int NW>
__global__ __launch_bounds__(64 * NW, 512 / (64 * NW)) void step_bwd_dq_kernel(BwdParams p) {
  constexpr int BK = 32 * KB, DK = D / 16, DB = D / 32, BQ = 32 * NW, NT = 64 * NW;
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
  const int q_blk0 = p.q_runs.tile_of(bm.tile) * BQ, q_blk1 = min(q_blk0 + BQ, sq);
  const int q_w0 = q_blk0 + wave * 32, q_w1 = min(q_w0 + 32, sq);

  const int row = min(q_w0 + r, sq - 1);
  const int qpos = axis_position(axis_of<true>(mk), row);
  bf16x8 qreg[DK], doreg[DK];
  {
    const __bf16* qs = (const __bf16*)p.q.ptr + b * p.q.sb + hq * p.q.sh + (int64_t)row * p.q.ss + 8 * h;
    const __bf16* gs = (const __bf16*)p.d_o.ptr + b * p.d_o.sb + hq * p.d_o.sh + (int64_t)row * p.d_o.ss + 8 * h;
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) {
      qreg[ks] = *reinterpret_cast<const bf16x8*>(qs + ks * 16);
      doreg[ks] = *reinterpret_cast<const bf16x8*>(gs + ks * 16);
    }
  }
  const float lse2 = lse_to_log2(p.lse.ptr[b * p.lse.sb + hq * p.lse.sh + row]);
  const float dval = p.d.ptr[b * p.d.sb + hq * p.d.sh + row];
  const float c = p.scale * kLog2e;

  f32x16 dq[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db) zero16(dq[db]);

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
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
        f32x16 sd[2];   // S^T and dP^T of this key block: two independent accumulator chains
#pragma unroll
        for (int v = 0; v < 16; ++v) sd[1][v] = -dval;   // dP - D comes out of the GEMM: the lane owns the row, D is its constant
        gemm_rows_pair<PITCH, DK, kRowsAhead, true>(kt, vt, kb * 32, qreg, doreg, sd[0], sd[1], r, h);   // sd[0] starts from a literal zero
        if (cls == TILE_PARTIAL) mask_tile<true>(sd[0], mk, k0 + kb * 32, h, sk, qpos);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float pr = __builtin_amdgcn_exp2f(c * sd[0][v] - lse2);
          sd[0][v] = pr * sd[1][v];
        }
        bf16x8 ds[2] = {pack8(sd[0], 0), pack8(sd[0], 1)};
        gemm_cols<PITCH, DB, 2, kColsAhead>(kt, kb * 32, ds, dq, lane);
      }
    }
    if (more) walk.commit(smem + (buf ^ 1) * 2 * TILE, smem + (buf ^ 1) * 2 * TILE + TILE);
    __syncthreads();
    buf ^= 1;
    k0 = k0n;
    cls = cls_n;
    have = more;
  }

  if (q_w0 + r < sq) {
    float* dst = (float*)p.dq.ptr + b * p.dq.sb + (int64_t)(q_w0 + r) * p.dq.ss + hq * p.dq.sh;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float* q4 = dst + db * 32 + 8 * g + 4 * h;
        f32x4 x = {dq[db][4 * g] * p.scale, dq[db][4 * g + 1] * p.scale, dq[db][4 * g + 2] * p.scale,
                   dq[db][4 * g + 3] * p.scale};
        if (p.acc_dq) x += *reinterpret_cast<const f32x4*>(q4);
        *reinterpret_cast<f32x4*>(q4) = x;
      }
  }
}

// ---------------------------------------------------------------------------------------------
// Eight waves per work-group, two per SIMD, in two roles that share each block of 32 key rows:
//   P-wave  (waves 0-3): K rows in registers; S = Q K^T, P = exp2(..) -> bf16, hands P over through
//                        LDS, then dV^T += dO^T P.  Also stages the next query tile.
//   dS-wave (waves 4-7): V rows in registers; dP = dO V^T, then dS = P o (dP - D), dK^T += Q^T dS.
// Each role carries one 32 x D accumulator and one stationary operand, which is what lets two
// waves fit on a SIMD.  The dS-wave finishes a query tile one iteration late: in iteration t it
// first turns the dP it kept in registers and the P of tile t-1 into dS and dK, and only then
// computes dP of tile t, while the P-wave of the same SIMD runs S, softmax, dV of tile t and moves
// tile t+1 from global memory to LDS.  One barrier per tile: everything a wave reads in iteration
// t was written before the barrier that ended iteration t-1.
//   LDS: Q tiles and D rows in three slots (tile t-1 for dK, t for S, t+1 being staged), dO tiles,
//   lse rows and the P hand-over area in two.
template <int D, int BQ>
struct DkdvLds {
  static constexpr int PITCH = 2 * D + 16, TILE = BQ * PITCH, QBK = BQ / 32;
  static constexpr int Q_OFF = 0, DO_OFF = 3 * TILE, LSE_OFF = 5 * TILE, D_OFF = LSE_OFF + 2 * BQ * 4;
  static constexpr int P_OFF = D_OFF + 3 * BQ * 4;
  static constexpr int P_SLOT = 4 * QBK * 2 * 64;          // bf16x8 units: [pair][qb][half][lane]
  static constexpr int BYTES = P_OFF + 2 * P_SLOT * 16;
};

template <int D, int BQ, int ROLE>
__device__ __forceinline__ void dkdv_role(const BwdParams& p, char* smem, int b, int hk, int kv_tile, int pair) {
  constexpr int DK = D / 16, DB = D / 32, QBK = BQ / 32, BKV = 128, NT = 256;   // NT: staging threads
  using L = DkdvLds<D, BQ>;
  constexpr int PITCH = L::PITCH, TILE = L::TILE;
  float* lse_slots = reinterpret_cast<float*>(smem + L::LSE_OFF);
  float* d_slots = reinterpret_cast<float*>(smem + L::D_OFF);
  bf16x8* pbuf = reinterpret_cast<bf16x8*>(smem + L::P_OFF);

  const int group = p.q_heads / p.kv_heads;
  const int tid = threadIdx.x & 255, lane = tid & 63, r = lane & 31, h = lane >> 5;   // tid within the role
  const int sq = p.sq, sk = p.sk;
  const MaskDev mk = p.mask;
  const int k_blk0 = p.k_runs.tile_of(kv_tile) * BKV, k_blk1 = min(k_blk0 + BKV, sk);
  const int k_w0 = k_blk0 + pair * 32, k_w1 = min(k_w0 + 32, sk);

  const int krow = min(k_w0 + r, sk - 1);
  const int kpos = axis_position(axis_of<false>(mk), krow);
  bf16x8 xreg[DK];   // K rows (P-wave) or V rows (dS-wave) as the B operand
  {
    const TensorDev& src = ROLE == 0 ? p.k : p.v;
    const __bf16* s_ = (const __bf16*)src.ptr + b * src.sb + hk * src.sh + (int64_t)krow * src.ss + 8 * h;
#pragma unroll
    for (int ks = 0; ks < DK; ++ks) xreg[ks] = *reinterpret_cast<const bf16x8*>(s_ + ks * 16);
  }
  const float c = p.scale * kLog2e;

  f32x16 acc[DB];   // dV^T (P-wave) or dK^T (dS-wave)
#pragma unroll
  for (int db = 0; db < DB; ++db) zero16(acc[db]);

  // Position ranges of the work-group's 128 key rows and of this pair's 32: loop invariants of the
  // tile classification.
  int klo_blk, khi_blk, klo_w = 0, khi_w = 0;
  range_minmax<false>(mk, k_blk0, k_blk1, klo_blk, khi_blk);
  const bool has_keys = k_w0 < k_w1;
  if (has_keys) range_minmax<false>(mk, k_w0, k_w1, klo_w, khi_w);
  // Class of a whole query tile against this pair's 32 key rows (same for both waves of the pair).
  // A tile the mask only partly empties is computed whole with the per-element predicate.
  BlockClassifier<true> q_class;
  q_class.init(mk, klo_w, khi_w, sq, !has_keys);
  auto tile_class = [&](int q0) { return q_class(mk, q0, min(q0 + BQ, sq), q0 + BQ > sq); };

  // Walk over (query head of the group, query tile that can see the key block), flattened so the
  // pipeline runs across head boundaries.  The visible tiles of a head are one run of consecutive
  // tiles; inside it the cursor moves by adding constants, and only a head change recomputes addresses.
  const TileRun qr = visible_tiles<true, BQ>(mk, klo_blk, khi_blk, sq);
  bool c_valid = qr.len > 0;                       // the cursor is on an item
  int c_left = qr.len, c_head = 0;                 // cursor: tiles left in the head's run, head of the group
  int q0n = qr.start * BQ;                         // first row of the tile under the cursor

  TileStager<D, BQ, NT> stage_q, stage_do;         // P-wave only
  float stage_row = 0.f;   // threads [0, BQ): lse of a row; threads [BQ, 2*BQ): D of a row
  const char *q_tile = nullptr, *do_tile = nullptr;   // first row of the tile under the cursor
  const float* row_head = nullptr;                    // lse (threads < BQ) or D of the cursor's head
  const int64_t q_step = (int64_t)BQ * p.q.ss * 2, do_step = (int64_t)BQ * p.d_o.ss * 2;
  if (ROLE == 0) {
    stage_q.init(p.q.ss, tid);
    stage_do.init(p.d_o.ss, tid);
  }
  // which row vector this thread stages (selected once: a select between pointers inside the walk ends up
  // as an indexed array in scratch memory)
  const bool stages_lse = tid < BQ;
  const float* const rowvec_ptr = stages_lse ? p.lse.ptr : p.d.ptr;
  const int64_t rowvec_sb = stages_lse ? p.lse.sb : p.d.sb, rowvec_sh = stages_lse ? p.lse.sh : p.d.sh;
  auto point = [&]() {   // addresses of the tile under the cursor, from scratch
    if (ROLE != 0) return;
    const int hq = hk * group + c_head;
    q_tile = reinterpret_cast<const char*>((const __bf16*)p.q.ptr + b * p.q.sb + hq * p.q.sh + (int64_t)q0n * p.q.ss);
    do_tile = reinterpret_cast<const char*>((const __bf16*)p.d_o.ptr + b * p.d_o.sb + hq * p.d_o.sh +
                                            (int64_t)q0n * p.d_o.ss);
    row_head = rowvec_ptr + b * rowvec_sb + hq * rowvec_sh;
  };
  // Open flags of the query tiles against this work-group's key block (block-wise sparse mask)
  const uint8_t* open_flags = nullptr;
  if (mk.blk) {
    uint8_t* flags = reinterpret_cast<uint8_t*>(smem + L::BYTES);
    if (ROLE == 0) fill_open_flags<false, BQ>(mk, flags, k_blk0, sq, tid, NT);
    open_flags = flags;
    __syncthreads();
  }
  auto is_open = [&](int q0_) { return !open_flags || __builtin_amdgcn_readfirstlane(open_flags[q0_ / BQ]) != 0; };
  auto step = [&]() {   // cursor to the next tile of the walk
    if (--c_left > 0) {
      q0n += BQ;
      q_tile += q_step;
      do_tile += do_step;
    } else {
      ++c_head;
      c_left = qr.len;
      q0n = qr.start * BQ;
      if (c_head < group) point();
      else c_valid = false;
    }
  };
  auto advance = [&]() {   // cursor to the next item: the next tile that the block mask leaves open
    do step();
    while (c_valid && !is_open(q0n));
  };
  auto issue = [&]() {   // loads of the tile under the cursor
    if (ROLE != 0) return;
    if (q0n + BQ <= sq) {
      stage_q.load_at(q_tile);
      stage_do.load_at(do_tile);
    } else {   // last tile of a ragged chunk: row indices clamped per thread
      stage_q.load(reinterpret_cast<const __bf16*>(q_tile) - (int64_t)q0n * p.q.ss, p.q.ss, q0n, sq, tid);
      stage_do.load(reinterpret_cast<const __bf16*>(do_tile) - (int64_t)q0n * p.d_o.ss, p.d_o.ss, q0n, sq, tid);
    }
    // raw value only: converting here would wait for this load, and with it for the tile loads
    if (tid < 2 * BQ) stage_row = row_head[min(q0n + (tid & (BQ - 1)), sq - 1)];
  };
  auto commit = [&](int q_slot, int par) {   // q_slot: Q / D slot, par: dO / lse slot
    if (ROLE != 0) return;
    stage_q.store(smem + L::Q_OFF + q_slot * TILE);
    stage_do.store(smem + L::DO_OFF + par * TILE);
    if (tid < BQ) lse_slots[par * BQ + tid] = lse_to_log2(stage_row);
    else if (tid < 2 * BQ) d_slots[q_slot * BQ + tid - BQ] = -stage_row;   // -D: the dS-wave's dP accumulators start from it
  };

  wait_global_loads();
  int q0 = 0, cls = TILE_SKIP;   // first row and class of the tile in slot (qs_cur, par)
  if (c_valid) {
    point();
    if (!is_open(q0n)) advance();
  }
  bool have = c_valid;
  if (have) {
    issue();
    commit(0, 0);
    q0 = q0n;
    cls = tile_class(q0n);
    advance();
  }
  __syncthreads();
  int qs_prev = 2, qs_cur = 0, qs_next = 1, par = 0;
  int cls_prev = TILE_SKIP;
  f32x16 dp[QBK];   // dS-wave: dP of the tile staged one iteration ago
  // one iteration per item and a last one that only drains the dS-wave's lagging half
  for (;;) {
    const bool more = have && c_valid;
    int q0_next = 0, cls_next = TILE_SKIP;
    if (more) {
      issue();
      q0_next = q0n;
      cls_next = tile_class(q0n);
      advance();
    }
    const char* dot_ = smem + L::DO_OFF + par * TILE;
    if (ROLE == 0) {
      if (cls != TILE_SKIP) {
        const char* qt_ = smem + L::Q_OFF + qs_cur * TILE;
        const float* lse2 = lse_slots + par * BQ;
        bf16x8* pw = pbuf + par * L::P_SLOT;
        bf16x8 pk[2 * QBK];
        f32x16 s[QBK];
        gemm_rows<PITCH, QBK, DK, kRowsAhead, true>(qt_, 0, xreg, s, r, h);   // first MFMA of each block adds to a literal zero
#pragma unroll
        for (int qb = 0; qb < QBK; ++qb) {
          if (cls == TILE_PARTIAL) mask_tile<false>(s[qb], mk, q0 + qb * 32, h, sq, kpos);
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const f32x4 l4 = *reinterpret_cast<const f32x4*>(lse2 + qb * 32 + 8 * g + 4 * h);
#pragma unroll
            for (int j = 0; j < 4; ++j) s[qb][4 * g + j] = __builtin_amdgcn_exp2f(c * s[qb][4 * g + j] - l4[j]);
          }
          pk[2 * qb] = pack8(s[qb], 0);
          pk[2 * qb + 1] = pack8(s[qb], 1);
          pw[((pair * QBK + qb) * 2 + 0) * 64 + lane] = pk[2 * qb];
          pw[((pair * QBK + qb) * 2 + 1) * 64 + lane] = pk[2 * qb + 1];
        }
        gemm_cols<PITCH, DB, 2 * QBK, kColsAhead>(dot_, 0, pk, acc, lane);
      }
    } else {
      if (cls_prev != TILE_SKIP) {
        const char* qt_ = smem + L::Q_OFF + qs_prev * TILE;
        const bf16x8* pr_ = pbuf + (par ^ 1) * L::P_SLOT;
        bf16x8 dsp[2 * QBK];
#pragma unroll
        for (int qb = 0; qb < QBK; ++qb) {
          const bf16x8 p0 = pr_[((pair * QBK + qb) * 2 + 0) * 64 + lane];
          const bf16x8 p1 = pr_[((pair * QBK + qb) * 2 + 1) * 64 + lane];
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const float pr = (float)(v < 8 ? p0[v & 7] : p1[v & 7]);
            dp[qb][v] = pr * dp[qb][v];   // dp already holds dP - D
          }
          dsp[2 * qb] = pack8(dp[qb], 0);
          dsp[2 * qb + 1] = pack8(dp[qb], 1);
        }
        gemm_cols<PITCH, DB, 2 * QBK, kColsAhead>(qt_, 0, dsp, acc, lane);
      }
      if (cls != TILE_SKIP) {
        // dP - D: the accumulators start from -D of their query rows (registers run over rows here)
        const float* nd_ = d_slots + qs_cur * BQ;
#pragma unroll
        for (int qb = 0; qb < QBK; ++qb)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const f32x4 d4 = *reinterpret_cast<const f32x4*>(nd_ + qb * 32 + 8 * g + 4 * h);
#pragma unroll
            for (int j = 0; j < 4; ++j) dp[qb][4 * g + j] = d4[j];
          }
        gemm_rows<PITCH, QBK, DK, kRowsAhead>(dot_, 0, xreg, dp, r, h);
      }
    }
    if (more) commit(qs_next, par ^ 1);
    __syncthreads();
    const int t_ = qs_prev;
    qs_prev = qs_cur;
    qs_cur = qs_next;
    qs_next = t_;
    par ^= 1;
    cls_prev = cls;
    q0 = q0_next;
    cls = cls_next;
    if (!have) break;
    have = more;
  }

  if (k_w0 + r < sk) {
    const TensorDev& dst = ROLE == 0 ? p.dv : p.dk;
    const bool accumulate = ROLE == 0 ? p.acc_dv : p.acc_dk;
    const float mul = ROLE == 0 ? 1.f : p.scale;
    float* dp_ = (float*)dst.ptr + b * dst.sb + (int64_t)(k_w0 + r) * dst.ss + hk * dst.sh;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int off = db * 32 + 8 * g + 4 * h;
        f32x4 x = {acc[db][4 * g] * mul, acc[db][4 * g + 1] * mul, acc[db][4 * g + 2] * mul, acc[db][4 * g + 3] * mul};
        if (accumulate) x += *reinterpret_cast<const f32x4*>(dp_ + off);
        *reinterpret_cast<f32x4*>(dp_ + off) = x;
      }
  }
}

template <int D, int BQ>
__global__ __launch_bounds__(512, 1) void step_bwd_dkdv_kernel(BwdParams p) {
  extern __shared__ __attribute__((aligned(16))) char smem[];   // laid out by DkdvLds
  const BlockMap bm = map_block<false>(blockIdx.x, p.batch * p.kv_heads, 1, p.k_runs.total());
  if (!bm.valid) return;
  const int b = bm.key / p.kv_heads, hk = bm.key - b * p.kv_heads;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: the role branch is uniform
  // Two complete, separate instruction streams (same barrier count per tile in both), so that each
  // role is register-allocated on its own.
  if (wave < 4) dkdv_role<D, BQ, 0>(p, smem, b, hk, bm.tile, wave);
  else dkdv_role<D, BQ, 1>(p, smem, b, hk, bm.tile, wave - 4);
}

template <int D>
static hipError_t launch_bwd_t(BwdParams p, hipStream_t stream) {
  const int n_keys = p.batch * p.kv_heads, group = p.q_heads / p.kv_heads;
  hipError_t e = hipSuccess;
  if (p.dq.ptr) {
    constexpr int KB = BURST_DQ_KB;
    constexpr int LDS = 2 * 2 * 32 * KB * (2 * D + 16) + kMaxBlockCacheTiles;
    p.q_runs = nonempty_runs(p.mask, p.sq, p.sk, kDqBQ, true);
    // query tiles that see no key get no work-group: "=" must still leave zeros there
    if (!p.acc_dq && p.q_runs.total() < (p.sq + kDqBQ - 1) / kDqBQ) {
      e = launch_zero_tensor(p.dq, p.batch, p.sq, p.q_heads, p.head_dim, stream);
      if (e != hipSuccess) return e;
    }
    if (p.q_runs.total() > 0) {
      const int grid = mapped_grid(n_keys, group, p.q_runs.total());
      hipLaunchKernelGGL((step_bwd_dq_kernel<D, KB, kDqBQ / 32>), dim3(grid), dim3(2 * kDqBQ), LDS, stream, p);
      e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
  }
  if (p.dk.ptr) {
    constexpr int BQ = 64;
    constexpr int LDS = DkdvLds<D, BQ>::BYTES + kMaxBlockCacheTiles;
    p.k_runs = nonempty_runs(p.mask, p.sq, p.sk, 128, false);
    if (p.k_runs.total() < (p.sk + 127) / 128) {
      if (!p.acc_dk) e = launch_zero_tensor(p.dk, p.batch, p.sk, p.kv_heads, p.head_dim, stream);
      if (e == hipSuccess && !p.acc_dv) e = launch_zero_tensor(p.dv, p.batch, p.sk, p.kv_heads, p.head_dim, stream);
      if (e != hipSuccess) return e;
    }
    if (p.k_runs.total() > 0) {
      const int grid = mapped_grid(n_keys, 1, p.k_runs.total());
      hipLaunchKernelGGL((step_bwd_dkdv_kernel<D, BQ>), dim3(grid), dim3(512), LDS, stream, p);
      e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
  }
  return hipSuccess;
}

hipError_t launch_step_bwd(const BwdParams& p, hipStream_t stream) {
  if (p.head_dim == 128) return launch_bwd_t<128>(p, stream);
  return launch_bwd_t<64>(p, stream);
}

}  // namespace burst
