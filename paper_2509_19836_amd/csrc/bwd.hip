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

#ifndef BURST_FOLD_SCALE
#define BURST_FOLD_SCALE 1   // dK/dV kernel: softmax scale folded into the K operand (see dkdv_role)
#endif
constexpr bool kFoldScale = BURST_FOLD_SCALE != 0;
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
// dK/dV kernel.  Eight waves per work-group, two per SIMD, in two roles that share each block of 32 key rows:
//   P-wave  (waves 0-3): K rows in registers; S = Q K^T, P = exp2(..) -> bf16, handed over through LDS,
//                        dV^T += dO^T P.  Also stages the query tiles.
//   dS-wave (waves 4-7): V rows in registers; dP = dO V^T - D, dS = P o dP, dK^T += Q^T dS.
// Each role carries one 32 x D accumulator and one stationary operand, which is what lets two waves fit on a
// SIMD; the two roles are separate instruction streams, register-allocated on their own.  Each stream is
// software-pipelined: the vector work of one unit of 32 query rows is sliced behind the MFMAs of the next
// unit, so both waves of a SIMD offer MFMAs to the matrix pipe nearly all the time:
//   P-wave,  unit u:  S(u+1) = Q K^T  with the slices of P(u) = exp2(c S(u) - lse) behind its MFMAs,
//                     then dV^T += dO^T P(u)  (its first MFMAs carry the last slices), P(u) -> LDS;
//   dS-wave, unit u:  dP(u+1) = dO V^T - D  with the slices of dS(u) = P(u) o dP(u) behind its MFMAs,
//                     then dK^T += Q^T dS(u).
// Query tiles are 64 rows (two units, a and b).  One barrier per tile, which the P-waves pass between the two
// units of tile t and the dS-waves before they start tile t: a dS-wave then works on dP of tile t and on dS / dK
// of unit b of tile t-1 and unit a of tile t, whose P the P-waves wrote before that barrier.  Q tiles live in
// four LDS slots (t-2 and t-1 for dK, t and t+1 for S, one of them being written), dO tiles, lse and -D rows in
// three, the P hand-over area in two per unit.  The P-waves stage the tiles.
template <int D>
struct DkdvLds {
  static constexpr int BQ = 64, PITCH = 2 * D + 16, TILE = BQ * PITCH;
  static constexpr int Q_OFF = 0, DO_OFF = 4 * TILE, LSE_OFF = 7 * TILE, D_OFF = LSE_OFF + 3 * BQ * 4;
  static constexpr int P_OFF = D_OFF + 3 * BQ * 4;
  static constexpr int P_UNIT = 4 * 2 * 64;                // bf16x8 per unit: [pair][half][lane]
  static constexpr int BYTES = P_OFF + 2 * 2 * P_UNIT * 16;   // [tile parity][unit]
};

template <int D, int ROLE>
__device__ __forceinline__ void dkdv_role(const BwdParams& p, char* smem, int b, int hk, int kv_tile, int pair) {
  constexpr int DK = D / 16, DB = D / 32, BQ = 64, BKV = 128, NT = 256;
  constexpr int PRE_R = kRowsAhead, PRE_C = kColsAhead;
  using L = DkdvLds<D>;
  constexpr int PITCH = L::PITCH, TILE = L::TILE;
  float* lse_slots = reinterpret_cast<float*>(smem + L::LSE_OFF);
  float* d_slots = reinterpret_cast<float*>(smem + L::D_OFF);
  bf16x8* pbuf = reinterpret_cast<bf16x8*>(smem + L::P_OFF);

  const int group = p.q_heads / p.kv_heads;
  const int tid = threadIdx.x & 255, lane = tid & 63, r = lane & 31, h = lane >> 5;
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
  if (ROLE == 0 && kFoldScale) {
    // K rows carry the factor scale * log2(e) (rounded to bf16 once per work-group) and the S accumulators start
    // from -lse: P = exp2 of the accumulator, no per-score multiply-add.  The extra rounding of K moves P by a
    // few 1e-3 relative, the size of the bf16 rounding P undergoes anyway before the dV product (the paper
    // fixes no precision); only this kernel does it: the forward kernel's Lse is held to 1e-3 absolute and
    // keeps the exact multiply-add.
#pragma unroll
    for (int ks = 0; ks < DK; ++ks)
#pragma unroll
      for (int e = 0; e < 8; ++e) xreg[ks][e] = (__bf16)((float)xreg[ks][e] * c);
  }

  f32x16 acc[DB];   // dV^T (P-wave) or dK^T (dS-wave)
#pragma unroll
  for (int db = 0; db < DB; ++db) zero16(acc[db]);

  int klo_blk, khi_blk, klo_w = 0, khi_w = 0;
  range_minmax<false>(mk, k_blk0, k_blk1, klo_blk, khi_blk);
  const bool has_keys = k_w0 < k_w1;
  if (has_keys) range_minmax<false>(mk, k_w0, k_w1, klo_w, khi_w);
  // A tile runs under the per-element predicate unless all of it is visible to this pair's keys; tiles that
  // are empty for this pair alone do too (their P is 0), so that the pipeline has no per-wave holes.
  BlockClassifier<true> q_class;
  q_class.init(mk, klo_w, khi_w, sq, !has_keys);
  auto tile_masked = [&](int q0_) { return q_class(mk, q0_, min(q0_ + BQ, sq), q0_ + BQ > sq) != TILE_FULL; };

  // Walk over (query head of the group, query tile that can see the key block) as one sequence; both roles
  // move the same cursor, only the P-waves load.
  const TileRun qr = visible_tiles<true, BQ>(mk, klo_blk, khi_blk, sq);
  bool c_valid = qr.len > 0;
  int c_left = qr.len, c_head = 0;
  int q0n = qr.start * BQ;

  TileStager<D, BQ, NT> stage_q, stage_do;   // P-wave only
  float stage_row = 0.f;
  const char *q_tile = nullptr, *do_tile = nullptr;
  const float* row_head = nullptr;
  const int64_t q_step = (int64_t)BQ * p.q.ss * 2, do_step = (int64_t)BQ * p.d_o.ss * 2;
  if (ROLE == 0) {
    stage_q.init(p.q.ss, tid);
    stage_do.init(p.d_o.ss, tid);
  }
  const bool stages_lse = tid < BQ;
  const float* const rowvec_ptr = stages_lse ? p.lse.ptr : p.d.ptr;
  const int64_t rowvec_sb = stages_lse ? p.lse.sb : p.d.sb, rowvec_sh = stages_lse ? p.lse.sh : p.d.sh;
  auto point = [&]() {
    if (ROLE != 0) return;
    const int hq = hk * group + c_head;
    q_tile = reinterpret_cast<const char*>((const __bf16*)p.q.ptr + b * p.q.sb + hq * p.q.sh + (int64_t)q0n * p.q.ss);
    do_tile = reinterpret_cast<const char*>((const __bf16*)p.d_o.ptr + b * p.d_o.sb + hq * p.d_o.sh +
                                            (int64_t)q0n * p.d_o.ss);
    row_head = rowvec_ptr + b * rowvec_sb + hq * rowvec_sh;
  };
  const uint8_t* open_flags = nullptr;
  if (mk.blk) {
    uint8_t* flags = reinterpret_cast<uint8_t*>(smem + L::BYTES);
    if (ROLE == 0) fill_open_flags<false, BQ>(mk, flags, k_blk0, sq, tid, NT);
    open_flags = flags;
    __syncthreads();
  }
  auto is_open = [&](int q0_) { return !open_flags || __builtin_amdgcn_readfirstlane(open_flags[q0_ / BQ]) != 0; };
  auto step = [&]() {
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
  auto advance = [&]() {
    do step();
    while (c_valid && !is_open(q0n));
  };
  auto issue = [&]() {
    if (ROLE != 0) return;
    if (q0n + BQ <= sq) {
      stage_q.load_at(q_tile);
      stage_do.load_at(do_tile);
    } else {
      stage_q.load(reinterpret_cast<const __bf16*>(q_tile) - (int64_t)q0n * p.q.ss, p.q.ss, q0n, sq, tid);
      stage_do.load(reinterpret_cast<const __bf16*>(do_tile) - (int64_t)q0n * p.d_o.ss, p.d_o.ss, q0n, sq, tid);
    }
    if (tid < 2 * BQ) stage_row = row_head[min(q0n + (tid & (BQ - 1)), sq - 1)];
  };
  auto commit = [&](int q_slot, int o_slot) {
    if (ROLE != 0) return;
    stage_q.store(smem + L::Q_OFF + q_slot * TILE);
    stage_do.store(smem + L::DO_OFF + o_slot * TILE);
    if (tid < BQ) lse_slots[o_slot * BQ + tid] = kFoldScale ? -lse_to_log2(stage_row) : lse_to_log2(stage_row);
    else if (tid < 2 * BQ) d_slots[o_slot * BQ + tid - BQ] = -stage_row;   // -D: the dP accumulators start from it
  };

  wait_global_loads();
  if (c_valid) {
    point();
    if (!is_open(q0n)) advance();
  }
  if (c_valid) {   // uniform over the work-group: both roles take the same number of barriers
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    // 16 per-row values of a unit (rows 8g + 4h + j of its 32) from an LDS row vector
    auto rows16 = [&](const float* vec, f32x16& out) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const f32x4 x = *reinterpret_cast<const f32x4*>(vec + 8 * g + 4 * h);
#pragma unroll
        for (int j = 0; j < 4; ++j) out[4 * g + j] = x[j];
      }
    };
    auto words_to_operand = [&](const uint32_t (&w)[8], int half) {
      const u32x4 x = {w[4 * half], w[4 * half + 1], w[4 * half + 2], w[4 * half + 3]};
      return __builtin_bit_cast(bf16x8, x);
    };
    // Values of a lane's 16 that go behind slot j of the first stream of a unit (DK MFMAs: values 0..11) and of
    // the first DB MFMAs of the second (values 12..15): the second stream's chunk 0 needs values 0..7 only.
    auto first_lo = [](int j) { return 12 * j / DK; };
    auto second_lo = [](int j) { return 12 + 4 * j / DB; };
    const int p_lane = pair * 2 * 64 + lane;   // this pair's place inside a unit of the hand-over area

    // cursor bookkeeping shared by the roles
    issue();
    commit(0, 0);
    int q0_cur = q0n;
    bool msk_cur = tile_masked(q0n);
    advance();
    bool more = c_valid;
    int q0_nxt = 0;
    bool msk_nxt = false;
    if (more) {
      issue();
      q0_nxt = q0n;
      msk_nxt = tile_masked(q0n);
      advance();
    }
    __syncthreads();   // tile 0 is in LDS
    int qs = 0, os = 0, par = 0;   // Q slot, dO / row slot and hand-over parity of the current tile

    if (ROLE == 0) {
      f32x16 s0, s1, l2;
      uint32_t pw[8];
      bf16x8 pk[2];
      // P(u) slices: values [v0, v1) of tile s
      auto p_vals = [&](f32x16& s, int v0, int v1) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          if (v < v0 || v >= v1) continue;
          s[v] = kFoldScale ? __builtin_amdgcn_exp2f(s[v]) : __builtin_amdgcn_exp2f(c * s[v] - l2[v]);
          if (v & 1) {
            const bf16x2 pr = {(__bf16)s[v - 1], (__bf16)s[v]};
            pw[v >> 1] = __builtin_bit_cast(uint32_t, pr);
          }
        }
      };
      // second half of a unit: dV^T += dO^T P with the last slices and the hand-over store behind its MFMAs
      auto dv_stream = [&](f32x16& s, int o_slot, int row0, int unit) {
        pk[0] = words_to_operand(pw, 0);
        pk[1] = pk[0];   // placeholder until the hooks below have produced values 8..15
        bf16x8* dst = pbuf + (par * 2 + unit) * L::P_UNIT + p_lane;
        cols_stream<PITCH, DB, 2, PRE_C>(smem + L::DO_OFF + o_slot * TILE, row0, pk, acc, lane, [&](int i) {
          if (i < DB) p_vals(s, second_lo(i), second_lo(i + 1));
          if (i == DB - 1) pk[1] = words_to_operand(pw, 1);
          if (i == DB) dst[0] = pk[0];
          if (i == DB + 1) dst[64] = pk[1];
        });
      };
      // S of the unit at rows row0 of the tile in (q_slot, o_slot) with hook(j) behind MFMA j
      auto s_stream = [&](f32x16& s, int q_slot, int o_slot, int row0, auto&& hook) {
        if (kFoldScale) {
          rows16(lse_slots + o_slot * BQ + row0, s);
          rows_stream<PITCH, DK, PRE_R, false>(smem + L::Q_OFF + q_slot * TILE, row0, xreg, s, r, h, hook);
        } else {
          rows_stream<PITCH, DK, PRE_R, true>(smem + L::Q_OFF + q_slot * TILE, row0, xreg, s, r, h, hook);
        }
      };
      s_stream(s0, 0, 0, 0, NoHook());
      for (;;) {
        const int qs1 = (qs + 1) & 3, os1 = os == 2 ? 0 : os + 1;
        // unit a of the tile (s0); S of unit b is produced meanwhile (s1)
        if (!kFoldScale) rows16(lse_slots + os * BQ, l2);
        if (msk_cur) mask_tile<false>(s0, mk, q0_cur, h, sq, kpos);
        s_stream(s1, qs, os, 32, [&](int j) { p_vals(s0, first_lo(j), first_lo(j + 1)); });
        dv_stream(s0, os, 0, 0);
        if (more) commit(qs1, os1);
        __syncthreads();
        const bool more2 = more && c_valid;
        int q0_n2 = 0;
        bool msk_n2 = false;
        if (more2) {
          issue();
          q0_n2 = q0n;
          msk_n2 = tile_masked(q0n);
          advance();
        }
        // unit b (s1); S of the next tile's unit a is produced meanwhile (s0)
        if (!kFoldScale) rows16(lse_slots + os * BQ + 32, l2);
        if (msk_cur) mask_tile<false>(s1, mk, q0_cur + 32, h, sq, kpos);
        if (more) {
          s_stream(s0, qs1, os1, 0, [&](int j) { p_vals(s1, first_lo(j), first_lo(j + 1)); });
        } else {
          p_vals(s1, 0, 12);
        }
        dv_stream(s1, os, 32, 1);
        if (!more) break;
        qs = qs1;
        os = os1;
        par ^= 1;
        q0_cur = q0_nxt;
        msk_cur = msk_nxt;
        q0_nxt = q0_n2;
        msk_nxt = msk_n2;
        more = more2;
      }
      __syncthreads();   // the last unit's P is in LDS
    } else {
      f32x16 dpa, dpb;   // dP - D of unit a / unit b
      uint32_t dw[8];
      bf16x8 dsk[2], p0, p1;
      // dS(u) slices: values [v0, v1) from the P words p0 / p1 and the dP - D tile
      auto ds_vals = [&](f32x16& dpv, int v0, int v1) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          if (v < v0 || v >= v1) continue;
          const float pr = (float)(v < 8 ? p0[v & 7] : p1[v & 7]);
          dpv[v] = pr * dpv[v];
          if (v & 1) {
            const bf16x2 x = {(__bf16)dpv[v - 1], (__bf16)dpv[v]};
            dw[v >> 1] = __builtin_bit_cast(uint32_t, x);
          }
        }
      };
      auto load_p = [&](int parity, int unit) {
        const bf16x8* src = pbuf + (parity * 2 + unit) * L::P_UNIT + p_lane;
        p0 = src[0];
        p1 = src[64];
      };
      // dP - D of the unit at rows row0 of the tile in o_slot, with dS slices of tile `dsv` behind its MFMAs
      auto dp_stream = [&](f32x16& dpv, int o_slot, int row0, f32x16* dsv) {
        rows16(d_slots + o_slot * BQ + row0, dpv);
        if (dsv) {
          rows_stream<PITCH, DK, PRE_R, false>(smem + L::DO_OFF + o_slot * TILE, row0, xreg, dpv, r, h,
                                                    [&](int j) { ds_vals(*dsv, first_lo(j), first_lo(j + 1)); });
        } else {
          rows_stream<PITCH, DK, PRE_R, false>(smem + L::DO_OFF + o_slot * TILE, row0, xreg, dpv, r, h);
        }
      };
      auto dk_stream = [&](f32x16& dsv, int q_slot, int row0) {
        dsk[0] = words_to_operand(dw, 0);
        dsk[1] = dsk[0];
        cols_stream<PITCH, DB, 2, PRE_C>(smem + L::Q_OFF + q_slot * TILE, row0, dsk, acc, lane, [&](int i) {
          if (i < DB) ds_vals(dsv, second_lo(i), second_lo(i + 1));
          if (i == DB - 1) dsk[1] = words_to_operand(dw, 1);
        });
      };
      bool first = true;
      for (;;) {
        __syncthreads();   // P of unit a of this tile and of unit b of the previous one is in LDS
        const int qs1 = (qs + 1) & 3, os1 = os == 2 ? 0 : os + 1;
        const bool more2 = more && c_valid;
        if (more2) advance();
        if (!first) {
          load_p(par ^ 1, 1);
          dp_stream(dpa, os, 0, &dpb);
          dk_stream(dpb, (qs + 3) & 3, 32);
        } else {
          dp_stream(dpa, os, 0, nullptr);
        }
        load_p(par, 0);
        dp_stream(dpb, os, 32, &dpa);
        dk_stream(dpa, qs, 0);
        first = false;
        if (!more) break;
        qs = qs1;
        os = os1;
        par ^= 1;
        more = more2;
      }
      __syncthreads();
      load_p(par, 1);
      ds_vals(dpb, 0, 12);
      dk_stream(dpb, qs, 32);
    }
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

template <int D>
__global__ __launch_bounds__(512, 1) void step_bwd_dkdv_kernel(BwdParams p) {
  extern __shared__ __attribute__((aligned(16))) char smem[];   // laid out by DkdvLds
  const BlockMap bm = map_block<false>(blockIdx.x, p.batch * p.kv_heads, 1, p.k_runs.total());
  if (!bm.valid) return;
  const int b = bm.key / p.kv_heads, hk = bm.key - b * p.kv_heads;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (wave < 4) dkdv_role<D, 0>(p, smem, b, hk, bm.tile, wave);
  else dkdv_role<D, 1>(p, smem, b, hk, bm.tile, wave - 4);
}


template <int D>
static hipError_t launch_dq_t(BwdParams p, hipStream_t stream) {
  const int n_keys = p.batch * p.kv_heads, group = p.q_heads / p.kv_heads;
  constexpr int KB = BURST_DQ_KB;
  constexpr int LDS = 2 * 2 * 32 * KB * (2 * D + 16) + kMaxBlockCacheTiles;
  p.q_runs = nonempty_runs(p.mask, p.sq, p.sk, kDqBQ, true);
  // query tiles that see no key get no work-group: "=" must still leave zeros there
  if (!p.acc_dq && p.q_runs.total() < (p.sq + kDqBQ - 1) / kDqBQ) {
    hipError_t e = launch_zero_tensor(p.dq, p.batch, p.sq, p.q_heads, p.head_dim, stream);
    if (e != hipSuccess) return e;
  }
  if (p.q_runs.total() == 0) return hipSuccess;
  const int grid = mapped_grid(n_keys, group, p.q_runs.total());
  hipLaunchKernelGGL((step_bwd_dq_kernel<D, KB, kDqBQ / 32>), dim3(grid), dim3(2 * kDqBQ), LDS, stream, p);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_dkdv_t(BwdParams p, hipStream_t stream) {
  const int n_keys = p.batch * p.kv_heads;
  constexpr int LDS = DkdvLds<D>::BYTES + kMaxBlockCacheTiles;
  static_assert(LDS <= 160 * 1024, "LDS of a CU");
  p.k_runs = nonempty_runs(p.mask, p.sq, p.sk, 128, false);
  if (p.k_runs.total() < (p.sk + 127) / 128) {
    hipError_t e = hipSuccess;
    if (!p.acc_dk) e = launch_zero_tensor(p.dk, p.batch, p.sk, p.kv_heads, p.head_dim, stream);
    if (e == hipSuccess && !p.acc_dv) e = launch_zero_tensor(p.dv, p.batch, p.sk, p.kv_heads, p.head_dim, stream);
    if (e != hipSuccess) return e;
  }
  if (p.k_runs.total() == 0) return hipSuccess;
  const int grid = mapped_grid(n_keys, 1, p.k_runs.total());
  hipLaunchKernelGGL((step_bwd_dkdv_kernel<D>), dim3(grid), dim3(512), LDS, stream, p);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_bwd_t(const BwdParams& p0, hipStream_t stream) {
  hipError_t e = hipSuccess;
  if (p0.dq.ptr) {   // the dQ kernel streams the key axis
    const std::vector<RowRange> ranges = chunk_ranges(p0.mask.k_nseg, p0.mask.k_seg_len, p0.sk, p0.mask.blk ? p0.mask.blk_k : 0);
    bool first = true;
    for (const RowRange& rg : ranges) {
      BwdParams p = p0;
      if (ranges.size() > 1) {
        p.mask = sub_mask<false>(p0.mask, rg.r0, rg.r1);
        p.sk = rg.r1 - rg.r0;
        offset_rows(p.k, rg.r0);
        offset_rows(p.v, rg.r0);
        if (!first) p.acc_dq = 1;
      }
      e = launch_dq_t<D>(p, stream);
      if (e != hipSuccess) return e;
      first = false;
    }
  }
  if (p0.dk.ptr) {   // the dK/dV kernel streams the query axis
    const std::vector<RowRange> ranges = chunk_ranges(p0.mask.q_nseg, p0.mask.q_seg_len, p0.sq, p0.mask.blk ? p0.mask.blk_q : 0);
    bool first = true;
    for (const RowRange& rg : ranges) {
      BwdParams p = p0;
      if (ranges.size() > 1) {
        p.mask = sub_mask<true>(p0.mask, rg.r0, rg.r1);
        p.sq = rg.r1 - rg.r0;
        offset_rows(p.q, rg.r0);
        offset_rows(p.d_o, rg.r0);
        p.lse.ptr += rg.r0;
        p.d.ptr += rg.r0;
        if (!first) p.acc_dk = p.acc_dv = 1;
      }
      e = launch_dkdv_t<D>(p, stream);
      if (e != hipSuccess) return e;
      first = false;
    }
  }
  return hipSuccess;
}

// Host view of the launcher's plan for tests: the ranges the query axis (dK/dV kernel) or the key axis (dQ
// kernel) of a step is cut into, each with the piece description of its sub-mask and the block-mask offset.
int chunk_plan(const MaskDev& mk, int sq, int sk, bool query_axis, int max_ranges, int64_t* out) {
  const std::vector<RowRange> ranges = query_axis ? chunk_ranges(mk.q_nseg, mk.q_seg_len, sq, mk.blk ? mk.blk_q : 0)
                                                  : chunk_ranges(mk.k_nseg, mk.k_seg_len, sk, mk.blk ? mk.blk_k : 0);
  int n = 0;
  for (const RowRange& rg : ranges) {
    if (n == max_ranges) break;
    const MaskDev m = ranges.size() > 1 ? (query_axis ? sub_mask<true>(mk, rg.r0, rg.r1) : sub_mask<false>(mk, rg.r0, rg.r1)) : mk;
    int64_t* o = out + 7 * n++;
    o[0] = rg.r0;
    o[1] = rg.r1;
    o[2] = query_axis ? m.q_nseg : m.k_nseg;
    o[3] = query_axis ? m.q_seg_len : m.k_seg_len;
    o[4] = query_axis ? m.q_pos0 : m.k_pos0;
    o[5] = query_axis ? m.q_period : m.k_period;
    o[6] = m.blk ? (int64_t)(m.blk - mk.blk) : 0;
  }
  return (int)ranges.size();
}

hipError_t launch_step_bwd(const BwdParams& p, hipStream_t stream) {
  if (p.head_dim == 128) return launch_bwd_t<128>(p, stream);
  return launch_bwd_t<64>(p, stream);
}

}  // namespace burst
