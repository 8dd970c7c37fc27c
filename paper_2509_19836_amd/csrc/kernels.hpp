// Kernel parameter blocks and host-side launchers shared between the C-ABI layer and the kernels.
#pragma once
#include <vector>

#include "common.hpp"

namespace burst {

// Rows may keep a stale running maximum until one of the wave's rows grows by more than
// 2^kLazyLog2; exp2 arguments then stay <= kLazyLog2, far inside fp32 / bf16 range.
constexpr float kLazyLog2 = 6.0f;

// LDS operand prefetch distances: k-steps ahead for row-wise GEMMs, operands ahead for column-wise.
#ifndef BURST_ROWS_AHEAD
#define BURST_ROWS_AHEAD 2
#endif
#ifndef BURST_COLS_AHEAD
#define BURST_COLS_AHEAD 3
#endif
constexpr int kRowsAhead = BURST_ROWS_AHEAD, kColsAhead = BURST_COLS_AHEAD;

struct FwdParams {
  int32_t batch, q_heads, kv_heads, head_dim;
  int32_t sq, sk;
  float scale;
  MaskDev mask;
  TileRuns q_runs;      // query tiles with work (filled by the launcher)
  TensorDev q, k, v;
  TensorDev o_part;     // ptr == nullptr: not requested
  RowvecDev lse_part;
  TensorDev o_acc;      // ptr == nullptr: no fused merge
  RowvecDev lse_acc;
};

struct BwdParams {
  int32_t batch, q_heads, kv_heads, head_dim;
  int32_t sq, sk;
  float scale;
  MaskDev mask;
  TileRuns q_runs, k_runs;   // query / key tiles with work (filled by the launcher)
  TensorDev q, k, v, d_o;
  RowvecDev lse, d;
  TensorDev dq, dk, dv;   // fp32; ptr == nullptr: skip
  int32_t acc_dq, acc_dk, acc_dv;
};

struct MergeParams {
  int32_t batch, q_heads, head_dim, sq;
  TensorDev o_acc, o_part, o_out;   // o_out.ptr may be nullptr
  RowvecDev lse_acc, lse_part;
};

struct PreParams {
  int32_t batch, q_heads, head_dim, sq;
  TensorDev o, d_o;
  RowvecDev d;
};

// Runs of non-empty tiles along the query axis (each tile against the whole key chunk) or along
// the key axis (each tile against the whole query chunk); the same classification the kernels use.
inline TileRuns nonempty_runs(const MaskDev& mk, int sq, int sk, int tile_rows, bool q_axis) {
  const int rows = q_axis ? sq : sk;
  const int n = (rows + tile_rows - 1) / tile_rows;
  TileRuns tr{{0, 0}, {0, 0}};
  int nruns = 0;
  bool in_run = false;
  for (int t = 0; t < n; ++t) {
    const int r0 = t * tile_rows, r1 = r0 + tile_rows < rows ? r0 + tile_rows : rows;
    const int cls = q_axis ? classify(mk, r0, r1, 0, sk, false) : classify(mk, 0, sq, r0, r1, false);
    if (cls == TILE_SKIP) {
      in_run = false;
      continue;
    }
    if (!in_run) {
      if (nruns == 2) return TileRuns{{0, 0}, {n, 0}};   // more than two runs: launch every tile
      tr.start[nruns++] = t;
      in_run = true;
    }
    ++tr.len[nruns - 1];
  }
  return tr;
}

// ---------------------------------------------------------------------------------------------
// Chunked launches.  The work-groups that share an XCD's L2 (4 MiB) walk the streamed axis side by side,
// so a tile of it is fetched from HBM about once -- as long as the walk is short enough for them to stay
// together.  Over a walk of thousands of tiles they drift apart and each streams its own copy (at 131072-row
// chunks the dQ kernel fetched 107 GB per step instead of 32 GB).  A long streamed axis is therefore cut into
// row ranges of about chunk_rows() rows, one launch per range on the same stream, the stationary side's
// result accumulating in HBM from launch to launch (dQ; dK and dV; the forward kernel's running O and Lse,
// when the step result itself is not asked for).  Ranges of 32768 rows cost no time (16384: 1 %, 8192: 4 %).
// A range lies inside one piece of the axis or covers whole pieces, so it is again a chunk the mask
// descriptor can express.
int chunk_rows();   // the range length in force (set_chunk_rows; api.hip holds the value)

struct RowRange {
  int r0, r1;
};
// Ranges that cover [0, rows) of an axis of nseg pieces of seg_len rows; one range (no chunking) when the
// axis is short or a block mask's row blocks would be cut.
inline std::vector<RowRange> chunk_ranges(int nseg, int seg_len, int rows, int blk_rows) {
  const int target = chunk_rows();
  std::vector<RowRange> out;
  const bool cuts_blocks = blk_rows > 0 && ((nseg > 1 && seg_len % blk_rows != 0) || target % blk_rows != 0);
  if (rows <= 2 * target || cuts_blocks) {
    out.push_back({0, rows});
    return out;
  }
  if (nseg <= 1 || seg_len >= target) {   // ranges inside each piece
    const int pieces = nseg <= 1 ? 1 : nseg, len = nseg <= 1 ? rows : seg_len;
    for (int s = 0; s < pieces; ++s)
      for (int a = 0; a < len; a += target) out.push_back({s * len + a, s * len + (a + target < len ? a + target : len)});
  } else {                                // whole pieces per range
    const int per = target / seg_len > 0 ? target / seg_len : 1;
    for (int s = 0; s < nseg; s += per) out.push_back({s * seg_len, (s + per < nseg ? s + per : nseg) * seg_len});
  }
  return out;
}
// The mask of rows [r0, r1) of the query axis (Q_AXIS) or the key axis against the whole other axis.
template <bool Q_AXIS>
inline MaskDev sub_mask(const MaskDev& mk, int r0, int r1) {
  MaskDev m = mk;
  int32_t& nseg = Q_AXIS ? m.q_nseg : m.k_nseg;
  int32_t& seg_len = Q_AXIS ? m.q_seg_len : m.k_seg_len;
  int32_t& pos0 = Q_AXIS ? m.q_pos0 : m.k_pos0;
  int32_t& period = Q_AXIS ? m.q_period : m.k_period;
  if (nseg <= 1) {
    pos0 += r0 * m.pos_stride;
    seg_len = r1 - r0;
  } else {
    const int s0 = r0 / seg_len;
    if ((r1 - 1) / seg_len == s0) {   // inside piece s0
      pos0 += s0 * period + (r0 - s0 * seg_len) * m.pos_stride;
      nseg = 1;
      period = 0;
      seg_len = r1 - r0;
    } else {                          // pieces s0 .. (r1 / seg_len) - 1, whole
      pos0 += s0 * period;
      nseg = (r1 - r0) / seg_len;
    }
  }
  if (m.blk) m.blk += Q_AXIS ? (int64_t)(r0 / m.blk_q) * m.blk_pitch : (int64_t)(r0 / m.blk_k);
  return m;
}
inline void offset_rows(TensorDev& t, int r0) { t.ptr = (char*)t.ptr + (int64_t)r0 * t.ss * (t.is_f32 ? 4 : 2); }

// Fused LM head + cross-entropy (Alg. 3).  Sizes are validated on the host; the workspace is carved up there.
struct LmHeadParams {
  int32_t n_tokens, d_model, vocab, tile_tokens;
  int32_t v_pad;        // vocab rounded up to 256: row length of the two workspace matrices
  float grad_scale;
  const __bf16* h;      // [n_tokens][ld_h]
  const __bf16* w;      // [vocab][ld_w]
  int64_t ld_h, ld_w;
  const int64_t* y;
  float* loss;
  float* lse;           // may be nullptr
  void* dh;             // may be nullptr
  int32_t dh_is_f32;
  int64_t ld_dh;
  float* dw;            // may be nullptr
  int64_t ld_dw;
  int32_t acc_dw;
  float* logits;        // workspace [tile_tokens][v_pad]
  __bf16* dlogits;      // workspace [tile_tokens][v_pad]
  float2* part;         // workspace [v_pad / 128][tile_tokens]: (max, sum of exp) over 128 words
  __bf16* ht;           // workspace [d_model][tile_tokens]: the sequence tile's rows of h, transposed
};
int64_t lm_head_workspace_bytes(int64_t tile_tokens, int64_t vocab, int64_t d_model);
hipError_t launch_lm_head_loss(const LmHeadParams& p, hipStream_t stream);

hipError_t launch_step_fwd(const FwdParams& p, hipStream_t stream);
hipError_t launch_step_bwd(const BwdParams& p, hipStream_t stream);
// rows of the streamed axis per launch of a step kernel (longer axes are cut into several launches)
void set_chunk_rows(int rows);
int chunk_plan(const MaskDev& mk, int sq, int sk, bool query_axis, int max_ranges, int64_t* out);
hipError_t launch_lse_merge(const MergeParams& p, hipStream_t stream);
hipError_t launch_preprocess_bwd(const PreParams& p, hipStream_t stream);
// o_part = 0 / lse_part = -inf for a step with no key rows; zero-fill of fp32 gradients
hipError_t launch_fill_empty_fwd(const FwdParams& p, hipStream_t stream);
hipError_t launch_mfma_probe(float* sink, int iters, int random_operands, int64_t* flops, hipStream_t stream);
hipError_t launch_zero_tensor(const TensorDev& t, int32_t batch, int32_t rows, int32_t heads, int32_t head_dim,
                              hipStream_t stream);

}  // namespace burst
