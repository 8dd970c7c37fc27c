// Kernel parameter blocks and host-side launchers shared between the C-ABI layer and the kernels.
#pragma once
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
// rows of the streamed axis per launch of a backward kernel (longer axes are cut into several launches)
void set_bwd_chunk_rows(int rows);
int bwd_chunk_plan(const MaskDev& mk, int sq, int sk, bool query_axis, int max_ranges, int64_t* out);
hipError_t launch_lse_merge(const MergeParams& p, hipStream_t stream);
hipError_t launch_preprocess_bwd(const PreParams& p, hipStream_t stream);
// o_part = 0 / lse_part = -inf for a step with no key rows; zero-fill of fp32 gradients
hipError_t launch_fill_empty_fwd(const FwdParams& p, hipStream_t stream);
hipError_t launch_mfma_probe(float* sink, int iters, int random_operands, int64_t* flops, hipStream_t stream);
hipError_t launch_zero_tensor(const TensorDev& t, int32_t batch, int32_t rows, int32_t heads, int32_t head_dim,
                              hipStream_t stream);

}  // namespace burst
