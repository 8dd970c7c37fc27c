/*
 * libburstattn -- sequence-level fusion of the language-modelling head and the loss function
 * (Sec. 3.3, Eq. 9, Alg. 3), the second single-device kernel family of the method.  Same library,
 * same conventions as burst_attn.h: every data pointer is DEVICE memory unless marked host, the
 * caller owns every buffer, the library allocates nothing, retains nothing, does not synchronise
 * and enqueues only on the given stream; all argument checks run on the host before any launch;
 * calls return BURST_OK (0) or a negative burst_status_t.
 *
 * For hidden states H_last (N x d), head weights W_head (v x d) and targets Y (N):
 *   Logits = H_last W_head^T;  Lse_i = log sum_j exp(Logits_ij);  loss_i = Lse_i - Logits_i,Y_i
 *   dLogits = grad_scale * (exp(Logits - Lse) - E),  E_ij = 1 iff j == Y_i
 *   dH = dLogits W_head;   dW = dLogits^T H_last
 * computed one sequence tile of tile_tokens rows at a time (the B_s of Alg. 3): the logits of the
 * tile are kept in the workspace between the forward sweep and the backward sweep, so nothing of
 * size N x v is ever stored and no logit is computed twice.  E is subtracted: the algorithm prints
 * it added, which is not the gradient of the loss it prints.  A target outside [0, v) marks an
 * ignored token: loss 0, no gradient.
 */
#ifndef BURST_LM_HEAD_H
#define BURST_LM_HEAD_H

#include <stdint.h>

#include "burst_attn.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  int64_t n_tokens;    /* N >= 0: rows of H_last on this device */
  int64_t d_model;     /* d: a positive multiple of 256 */
  int64_t vocab;       /* v >= 1 */
  int64_t tile_tokens; /* B_s: a positive multiple of 256; the workspace grows with it, the number
                          of passes over dW shrinks with it */
  float grad_scale;    /* gradient of the caller's scalar w.r.t. each token's loss (1: sum, 1/N: mean) */
  int32_t _pad;
} burst_lm_head_shape_t;

/* Bytes of workspace burst_lm_head_loss needs for this shape (n_tokens and grad_scale play no
 * part), or -1 for an invalid shape.  Host only. */
int64_t burst_lm_head_workspace_bytes(const burst_lm_head_shape_t* shape);

/*
 * Alg. 3, forward and backward in one call.
 *   h_last : bf16 [N][ld_h], w_head : bf16 [v][ld_w]  (row-major, leading dimensions in elements,
 *            multiples of 8, >= d; base pointers 16-byte aligned); y : int64 [N].  With N = 0
 *            the per-token pointers (h_last, y, loss, lse, d_h) are not looked at.
 *   loss   : fp32 [N], written.  lse : fp32 [N], written; may be NULL.
 *   d_h    : [N][ld_dh], BURST_F32 or BURST_BF16 (burst_dtype_t), OVERWRITTEN; NULL: not wanted.
 *   d_w    : fp32 [v][ld_dw]; accumulate_dw != 0 adds to its contents, else it is overwritten;
 *            NULL: not wanted.  With both gradients NULL only the forward sweep runs.
 *   workspace : at least burst_lm_head_workspace_bytes(shape) bytes, 256-byte aligned; contents
 *            on entry are irrelevant, contents on return are unspecified.  Calls that share a
 *            workspace must be ordered on one stream.
 * Non-finite inputs give non-finite outputs, possibly also in other rows of the same tile.
 * Errors: BURST_ERR_INVALID_ARG (null / misaligned pointers, bad sizes or leading dimensions,
 * workspace too small), BURST_ERR_UNSUPPORTED (d not a multiple of 256, sizes beyond 2^31 - 1
 * rows or a workspace row beyond 2^31 bytes), BURST_ERR_HIP (launch failed).
 */
int burst_lm_head_loss(const burst_lm_head_shape_t* shape, const void* h_last, int64_t ld_h,
                       const void* w_head, int64_t ld_w, const int64_t* y, float* loss, float* lse,
                       void* d_h, int32_t d_h_dtype, int64_t ld_dh, float* d_w, int64_t ld_dw,
                       int32_t accumulate_dw, void* workspace, int64_t workspace_bytes, void* hip_stream);

/*
 * The same computation for callers that cannot allocate device memory or hand over a workspace of
 * their own: code running under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Arguments, results and errors are those of burst_lm_head_loss without the workspace
 * pair: the scratch memory is an array built into the library's code object, 64 MiB per GPU
 * (burst_lm_head_static_scratch_bytes()), present from the moment the library is loaded until the
 * process ends.  The call allocates nothing and frees nothing, on the host or on the device.
 *   - A shape whose burst_lm_head_workspace_bytes() exceeds that size is refused with
 *     BURST_ERR_SCRATCH and nothing is enqueued (64 MiB holds e.g. tile_tokens = 256 with a
 *     32000-word vocabulary and d = 4096); choose a smaller tile_tokens or use burst_lm_head_loss.
 *   - The array used is that of the GPU that is current on the calling thread when the call is
 *     made; the stream must belong to that GPU.
 *   - Every call on a GPU shares that GPU's array, which keeps whatever the last call left in it
 *     (no call depends on its previous contents).  Calls that may overlap on one GPU -- different
 *     streams, or this entry point from two threads -- race on it: order them on one stream.
 */
int64_t burst_lm_head_static_scratch_bytes(void);
int burst_lm_head_loss_noalloc(const burst_lm_head_shape_t* shape, const void* h_last, int64_t ld_h,
                               const void* w_head, int64_t ld_w, const int64_t* y, float* loss, float* lse,
                               void* d_h, int32_t d_h_dtype, int64_t ld_dh, float* d_w, int64_t ld_dw,
                               int32_t accumulate_dw, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif
