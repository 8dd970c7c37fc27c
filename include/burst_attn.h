/*
 * libburstattn -- the per-device compute step of BurstAttention on AMD MI355X (gfx950).
 *
 * A device that holds a local query chunk Q_i meets one key/value chunk (K_j, V_j) per ring
 * step.  This library is that step: blockwise attention of Q_i against (K_j, V_j) forward and
 * backward, the online-softmax merge of step results into the running (O_i, Lse_i), and the
 * once-per-ring D = rowsum(dO o O).  The ring itself (who sends what to whom) is the caller's.
 *
 * Conventions common to every call
 *   - All tensor pointers are DEVICE pointers owned by the caller; the library never allocates,
 *     frees, retains or synchronises.  Work is enqueued on `hip_stream` (a hipStream_t passed as
 *     void*; NULL = the default stream) and the buffers must stay alive until it has run.
 *   - Structs are read on the host during the call and may be freed right after it returns.
 *   - Return value: BURST_OK (0) or a negative burst_status_t.  On any error other than
 *     BURST_ERR_HIP nothing has been enqueued.  burst_attn_last_hip_error() gives the raw HIP
 *     code of the last BURST_ERR_HIP on the calling thread.
 *   - Layouts: 4-D tensors are [batch, seq, heads, head_dim] with head_dim contiguous and the
 *     other strides given in ELEMENTS; row vectors (lse, D) are fp32 [batch, heads, seq] with seq
 *     contiguous and strides in elements.  4-D tensor pointers must be 16-byte aligned and their
 *     strides multiples of 8 elements (bf16) or 4 elements (fp32), stride_s at most 2^24 elements
 *     (BURST_ERR_UNSUPPORTED beyond); row vectors need only their natural 4-byte alignment.
 *     Tensors and row vectors that a call WRITES must not map two elements to one address: taking
 *     their dimensions of extent > 1 by increasing stride, every stride must cover the span of the
 *     dimensions before it (BURST_ERR_INVALID_ARG otherwise).  Inputs may overlap (a stride of 0
 *     broadcasts a head or a batch entry).
 *   - q, k, v, dO are bfloat16.  Accumulation, softmax, lse and D are fp32.
 *   - head_dim is 64 or 128; q_heads must be a multiple of kv_heads; query head h uses key/value
 *     head h / (q_heads / kv_heads).  sq and sk may be any non-negative number (ragged tails and
 *     empty chunks are handled).
 */
#ifndef BURST_ATTN_H
#define BURST_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  BURST_OK = 0,
  BURST_ERR_INVALID_ARG = -1, /* null pointer, bad size/stride/alignment, inconsistent mask */
  BURST_ERR_UNSUPPORTED = -2, /* valid request this build has no kernel for (dtype, head_dim) */
  BURST_ERR_HIP = -3,         /* a HIP call failed; see burst_attn_last_hip_error() */
  BURST_ERR_SCRATCH = -4      /* the shape needs more scratch than the library's built-in buffer holds */
} burst_status_t;

typedef enum { BURST_BF16 = 0, BURST_F32 = 1 } burst_dtype_t;

typedef enum { BURST_MASK_FULL = 0, BURST_MASK_CAUSAL = 1 } burst_mask_mode_t;

/* Problem size of one step: Q chunk of sq rows against a K/V chunk of sk rows. */
typedef struct {
  int32_t batch, q_heads, kv_heads, head_dim;
  int64_t sq, sk;
  float scale; /* softmax scale applied to Q K^T, normally 1/sqrt(head_dim) (Eq. 1, Eq. 4) */
} burst_shape_t;

typedef struct {
  void* ptr;       /* device */
  int32_t dtype;   /* burst_dtype_t */
  int32_t _pad;
  int64_t stride_b, stride_s, stride_h; /* elements */
} burst_tensor_t;

typedef struct {
  float* ptr;      /* device */
  int64_t stride_b, stride_h; /* elements */
} burst_rowvec_t;

/*
 * Which (query row, key row) pairs of the step are visible.  A chunk is q_nseg / k_nseg (>= 1)
 * pieces of equal length stored one after the other; local row r lies in piece s = r / seg_len
 * and has global token position
 *     seg_pos[0] + s * (seg_pos[1] - seg_pos[0]) + (r - s*seg_len) * pos_stride
 * (with one piece seg_pos[1] is not read).  The pieces must follow each other in position order
 * without overlapping -- seg_pos[1] - seg_pos[0] > (seg_len - 1) * pos_stride -- so that the
 * position grows with the local row (BURST_ERR_INVALID_ARG otherwise); with more than two pieces a
 * piece needs at least 32 rows (BURST_ERR_UNSUPPORTED below that).
 *   FULL  : every pair is visible.
 *   CAUSAL: a pair is visible iff position(q) >= position(k)  (Eq. 10: a token attends to itself
 *           and to everything before it); with window > 0 also position(q) - position(k) < window
 *           (sliding-window attention, the sparse pattern of Sec. 3.4: the token itself and the
 *           window - 1 positions before it).  window = 0: no window.  A window needs mode CAUSAL.
 * The zigzag split (Eq. 11-12) is two pieces (front, back); the contiguous split is one; the striped
 * split (Eq. 13-14) is one piece with pos_stride = G; the block-striped split of block-wise sparse
 * attention (Sec. 3.4: slice i of every block of N_blk tokens) is N / N_blk pieces of N_blk / G rows,
 * N_blk positions apart.
 * sq == q_nseg*q_seg_len and sk == k_nseg*k_seg_len must hold.
 * block_mask (device memory, or NULL for none) is a block-wise sparse mask of the step, the other
 * sparse pattern of Sec. 3.4, given on LOCAL rows: byte [q_row / q_block_rows][k_row / k_block_rows]
 * of a row-major array of ceil(sq / q_block_rows) rows with block_pitch bytes each; a pair is
 * visible iff the mode's predicate holds AND its byte is nonzero.  q_block_rows must be a positive
 * multiple of 256 and k_block_rows of 128 (the kernels' tiles then never straddle a block), and
 * block_pitch >= ceil(sk / k_block_rows); chunks of more than 262144 rows are UNSUPPORTED with a
 * block mask.  The caller owns the array; it must stay valid until the step has run on its stream.
 * Tiles whose block is closed are neither loaded nor computed.
 */
typedef struct {
  int32_t mode; /* burst_mask_mode_t */
  int32_t q_nseg, k_nseg, _pad;
  int64_t q_seg_pos[2], k_seg_pos[2];
  int64_t q_seg_len, k_seg_len;
  int64_t pos_stride;
  int64_t window;
  const uint8_t* block_mask; /* device, or NULL */
  int64_t q_block_rows, k_block_rows, block_pitch;
} burst_mask_t;

/*
 * Forward step (Eq. 5-6; forward algorithm).  For every (batch, query head):
 *   S = scale * Q K^T over the visible pairs, Lse_cur = rowwise log-sum-exp(S) (natural log),
 *   O_ij = exp(S - Lse_cur) V.
 * Outputs, each optional but at least one pair required:
 *   o_part (fp32 or bf16) / lse_part : the normalised step result (O_ij, Lse_cur); a query row
 *       with no visible key gets O = 0, Lse = -inf.
 *   o_acc (fp32) / lse_acc : running state, updated in place with the online-softmax merge
 *       Lse' = log(e^Lse_acc + e^Lse_cur); O_acc = e^(Lse_cur-Lse') O_ij + e^(Lse_acc-Lse') O_acc
 *       (initialise to O = 0, Lse = -inf before the first step).
 * k and v have kv_heads heads and sk rows; q and the outputs have q_heads heads and sq rows.
 */
int burst_attn_step_fwd(const burst_shape_t* shape, const burst_mask_t* mask,
                        const burst_tensor_t* q, const burst_tensor_t* k, const burst_tensor_t* v,
                        const burst_tensor_t* o_part, const burst_rowvec_t* lse_part,
                        const burst_tensor_t* o_acc, const burst_rowvec_t* lse_acc,
                        void* hip_stream);

/*
 * Online-softmax merge of a step result into the running state (forward algorithm):
 * (o_acc, lse_acc) <- (o_acc, lse_acc) (+) (o_part, lse_part), with exp(-inf) = 0 so that a row
 * whose two Lse are both -inf stays (0, -inf).  o_acc fp32 in/out; o_part fp32 or bf16.
 * o_out_cast, if not NULL, also receives the merged O as bf16 (for the last step).
 * Only shape->batch, q_heads, head_dim and sq are read.
 */
int burst_attn_lse_merge(const burst_shape_t* shape,
                         const burst_tensor_t* o_acc, const burst_rowvec_t* lse_acc,
                         const burst_tensor_t* o_part, const burst_rowvec_t* lse_part,
                         const burst_tensor_t* o_out_cast, void* hip_stream);

/*
 * D = rowsum(dO o O), once per ring (Alg. 2).  o is fp32 or bf16, d_o is bf16,
 * d_out fp32 [batch, q_heads, sq].  Only shape->batch, q_heads, head_dim and sq are read.
 */
int burst_attn_preprocess_bwd(const burst_shape_t* shape, const burst_tensor_t* o,
                              const burst_tensor_t* d_o, const burst_rowvec_t* d_out,
                              void* hip_stream);

/*
 * Backward step (the local step that Alg. 1 and Alg. 2 share, with the softmax scale restored):
 *   S = scale * Q K^T; P = exp(S - Lse); dV += P^T dO; dP = dO V^T; dS = P o (dP - D);
 *   dK += scale * dS^T Q; dQ += scale * dS K.
 * lse and d are the FINAL (all steps merged) Lse and D of the query rows.  dq [.., sq, q_heads, ..],
 * dk and dv [.., sk, kv_heads, ..] are fp32; with kv_heads < q_heads, dk and dv receive the sum
 * over the query heads of the group.  accumulate_flags: bit 0 dq, bit 1 dk, bit 2 dv; a set bit
 * means "+=" into the existing contents, a clear bit means overwrite.  Any of dq / dk / dv may be
 * NULL to skip it (dk and dv only together).  The same call serves both travel orders of the
 * backward ring: only which buffers the caller passes differs.
 */
#define BURST_ACC_DQ 1
#define BURST_ACC_DK 2
#define BURST_ACC_DV 4
int burst_attn_step_bwd(const burst_shape_t* shape, const burst_mask_t* mask,
                        const burst_tensor_t* q, const burst_tensor_t* k, const burst_tensor_t* v,
                        const burst_tensor_t* d_o, const burst_rowvec_t* lse, const burst_rowvec_t* d,
                        const burst_tensor_t* dq, const burst_tensor_t* dk, const burst_tensor_t* dv,
                        int32_t accumulate_flags, void* hip_stream);

/* Host helpers (no GPU involved). */

/* Mask of device dev_i's queries against shard_j's keys on a ring of G devices over N tokens.
 * zigzag (Eq. 11, 0-based): device i holds [i*P,(i+1)*P) and [N-(i+1)*P, N-i*P), P = N/(2G),
 * N must be a multiple of 2G.  contiguous: device i holds [i*N/G,(i+1)*N/G).  striped (Eq. 13):
 * device i holds tokens i + G*m.  causal = 0 gives a FULL mask with the same geometry.  The helpers
 * leave window = 0 and block_mask = NULL; set them afterwards for the sparse patterns. */
int burst_attn_fill_zigzag_mask(int32_t dev_i, int32_t shard_j, int32_t G, int64_t N, int32_t causal,
                                burst_mask_t* out);
int burst_attn_fill_contiguous_mask(int32_t dev_i, int32_t shard_j, int32_t G, int64_t N,
                                    int32_t causal, burst_mask_t* out);
int burst_attn_fill_striped_mask(int32_t dev_i, int32_t shard_j, int32_t G, int64_t N,
                                 int32_t causal, burst_mask_t* out);
/* Block-wise sparse attention (Sec. 3.4, "a strategy similar to striped-way workload balance"): the
 * sequence is cut into blocks of N_blk tokens (N a multiple of N_blk, N_blk a multiple of G) and device
 * i holds slice i, N_blk / G consecutive tokens, of every block.  Local row block b of N_blk / G rows is
 * then global block b on every device, so the step's block_mask is the global M_blk itself
 * (q_block_rows = k_block_rows = N_blk / G, which the kernels need to be a multiple of 256), and every
 * step of every device has the same number of visible pairs under a pure block pattern.  The same
 * holds for the striped split above, which deals token i + G*t of every block to device i and also
 * stays balanced under the causal rule and a window. */
int burst_attn_fill_block_striped_mask(int32_t dev_i, int32_t shard_j, int32_t G, int64_t N, int64_t N_blk,
                                       int32_t causal, burst_mask_t* out);

/* Number of visible (query row, key row) pairs of a step per (batch, head): the benchmark's work
 * unit (4*head_dim flop forward, 10*head_dim backward).  Returns -1 on an invalid mask.  The
 * count is that of the mode and window alone: block_mask lives in device memory and is not read
 * here. */
int64_t burst_attn_visible_pairs(const burst_mask_t* mask);

const char* burst_attn_status_string(int status);
int burst_attn_last_hip_error(void);
const char* burst_attn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* BURST_ATTN_H */
