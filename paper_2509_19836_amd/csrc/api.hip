// C-ABI layer of libburstattn: argument validation, host-side mask helpers and kernel dispatch.
// Every check runs on the host before anything is enqueued.
#include <hip/hip_runtime.h>
#include <algorithm>
#include <cmath>
#include <cstring>
#include <atomic>
#include <mutex>

#include "../../include/burst_attn.h"
#include "../../include/burst_attn_diag.h"
#include "../../include/burst_lm_head.h"
#include "kernels.hpp"

namespace burst {
// Rows of a streamed axis per launch of a step kernel (kernels.hpp: chunk_ranges); process-wide.
static std::atomic<int> g_chunk_rows{32768};
int chunk_rows() { return g_chunk_rows.load(); }
void set_chunk_rows(int rows) { g_chunk_rows.store(rows < 256 ? 256 : rows); }
}  // namespace burst

using namespace burst;

namespace {

thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e) {
  g_last_hip_error = (int)e;
  return BURST_ERR_HIP;
}

constexpr int64_t kMaxRows = (int64_t)1 << 30;
constexpr int64_t kMaxPos = ((int64_t)1 << 31) - 1;
constexpr int64_t kMaxRowStride = (int64_t)1 << 24;   // elements between consecutive sequence rows

int check_shape(const burst_shape_t* s) {
  if (!s) return BURST_ERR_INVALID_ARG;
  if (s->batch < 1 || s->q_heads < 1 || s->kv_heads < 1 || s->head_dim < 1) return BURST_ERR_INVALID_ARG;
  if (s->q_heads % s->kv_heads != 0) return BURST_ERR_INVALID_ARG;
  if (s->sq < 0 || s->sk < 0 || s->sq > kMaxRows || s->sk > kMaxRows) return BURST_ERR_INVALID_ARG;
  if (!(s->scale > 0.f) || !std::isfinite(s->scale)) return BURST_ERR_INVALID_ARG;
  if (s->head_dim != 64 && s->head_dim != 128) return BURST_ERR_UNSUPPORTED;
  return BURST_OK;
}

int check_tensor(const burst_tensor_t* t, int want_dtype_mask /* bit0 bf16 ok, bit1 f32 ok */, TensorDev* out) {
  if (!t || !t->ptr) return BURST_ERR_INVALID_ARG;
  if (t->dtype != BURST_BF16 && t->dtype != BURST_F32) return BURST_ERR_INVALID_ARG;
  if (!((want_dtype_mask >> t->dtype) & 1)) return BURST_ERR_UNSUPPORTED;
  if (((uintptr_t)t->ptr) & 15) return BURST_ERR_INVALID_ARG;
  const int64_t unit = (t->dtype == BURST_BF16) ? 8 : 4;
  if (t->stride_b % unit || t->stride_s % unit || t->stride_h % unit) return BURST_ERR_INVALID_ARG;
  if (t->stride_b < 0 || t->stride_s < 0 || t->stride_h < 0) return BURST_ERR_INVALID_ARG;
  if (t->stride_s > kMaxRowStride) return BURST_ERR_UNSUPPORTED;   // the tile stagers keep 32-bit byte offsets inside a tile
  out->ptr = t->ptr;
  out->sb = t->stride_b;
  out->ss = t->stride_s;
  out->sh = t->stride_h;
  out->is_f32 = (t->dtype == BURST_F32);
  return BURST_OK;
}

// An output tensor must not map two of its elements to one address: work-groups that own different
// rows or heads would then write (or read-modify-write) the same memory.  Sufficient test: walking the
// dimensions of extent > 1 by increasing stride, each stride covers the span of the ones before it.
// Inputs may overlap (a stride of 0 broadcasts a head or a batch entry), so they are not tested.
int check_no_overlap(const TensorDev& t, int64_t batch, int64_t rows, int64_t heads, int64_t head_dim) {
  int64_t stride[3] = {t.sh, t.ss, t.sb}, extent[3] = {heads, rows, batch};
  for (int a = 0; a < 3; ++a)
    for (int b = a + 1; b < 3; ++b)
      if (stride[b] < stride[a]) {
        std::swap(stride[a], stride[b]);
        std::swap(extent[a], extent[b]);
      }
  int64_t span = head_dim;   // elements covered so far, innermost dimension first
  for (int a = 0; a < 3; ++a) {
    if (extent[a] <= 1) continue;
    if (stride[a] < span) return BURST_ERR_INVALID_ARG;
    span = stride[a] * (extent[a] - 1) + span;
  }
  return BURST_OK;
}

int check_rowvec_no_overlap(const RowvecDev& t, int64_t batch, int64_t heads, int64_t rows) {
  int64_t lo = t.sh, lo_n = heads, hi = t.sb, hi_n = batch;
  if (hi < lo) {
    std::swap(lo, hi);
    std::swap(lo_n, hi_n);
  }
  int64_t span = rows;
  if (lo_n > 1) {
    if (lo < span) return BURST_ERR_INVALID_ARG;
    span = lo * (lo_n - 1) + span;
  }
  if (hi_n > 1 && hi < span) return BURST_ERR_INVALID_ARG;
  return BURST_OK;
}

int check_rowvec(const burst_rowvec_t* t, RowvecDev* out) {
  if (!t || !t->ptr) return BURST_ERR_INVALID_ARG;
  if (((uintptr_t)t->ptr) & 3) return BURST_ERR_INVALID_ARG;
  if (t->stride_b < 0 || t->stride_h < 0) return BURST_ERR_INVALID_ARG;
  out->ptr = t->ptr;
  out->sb = t->stride_b;
  out->sh = t->stride_h;
  return BURST_OK;
}

// One axis of a burst_mask_t: nseg pieces of seg_len rows, piece s starting at
// seg_pos[0] + s * (seg_pos[1] - seg_pos[0]); the pieces must follow each other in position order
// without overlapping, so that the position grows with the local row.
int check_axis(int32_t nseg, int64_t seg_len, const int64_t seg_pos[2], int64_t stride, int64_t rows, int32_t* pos0,
               int32_t* period) {
  if (nseg < 1 || seg_len < 0) return BURST_ERR_INVALID_ARG;
  if (seg_len > kMaxRows || nseg > kMaxRows) return BURST_ERR_UNSUPPORTED;
  if (seg_len * nseg != rows) return BURST_ERR_INVALID_ARG;
  if (seg_pos[0] < 0) return BURST_ERR_INVALID_ARG;
  if (seg_pos[0] > kMaxPos) return BURST_ERR_UNSUPPORTED;
  int64_t per = 0;
  if (nseg > 1) {
    per = seg_pos[1] - seg_pos[0];
    if (seg_pos[1] < 0 || per <= 0) return BURST_ERR_INVALID_ARG;             // pieces in increasing position order
    if (seg_len > 0 && per <= (seg_len - 1) * stride) return BURST_ERR_INVALID_ARG;   // ... and not overlapping
    if (per > kMaxPos) return BURST_ERR_UNSUPPORTED;
    if (nseg > 2 && seg_len < 32) return BURST_ERR_UNSUPPORTED;   // a 32-row register tile may span two pieces, not three
  }
  // position just past the last row
  if (seg_pos[0] + (int64_t)(nseg - 1) * per + seg_len * stride > kMaxPos) return BURST_ERR_UNSUPPORTED;
  *pos0 = (int32_t)seg_pos[0];
  *period = (int32_t)per;
  return BURST_OK;
}

int check_mask(const burst_mask_t* m, int64_t sq, int64_t sk, MaskDev* out) {
  std::memset(out, 0, sizeof(*out));
  if (!m) {  // no mask given: everything visible
    out->causal = 0;
    out->q_nseg = out->k_nseg = 1;
    out->q_seg_len = (int32_t)sq;
    out->k_seg_len = (int32_t)sk;
    out->pos_stride = 1;
    out->window = kNoWindow;
    return BURST_OK;
  }
  if (m->mode != BURST_MASK_FULL && m->mode != BURST_MASK_CAUSAL) return BURST_ERR_INVALID_ARG;
  if (m->pos_stride < 1) return BURST_ERR_INVALID_ARG;
  // bounded before it is multiplied (the products then stay far inside int64)
  if (m->pos_stride > kMaxPos) return BURST_ERR_UNSUPPORTED;
  if (m->window < 0 || (m->window > 0 && m->mode != BURST_MASK_CAUSAL)) return BURST_ERR_INVALID_ARG;
  int st = check_axis(m->q_nseg, m->q_seg_len, m->q_seg_pos, m->pos_stride, sq, &out->q_pos0, &out->q_period);
  if (st != BURST_OK) return st;
  st = check_axis(m->k_nseg, m->k_seg_len, m->k_seg_pos, m->pos_stride, sk, &out->k_pos0, &out->k_period);
  if (st != BURST_OK) return st;
  out->causal = (m->mode == BURST_MASK_CAUSAL);
  out->q_nseg = m->q_nseg;
  out->k_nseg = m->k_nseg;
  out->q_seg_len = (int32_t)m->q_seg_len;
  out->k_seg_len = (int32_t)m->k_seg_len;
  out->pos_stride = (int32_t)m->pos_stride;
  out->window = (m->window == 0 || m->window >= kNoWindow) ? kNoWindow : (int32_t)m->window;
  if (m->block_mask) {
    if (m->q_block_rows <= 0 || m->q_block_rows % 256 != 0 || m->k_block_rows <= 0 || m->k_block_rows % 128 != 0)
      return BURST_ERR_INVALID_ARG;
    if (m->block_pitch < (sk + m->k_block_rows - 1) / m->k_block_rows || m->block_pitch > INT32_MAX)
      return BURST_ERR_INVALID_ARG;
    // the kernels cache one open flag per 64-row tile of the walked axis in LDS
    if (sq > 64ll * kMaxBlockCacheTiles || sk > 64ll * kMaxBlockCacheTiles) return BURST_ERR_UNSUPPORTED;
    out->blk = m->block_mask;
    out->blk_q = (int32_t)(m->q_block_rows > INT32_MAX ? INT32_MAX - 255 : m->q_block_rows);
    out->blk_k = (int32_t)(m->k_block_rows > INT32_MAX ? INT32_MAX - 127 : m->k_block_rows);
    out->blk_pitch = (int32_t)m->block_pitch;
  }
  return BURST_OK;
}

// Scratch memory of burst_lm_head_loss_noalloc: one array per GPU, part of the loaded code object,
// so the entry point never allocates.  The array's name is only a host-side handle: kernels get the
// device address that hipGetSymbolAddress reports for the current device, looked up once per device.
constexpr int64_t kStaticScratchBytes = (int64_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch_of_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e);
  if (dev < 0 || dev >= kMaxDevices) return BURST_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));   // the address on the current device
    if (e != hipSuccess || !ptr) return hip_fail(e == hipSuccess ? hipErrorInvalidSymbol : e);
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return BURST_OK;
}

#define BURST_TRY(expr)            \
  do {                             \
    int _st = (expr);              \
    if (_st != BURST_OK) return _st; \
  } while (0)

}  // namespace

extern "C" {

int burst_attn_step_fwd(const burst_shape_t* shape, const burst_mask_t* mask, const burst_tensor_t* q,
                        const burst_tensor_t* k, const burst_tensor_t* v, const burst_tensor_t* o_part,
                        const burst_rowvec_t* lse_part, const burst_tensor_t* o_acc,
                        const burst_rowvec_t* lse_acc, void* hip_stream) {
  BURST_TRY(check_shape(shape));
  FwdParams p;
  std::memset(&p, 0, sizeof(p));
  BURST_TRY(check_mask(mask, shape->sq, shape->sk, &p.mask));
  BURST_TRY(check_tensor(q, 1, &p.q));
  BURST_TRY(check_tensor(k, 1, &p.k));
  BURST_TRY(check_tensor(v, 1, &p.v));
  const bool want_part = o_part || lse_part, want_acc = o_acc || lse_acc;
  if (!want_part && !want_acc) return BURST_ERR_INVALID_ARG;
  if (want_part) {
    BURST_TRY(check_tensor(o_part, 3, &p.o_part));
    BURST_TRY(check_rowvec(lse_part, &p.lse_part));
    BURST_TRY(check_no_overlap(p.o_part, shape->batch, shape->sq, shape->q_heads, shape->head_dim));
    BURST_TRY(check_rowvec_no_overlap(p.lse_part, shape->batch, shape->q_heads, shape->sq));
  }
  if (want_acc) {
    BURST_TRY(check_tensor(o_acc, 2, &p.o_acc));
    BURST_TRY(check_rowvec(lse_acc, &p.lse_acc));
    BURST_TRY(check_no_overlap(p.o_acc, shape->batch, shape->sq, shape->q_heads, shape->head_dim));
    BURST_TRY(check_rowvec_no_overlap(p.lse_acc, shape->batch, shape->q_heads, shape->sq));
  }
  p.batch = shape->batch;
  p.q_heads = shape->q_heads;
  p.kv_heads = shape->kv_heads;
  p.head_dim = shape->head_dim;
  p.sq = (int32_t)shape->sq;
  p.sk = (int32_t)shape->sk;
  p.scale = shape->scale;
  if (p.sq == 0) return BURST_OK;
  hipStream_t stream = (hipStream_t)hip_stream;
  hipError_t e;
  if (p.sk == 0) {  // no key: the step result is (0, -inf) and the running state is unchanged
    if (!want_part) return BURST_OK;
    e = launch_fill_empty_fwd(p, stream);
  } else {
    e = launch_step_fwd(p, stream);
  }
  return e == hipSuccess ? BURST_OK : hip_fail(e);
}

int burst_attn_lse_merge(const burst_shape_t* shape, const burst_tensor_t* o_acc, const burst_rowvec_t* lse_acc,
                         const burst_tensor_t* o_part, const burst_rowvec_t* lse_part,
                         const burst_tensor_t* o_out_cast, void* hip_stream) {
  BURST_TRY(check_shape(shape));
  MergeParams p;
  std::memset(&p, 0, sizeof(p));
  BURST_TRY(check_tensor(o_acc, 2, &p.o_acc));
  BURST_TRY(check_rowvec(lse_acc, &p.lse_acc));
  BURST_TRY(check_tensor(o_part, 3, &p.o_part));
  BURST_TRY(check_rowvec(lse_part, &p.lse_part));
  if (o_out_cast) BURST_TRY(check_tensor(o_out_cast, 1, &p.o_out));
  BURST_TRY(check_no_overlap(p.o_acc, shape->batch, shape->sq, shape->q_heads, shape->head_dim));
  BURST_TRY(check_rowvec_no_overlap(p.lse_acc, shape->batch, shape->q_heads, shape->sq));
  if (o_out_cast) BURST_TRY(check_no_overlap(p.o_out, shape->batch, shape->sq, shape->q_heads, shape->head_dim));
  p.batch = shape->batch;
  p.q_heads = shape->q_heads;
  p.head_dim = shape->head_dim;
  p.sq = (int32_t)shape->sq;
  if (p.sq == 0) return BURST_OK;
  hipError_t e = launch_lse_merge(p, (hipStream_t)hip_stream);
  return e == hipSuccess ? BURST_OK : hip_fail(e);
}

int burst_attn_preprocess_bwd(const burst_shape_t* shape, const burst_tensor_t* o, const burst_tensor_t* d_o,
                              const burst_rowvec_t* d_out, void* hip_stream) {
  BURST_TRY(check_shape(shape));
  PreParams p;
  std::memset(&p, 0, sizeof(p));
  BURST_TRY(check_tensor(o, 3, &p.o));
  BURST_TRY(check_tensor(d_o, 1, &p.d_o));
  BURST_TRY(check_rowvec(d_out, &p.d));
  BURST_TRY(check_rowvec_no_overlap(p.d, shape->batch, shape->q_heads, shape->sq));
  p.batch = shape->batch;
  p.q_heads = shape->q_heads;
  p.head_dim = shape->head_dim;
  p.sq = (int32_t)shape->sq;
  if (p.sq == 0) return BURST_OK;
  hipError_t e = launch_preprocess_bwd(p, (hipStream_t)hip_stream);
  return e == hipSuccess ? BURST_OK : hip_fail(e);
}

int burst_attn_step_bwd(const burst_shape_t* shape, const burst_mask_t* mask, const burst_tensor_t* q,
                        const burst_tensor_t* k, const burst_tensor_t* v, const burst_tensor_t* d_o,
                        const burst_rowvec_t* lse, const burst_rowvec_t* d, const burst_tensor_t* dq,
                        const burst_tensor_t* dk, const burst_tensor_t* dv, int32_t accumulate_flags,
                        void* hip_stream) {
  BURST_TRY(check_shape(shape));
  BwdParams p;
  std::memset(&p, 0, sizeof(p));
  BURST_TRY(check_mask(mask, shape->sq, shape->sk, &p.mask));
  BURST_TRY(check_tensor(q, 1, &p.q));
  BURST_TRY(check_tensor(k, 1, &p.k));
  BURST_TRY(check_tensor(v, 1, &p.v));
  BURST_TRY(check_tensor(d_o, 1, &p.d_o));
  BURST_TRY(check_rowvec(lse, &p.lse));
  BURST_TRY(check_rowvec(d, &p.d));
  if (!dq && !dk && !dv) return BURST_ERR_INVALID_ARG;
  if ((dk == nullptr) != (dv == nullptr)) return BURST_ERR_INVALID_ARG;
  if (accumulate_flags & ~(BURST_ACC_DQ | BURST_ACC_DK | BURST_ACC_DV)) return BURST_ERR_INVALID_ARG;
  if (dq) {
    BURST_TRY(check_tensor(dq, 2, &p.dq));
    BURST_TRY(check_no_overlap(p.dq, shape->batch, shape->sq, shape->q_heads, shape->head_dim));
  }
  if (dk) {
    BURST_TRY(check_tensor(dk, 2, &p.dk));
    BURST_TRY(check_no_overlap(p.dk, shape->batch, shape->sk, shape->kv_heads, shape->head_dim));
  }
  if (dv) {
    BURST_TRY(check_tensor(dv, 2, &p.dv));
    BURST_TRY(check_no_overlap(p.dv, shape->batch, shape->sk, shape->kv_heads, shape->head_dim));
  }
  p.acc_dq = (accumulate_flags & BURST_ACC_DQ) != 0;
  p.acc_dk = (accumulate_flags & BURST_ACC_DK) != 0;
  p.acc_dv = (accumulate_flags & BURST_ACC_DV) != 0;
  p.batch = shape->batch;
  p.q_heads = shape->q_heads;
  p.kv_heads = shape->kv_heads;
  p.head_dim = shape->head_dim;
  p.sq = (int32_t)shape->sq;
  p.sk = (int32_t)shape->sk;
  p.scale = shape->scale;
  hipStream_t stream = (hipStream_t)hip_stream;
  hipError_t e = hipSuccess;
  if (p.sq == 0 || p.sk == 0) {
    // nothing contributes: "+=" leaves the gradients alone, "=" makes them zero
    if (dq && !p.acc_dq && p.sq > 0) e = launch_zero_tensor(p.dq, p.batch, p.sq, p.q_heads, p.head_dim, stream);
    if (e == hipSuccess && dk && !p.acc_dk && p.sk > 0)
      e = launch_zero_tensor(p.dk, p.batch, p.sk, p.kv_heads, p.head_dim, stream);
    if (e == hipSuccess && dv && !p.acc_dv && p.sk > 0)
      e = launch_zero_tensor(p.dv, p.batch, p.sk, p.kv_heads, p.head_dim, stream);
  } else {
    e = launch_step_bwd(p, stream);
  }
  return e == hipSuccess ? BURST_OK : hip_fail(e);
}

static int fill_common(int32_t dev_i, int32_t shard_j, int32_t G, int64_t N, burst_mask_t* out) {
  if (!out || G < 1 || dev_i < 0 || dev_i >= G || shard_j < 0 || shard_j >= G || N < 0) return BURST_ERR_INVALID_ARG;
  std::memset(out, 0, sizeof(*out));
  return BURST_OK;
}

int burst_attn_fill_zigzag_mask(int32_t dev_i, int32_t shard_j, int32_t G, int64_t N, int32_t causal,
                                burst_mask_t* out) {
  BURST_TRY(fill_common(dev_i, shard_j, G, N, out));
  if (N % (2 * (int64_t)G)) return BURST_ERR_INVALID_ARG;
  const int64_t P = N / (2 * (int64_t)G);
  out->mode = causal ? BURST_MASK_CAUSAL : BURST_MASK_FULL;
  out->q_nseg = out->k_nseg = 2;
  out->q_seg_len = out->k_seg_len = P;
  out->q_seg_pos[0] = dev_i * P;
  out->q_seg_pos[1] = N - (dev_i + 1) * P;
  out->k_seg_pos[0] = shard_j * P;
  out->k_seg_pos[1] = N - (shard_j + 1) * P;
  out->pos_stride = 1;
  return BURST_OK;
}

int burst_attn_fill_contiguous_mask(int32_t dev_i, int32_t shard_j, int32_t G, int64_t N, int32_t causal,
                                    burst_mask_t* out) {
  BURST_TRY(fill_common(dev_i, shard_j, G, N, out));
  if (N % G) return BURST_ERR_INVALID_ARG;
  const int64_t n = N / G;
  out->mode = causal ? BURST_MASK_CAUSAL : BURST_MASK_FULL;
  out->q_nseg = out->k_nseg = 1;
  out->q_seg_len = out->k_seg_len = n;
  out->q_seg_pos[0] = dev_i * n;
  out->k_seg_pos[0] = shard_j * n;
  out->pos_stride = 1;
  return BURST_OK;
}

int burst_attn_fill_striped_mask(int32_t dev_i, int32_t shard_j, int32_t G, int64_t N, int32_t causal,
                                 burst_mask_t* out) {
  BURST_TRY(fill_common(dev_i, shard_j, G, N, out));
  if (N % G) return BURST_ERR_INVALID_ARG;
  const int64_t n = N / G;
  out->mode = causal ? BURST_MASK_CAUSAL : BURST_MASK_FULL;
  out->q_nseg = out->k_nseg = 1;
  out->q_seg_len = out->k_seg_len = n;
  out->q_seg_pos[0] = dev_i;
  out->k_seg_pos[0] = shard_j;
  out->pos_stride = G;
  return BURST_OK;
}

int burst_attn_fill_block_striped_mask(int32_t dev_i, int32_t shard_j, int32_t G, int64_t N, int64_t N_blk, int32_t causal,
                                       burst_mask_t* out) {
  BURST_TRY(fill_common(dev_i, shard_j, G, N, out));
  if (N_blk < 1 || N % N_blk || N_blk % G) return BURST_ERR_INVALID_ARG;
  const int64_t m = N_blk / G, pieces = N / N_blk;
  if (pieces > INT32_MAX) return BURST_ERR_UNSUPPORTED;
  out->mode = causal ? BURST_MASK_CAUSAL : BURST_MASK_FULL;
  out->q_nseg = out->k_nseg = (int32_t)pieces;
  out->q_seg_len = out->k_seg_len = m;
  out->q_seg_pos[0] = dev_i * m;
  out->q_seg_pos[1] = dev_i * m + N_blk;
  out->k_seg_pos[0] = shard_j * m;
  out->k_seg_pos[1] = shard_j * m + N_blk;
  out->pos_stride = 1;
  return BURST_OK;
}

int64_t burst_attn_visible_pairs(const burst_mask_t* m) {
  if (!m) return -1;
  if (m->q_nseg < 1 || m->k_nseg < 1 || m->q_seg_len < 0 || m->k_seg_len < 0 || m->q_seg_len > kMaxRows ||
      m->k_seg_len > kMaxRows)
    return -1;
  const int64_t sq = m->q_nseg * m->q_seg_len, sk = m->k_nseg * m->k_seg_len;
  MaskDev mk;
  if (check_mask(m, sq, sk, &mk) != BURST_OK) return -1;
  if (!mk.causal) return sq * sk;
  // per query row: the keys at or before it, minus those that have left its window; positions grow
  // with the row on both axes, so both sets are prefixes of the key chunk
  const AxisMap qa = axis_of<true>(mk), ka = axis_of<false>(mk);
  int64_t total = 0;
  for (int64_t r = 0; r < sq; ++r) {
    const long long p = axis_position(qa, (int)r);
    total += rows_lt(ka, p + 1, (int)sk) - rows_lt(ka, p - (long long)mk.window + 1, (int)sk);
  }
  return total;
}

// The tile logic of the kernels, run on the host with the code the kernels compile.
int burst_attn_tile_class(const burst_mask_t* mask, int64_t q0, int64_t q1, int64_t k0, int64_t k1, int32_t method) {
  if (!mask || mask->q_nseg < 1 || mask->k_nseg < 1) return BURST_ERR_INVALID_ARG;
  const int64_t sq = mask->q_nseg * mask->q_seg_len, sk = mask->k_nseg * mask->k_seg_len;
  MaskDev mk;
  BURST_TRY(check_mask(mask, sq, sk, &mk));
  if (q0 < 0 || q1 > sq || q0 >= q1 || k0 < 0 || k1 > sk || k0 >= k1) return BURST_ERR_INVALID_ARG;
  if (method == 0) return classify(mk, (int)q0, (int)q1, (int)k0, (int)k1, false);
  int lo, hi;
  if (method == 1) {   // query block against a fixed key range
    range_minmax<false>(mk, (int)k0, (int)k1, lo, hi);
    BlockClassifier<true> c;
    c.init(mk, lo, hi, (int)sq, false);
    return c(mk, (int)q0, (int)q1, false);
  }
  if (method == 2) {   // key block against a fixed query range
    range_minmax<true>(mk, (int)q0, (int)q1, lo, hi);
    BlockClassifier<false> c;
    c.init(mk, lo, hi, (int)sk, false);
    return c(mk, (int)k0, (int)k1, false);
  }
  return BURST_ERR_INVALID_ARG;
}

int burst_attn_visible_tile_runs(const burst_mask_t* mask, int32_t query_axis, int32_t tile_rows, int64_t r0, int64_t r1,
                                 int32_t out_start_len[4]) {
  if (!mask || !out_start_len || mask->q_nseg < 1 || mask->k_nseg < 1) return BURST_ERR_INVALID_ARG;
  const int64_t sq = mask->q_nseg * mask->q_seg_len, sk = mask->k_nseg * mask->k_seg_len;
  MaskDev mk;
  BURST_TRY(check_mask(mask, sq, sk, &mk));
  const int64_t other = query_axis ? sk : sq;
  if (r0 < 0 || r1 > other || r0 >= r1) return BURST_ERR_INVALID_ARG;
  int lo, hi;
  TileRun tr;
  if (query_axis) {
    range_minmax<false>(mk, (int)r0, (int)r1, lo, hi);
    if (tile_rows == 64) tr = visible_tiles<true, 64>(mk, lo, hi, (int)sq);
    else if (tile_rows == 256) tr = visible_tiles<true, 256>(mk, lo, hi, (int)sq);
    else return BURST_ERR_UNSUPPORTED;
  } else {
    range_minmax<true>(mk, (int)r0, (int)r1, lo, hi);
    if (tile_rows == 64) tr = visible_tiles<false, 64>(mk, lo, hi, (int)sk);
    else if (tile_rows == 128) tr = visible_tiles<false, 128>(mk, lo, hi, (int)sk);
    else return BURST_ERR_UNSUPPORTED;
  }
  out_start_len[0] = tr.start;
  out_start_len[1] = tr.len;
  out_start_len[2] = 0;   // the kernels' walks are one run; the second pair stays empty
  out_start_len[3] = 0;
  return BURST_OK;
}

int burst_attn_set_chunk_rows(int32_t rows) {
  burst::set_chunk_rows(rows);
  return rows < 256 ? 256 : rows;
}

int burst_attn_chunk_plan(const burst_mask_t* mask, int32_t query_axis, int32_t max_ranges, int64_t* out) {
  if (!mask || !out || max_ranges < 0 || mask->q_nseg < 1 || mask->k_nseg < 1) return BURST_ERR_INVALID_ARG;
  const int64_t sq = mask->q_nseg * mask->q_seg_len, sk = mask->k_nseg * mask->k_seg_len;
  MaskDev mk;
  BURST_TRY(check_mask(mask, sq, sk, &mk));
  return chunk_plan(mk, (int)sq, (int)sk, query_axis != 0, max_ranges, out);
}

int burst_attn_mfma_probe(int32_t random_operands, int32_t iterations, float* sink, int64_t* flops_out,
                          void* hip_stream) {
  if (iterations < 1 || iterations > (1 << 24)) return BURST_ERR_INVALID_ARG;
  hipError_t e = launch_mfma_probe(sink, iterations, random_operands != 0, flops_out, (hipStream_t)hip_stream);
  return e == hipSuccess ? BURST_OK : hip_fail(e);
}

static int check_lm_shape(const burst_lm_head_shape_t* s) {
  if (!s) return BURST_ERR_INVALID_ARG;
  if (s->n_tokens < 0 || s->d_model < 1 || s->vocab < 1 || s->tile_tokens < 1 || s->tile_tokens % 256 != 0)
    return BURST_ERR_INVALID_ARG;
  if (!std::isfinite(s->grad_scale)) return BURST_ERR_INVALID_ARG;
  if (s->d_model % 256 != 0) return BURST_ERR_UNSUPPORTED;
  // 32-bit row indices in the kernels and 32-bit byte offsets inside a staged tile
  if (s->n_tokens > INT32_MAX - 256 || s->vocab > ((int64_t)1 << 22) || s->d_model > ((int64_t)1 << 22) ||
      s->tile_tokens > ((int64_t)1 << 20))
    return BURST_ERR_UNSUPPORTED;
  return BURST_OK;
}

int64_t burst_lm_head_workspace_bytes(const burst_lm_head_shape_t* shape) {
  if (check_lm_shape(shape) != BURST_OK) return -1;
  return lm_head_workspace_bytes(shape->tile_tokens, shape->vocab, shape->d_model);
}

// Checks and launch shared by the two entry points; `workspace` is already known to be large enough.
static int lm_head_loss_on(const burst_lm_head_shape_t* shape, const void* h_last, int64_t ld_h, const void* w_head,
                           int64_t ld_w, const int64_t* y, float* loss, float* lse, void* d_h, int32_t d_h_dtype,
                           int64_t ld_dh, float* d_w, int64_t ld_dw, int32_t accumulate_dw, void* workspace,
                           void* hip_stream) {
  const int64_t d = shape->d_model, max_ld = (int64_t)1 << 22;
  auto aligned = [](const void* ptr, uintptr_t a) { return ptr && (reinterpret_cast<uintptr_t>(ptr) % a) == 0; };
  if (!aligned(w_head, 16)) return BURST_ERR_INVALID_ARG;
  if (shape->n_tokens > 0 && (!aligned(h_last, 16) || !aligned(y, 8) || !aligned(loss, 4))) return BURST_ERR_INVALID_ARG;
  if (lse && !aligned(lse, 4)) return BURST_ERR_INVALID_ARG;
  if (ld_h < d || ld_h % 8 != 0 || ld_w < d || ld_w % 8 != 0) return BURST_ERR_INVALID_ARG;
  if (ld_h > max_ld || ld_w > max_ld) return BURST_ERR_UNSUPPORTED;
  if (d_h) {
    if (d_h_dtype != BURST_F32 && d_h_dtype != BURST_BF16) return BURST_ERR_INVALID_ARG;
    if (!aligned(d_h, 16) || ld_dh < d || ld_dh % 8 != 0) return BURST_ERR_INVALID_ARG;
    if (ld_dh > max_ld) return BURST_ERR_UNSUPPORTED;
  }
  if (d_w) {
    if (!aligned(d_w, 16) || ld_dw < d || ld_dw % 4 != 0) return BURST_ERR_INVALID_ARG;
    if (ld_dw > max_ld) return BURST_ERR_UNSUPPORTED;
  }
  LmHeadParams p;
  std::memset(&p, 0, sizeof(p));
  p.n_tokens = (int32_t)shape->n_tokens;
  p.d_model = (int32_t)d;
  p.vocab = (int32_t)shape->vocab;
  p.tile_tokens = (int32_t)shape->tile_tokens;
  p.v_pad = (int32_t)((shape->vocab + 255) / 256 * 256);
  p.grad_scale = shape->grad_scale;
  p.h = (const __bf16*)h_last;
  p.w = (const __bf16*)w_head;
  p.ld_h = ld_h;
  p.ld_w = ld_w;
  p.y = y;
  p.loss = loss;
  p.lse = lse;
  p.dh = d_h;
  p.dh_is_f32 = d_h_dtype == BURST_F32;
  p.ld_dh = ld_dh;
  p.dw = d_w;
  p.ld_dw = ld_dw;
  p.acc_dw = accumulate_dw != 0;
  char* ws = (char*)workspace;
  const int64_t cells = (int64_t)p.tile_tokens * p.v_pad;
  p.logits = (float*)ws;
  p.dlogits = (__bf16*)(ws + cells * 4);
  p.part = (float2*)(ws + cells * 6);
  p.ht = (__bf16*)(ws + cells * 6 + (int64_t)(p.v_pad / 128) * p.tile_tokens * 8);
  hipError_t e = launch_lm_head_loss(p, (hipStream_t)hip_stream);
  return e == hipSuccess ? BURST_OK : hip_fail(e);
}

int burst_lm_head_loss(const burst_lm_head_shape_t* shape, const void* h_last, int64_t ld_h, const void* w_head,
                       int64_t ld_w, const int64_t* y, float* loss, float* lse, void* d_h, int32_t d_h_dtype,
                       int64_t ld_dh, float* d_w, int64_t ld_dw, int32_t accumulate_dw, void* workspace,
                       int64_t workspace_bytes, void* hip_stream) {
  BURST_TRY(check_lm_shape(shape));
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % 256) != 0 ||
      workspace_bytes < lm_head_workspace_bytes(shape->tile_tokens, shape->vocab, shape->d_model))
    return BURST_ERR_INVALID_ARG;
  return lm_head_loss_on(shape, h_last, ld_h, w_head, ld_w, y, loss, lse, d_h, d_h_dtype, ld_dh, d_w, ld_dw, accumulate_dw,
                         workspace, hip_stream);
}

int64_t burst_lm_head_static_scratch_bytes(void) { return kStaticScratchBytes; }

int burst_lm_head_loss_noalloc(const burst_lm_head_shape_t* shape, const void* h_last, int64_t ld_h,
                               const void* w_head, int64_t ld_w, const int64_t* y, float* loss, float* lse, void* d_h,
                               int32_t d_h_dtype, int64_t ld_dh, float* d_w, int64_t ld_dw, int32_t accumulate_dw,
                               void* hip_stream) {
  BURST_TRY(check_lm_shape(shape));
  if (lm_head_workspace_bytes(shape->tile_tokens, shape->vocab, shape->d_model) > kStaticScratchBytes)
    return BURST_ERR_SCRATCH;
  void* ws = nullptr;
  BURST_TRY(static_scratch_of_current_device(&ws));
  return lm_head_loss_on(shape, h_last, ld_h, w_head, ld_w, y, loss, lse, d_h, d_h_dtype, ld_dh, d_w, ld_dw, accumulate_dw,
                         ws, hip_stream);
}

const char* burst_attn_status_string(int status) {
  switch (status) {
    case BURST_OK: return "ok";
    case BURST_ERR_INVALID_ARG: return "invalid argument";
    case BURST_ERR_UNSUPPORTED: return "unsupported dtype, head_dim or position range";
    case BURST_ERR_HIP: return "HIP runtime error";
    case BURST_ERR_SCRATCH: return "the shape needs more scratch memory than the library's built-in buffer holds";
    default: return "unknown status";
  }
}

int burst_attn_last_hip_error(void) { return g_last_hip_error; }

const char* burst_attn_version(void) { return "libburstattn 0.1 (gfx950)"; }

}  // extern "C"
