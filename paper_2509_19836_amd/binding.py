"""ctypes binding of libburstattn's C ABI (include/burst_attn.h).

Argument marshalling only: every function here has the name of the C entry point
it calls and does nothing but describe torch tensors as (pointer, strides) and
pass the current HIP stream.  There is no fallback: if the shared library has
not been built, importing this module raises.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("BURST_LIB_PATH", os.path.join(_HERE, "libburstattn.so"))   # override: another build

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} not found: build it first (python -m paper_2509_19836_amd.build, or "
        "__graft_entry__.build()); libburstattn has no CPU or PyTorch fallback")
_lib = C.CDLL(LIB_PATH)

BURST_OK, BURST_ERR_INVALID_ARG, BURST_ERR_UNSUPPORTED, BURST_ERR_HIP, BURST_ERR_SCRATCH = 0, -1, -2, -3, -4
BURST_BF16, BURST_F32 = 0, 1
BURST_MASK_FULL, BURST_MASK_CAUSAL = 0, 1
BURST_ACC_DQ, BURST_ACC_DK, BURST_ACC_DV = 1, 2, 4


class burst_shape_t(C.Structure):
    _fields_ = [("batch", C.c_int32), ("q_heads", C.c_int32), ("kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("sq", C.c_int64), ("sk", C.c_int64), ("scale", C.c_float)]


class burst_tensor_t(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("dtype", C.c_int32), ("_pad", C.c_int32),
                ("stride_b", C.c_int64), ("stride_s", C.c_int64), ("stride_h", C.c_int64)]


class burst_rowvec_t(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("stride_b", C.c_int64), ("stride_h", C.c_int64)]


class burst_mask_t(C.Structure):
    _fields_ = [("mode", C.c_int32), ("q_nseg", C.c_int32), ("k_nseg", C.c_int32), ("_pad", C.c_int32),
                ("q_seg_pos", C.c_int64 * 2), ("k_seg_pos", C.c_int64 * 2),
                ("q_seg_len", C.c_int64), ("k_seg_len", C.c_int64), ("pos_stride", C.c_int64),
                ("window", C.c_int64), ("block_mask", C.c_void_p),
                ("q_block_rows", C.c_int64), ("k_block_rows", C.c_int64), ("block_pitch", C.c_int64)]


_P = C.POINTER
_lib.burst_attn_step_fwd.restype = C.c_int
_lib.burst_attn_step_fwd.argtypes = [_P(burst_shape_t), _P(burst_mask_t)] + [_P(burst_tensor_t)] * 3 + [
    _P(burst_tensor_t), _P(burst_rowvec_t), _P(burst_tensor_t), _P(burst_rowvec_t), C.c_void_p]
_lib.burst_attn_lse_merge.restype = C.c_int
_lib.burst_attn_lse_merge.argtypes = [_P(burst_shape_t), _P(burst_tensor_t), _P(burst_rowvec_t),
                                      _P(burst_tensor_t), _P(burst_rowvec_t), _P(burst_tensor_t), C.c_void_p]
_lib.burst_attn_preprocess_bwd.restype = C.c_int
_lib.burst_attn_preprocess_bwd.argtypes = [_P(burst_shape_t), _P(burst_tensor_t), _P(burst_tensor_t),
                                           _P(burst_rowvec_t), C.c_void_p]
_lib.burst_attn_step_bwd.restype = C.c_int
_lib.burst_attn_step_bwd.argtypes = [_P(burst_shape_t), _P(burst_mask_t)] + [_P(burst_tensor_t)] * 4 + [
    _P(burst_rowvec_t)] * 2 + [_P(burst_tensor_t)] * 3 + [C.c_int32, C.c_void_p]
for _name in ("zigzag", "contiguous", "striped"):
    _f = getattr(_lib, f"burst_attn_fill_{_name}_mask")
    _f.restype = C.c_int
    _f.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int64, C.c_int32, _P(burst_mask_t)]
_lib.burst_attn_fill_block_striped_mask.restype = C.c_int
_lib.burst_attn_fill_block_striped_mask.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int64, C.c_int64, C.c_int32, _P(burst_mask_t)]
_lib.burst_attn_visible_pairs.restype = C.c_int64
_lib.burst_attn_visible_pairs.argtypes = [_P(burst_mask_t)]
_lib.burst_attn_tile_class.restype = C.c_int
_lib.burst_attn_tile_class.argtypes = [_P(burst_mask_t)] + [C.c_int64] * 4 + [C.c_int32]
_lib.burst_attn_visible_tile_runs.restype = C.c_int
_lib.burst_attn_visible_tile_runs.argtypes = [_P(burst_mask_t), C.c_int32, C.c_int32, C.c_int64, C.c_int64, _P(C.c_int32 * 4)]
_lib.burst_attn_set_chunk_rows.restype = C.c_int
_lib.burst_attn_set_chunk_rows.argtypes = [C.c_int32]
_lib.burst_attn_chunk_plan.restype = C.c_int
_lib.burst_attn_chunk_plan.argtypes = [_P(burst_mask_t), C.c_int32, C.c_int32, _P(C.c_int64)]
_lib.burst_attn_mfma_probe.restype = C.c_int
_lib.burst_attn_mfma_probe.argtypes = [C.c_int32, C.c_int32, C.c_void_p, _P(C.c_int64), C.c_void_p]


class burst_lm_head_shape_t(C.Structure):
    _fields_ = [("n_tokens", C.c_int64), ("d_model", C.c_int64), ("vocab", C.c_int64), ("tile_tokens", C.c_int64),
                ("grad_scale", C.c_float), ("_pad", C.c_int32)]


_lib.burst_lm_head_workspace_bytes.restype = C.c_int64
_lib.burst_lm_head_workspace_bytes.argtypes = [_P(burst_lm_head_shape_t)]
_lib.burst_lm_head_loss.restype = C.c_int
_lib.burst_lm_head_loss.argtypes = [_P(burst_lm_head_shape_t), C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p,
                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_void_p, C.c_int64,
                                    C.c_int32, C.c_void_p, C.c_int64, C.c_void_p]
_lib.burst_lm_head_static_scratch_bytes.restype = C.c_int64
_lib.burst_lm_head_static_scratch_bytes.argtypes = []
_lib.burst_lm_head_loss_noalloc.restype = C.c_int
_lib.burst_lm_head_loss_noalloc.argtypes = [_P(burst_lm_head_shape_t), C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p,
                                            C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_void_p, C.c_int64,
                                            C.c_int32, C.c_void_p]
_lib.burst_attn_status_string.restype = C.c_char_p
_lib.burst_attn_status_string.argtypes = [C.c_int]
_lib.burst_attn_last_hip_error.restype = C.c_int
_lib.burst_attn_version.restype = C.c_char_p

EXPORTS = ["burst_attn_step_fwd", "burst_attn_lse_merge", "burst_attn_preprocess_bwd", "burst_attn_step_bwd",
           "burst_attn_fill_zigzag_mask", "burst_attn_fill_contiguous_mask", "burst_attn_fill_striped_mask",
           "burst_attn_fill_block_striped_mask",
           "burst_attn_visible_pairs", "burst_attn_tile_class", "burst_attn_visible_tile_runs", "burst_attn_mfma_probe", "burst_attn_set_chunk_rows", "burst_attn_chunk_plan", "burst_attn_status_string", "burst_attn_last_hip_error",
           "burst_attn_version", "burst_lm_head_workspace_bytes", "burst_lm_head_loss",
           "burst_lm_head_static_scratch_bytes", "burst_lm_head_loss_noalloc"]


class BurstError(RuntimeError):
    def __init__(self, status):
        self.status = status
        msg = _lib.burst_attn_status_string(status).decode()
        if status == BURST_ERR_HIP:
            msg += f" (hip error {_lib.burst_attn_last_hip_error()})"
        super().__init__(f"libburstattn: {msg}")


def _check(status):
    if status != BURST_OK:
        raise BurstError(status)


def shape(batch, q_heads, kv_heads, head_dim, sq, sk, scale):
    return burst_shape_t(batch, q_heads, kv_heads, head_dim, sq, sk, scale)


def tensor(t):
    """Describe a [batch, seq, heads, head_dim] torch tensor (bf16 or fp32, last dim contiguous)."""
    if t is None:
        return None
    assert t.dim() == 4 and t.stride(3) == 1, "expected [batch, seq, heads, head_dim] with contiguous head_dim"
    dt = {torch.bfloat16: BURST_BF16, torch.float32: BURST_F32}[t.dtype]
    return burst_tensor_t(t.data_ptr(), dt, 0, t.stride(0), t.stride(1), t.stride(2))


def rowvec(t):
    """Describe a [batch, heads, seq] fp32 torch tensor (seq contiguous)."""
    if t is None:
        return None
    assert t.dim() == 3 and t.stride(2) == 1 and t.dtype == torch.float32
    return burst_rowvec_t(t.data_ptr(), t.stride(0), t.stride(1))


def _ref(x):
    return None if x is None else C.byref(x)


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    return C.c_void_p(stream)


def burst_attn_fill_zigzag_mask(dev_i, shard_j, G, N, causal=True):
    m = burst_mask_t()
    _check(_lib.burst_attn_fill_zigzag_mask(dev_i, shard_j, G, N, int(causal), C.byref(m)))
    return m


def burst_attn_fill_contiguous_mask(dev_i, shard_j, G, N, causal=True):
    m = burst_mask_t()
    _check(_lib.burst_attn_fill_contiguous_mask(dev_i, shard_j, G, N, int(causal), C.byref(m)))
    return m


def burst_attn_fill_striped_mask(dev_i, shard_j, G, N, causal=True):
    m = burst_mask_t()
    _check(_lib.burst_attn_fill_striped_mask(dev_i, shard_j, G, N, int(causal), C.byref(m)))
    return m


def burst_attn_fill_block_striped_mask(dev_i, shard_j, G, N, N_blk, causal=True):
    m = burst_mask_t()
    _check(_lib.burst_attn_fill_block_striped_mask(dev_i, shard_j, G, N, N_blk, int(causal), C.byref(m)))
    return m


def set_block_mask(mask, block_mask, q_block_rows, k_block_rows):
    """Attach a block-wise sparse mask (2-D uint8 device tensor, unit stride along its rows) to a
    burst_mask_t; the tensor must outlive the steps that use the mask."""
    if block_mask.dim() != 2 or block_mask.element_size() != 1 or block_mask.stride(1) != 1 or not block_mask.is_cuda:
        raise ValueError("block_mask: 2-D one-byte device tensor with unit row stride expected")
    mask.block_mask = block_mask.data_ptr()
    mask.q_block_rows, mask.k_block_rows, mask.block_pitch = q_block_rows, k_block_rows, block_mask.stride(0)
    return mask


def burst_attn_visible_pairs(mask):
    return _lib.burst_attn_visible_pairs(C.byref(mask))


def burst_attn_tile_class(mask, q0, q1, k0, k1, method=0):
    st = _lib.burst_attn_tile_class(C.byref(mask), q0, q1, k0, k1, method)
    if st < 0:
        raise BurstError(st)
    return st


def burst_attn_visible_tile_runs(mask, query_axis, tile_rows, r0, r1):
    """Runs of tiles as [(start, length), (start, length)]."""
    out = (C.c_int32 * 4)()
    _check(_lib.burst_attn_visible_tile_runs(C.byref(mask), int(query_axis), tile_rows, r0, r1, C.byref(out)))
    return [(out[0], out[1]), (out[2], out[3])]


def burst_attn_version():
    return _lib.burst_attn_version().decode()


def burst_attn_status_string(status):
    return _lib.burst_attn_status_string(status).decode()


def burst_attn_step_fwd(shp, mask, q, k, v, o_part=None, lse_part=None, o_acc=None, lse_acc=None, stream=None):
    _check(_lib.burst_attn_step_fwd(C.byref(shp), _ref(mask), _ref(tensor(q)), _ref(tensor(k)), _ref(tensor(v)),
                                    _ref(tensor(o_part)), _ref(rowvec(lse_part)), _ref(tensor(o_acc)),
                                    _ref(rowvec(lse_acc)), _stream(stream)))


def burst_attn_lse_merge(shp, o_acc, lse_acc, o_part, lse_part, o_out_cast=None, stream=None):
    _check(_lib.burst_attn_lse_merge(C.byref(shp), _ref(tensor(o_acc)), _ref(rowvec(lse_acc)),
                                     _ref(tensor(o_part)), _ref(rowvec(lse_part)), _ref(tensor(o_out_cast)),
                                     _stream(stream)))


def burst_attn_preprocess_bwd(shp, o, d_o, d_out, stream=None):
    _check(_lib.burst_attn_preprocess_bwd(C.byref(shp), _ref(tensor(o)), _ref(tensor(d_o)), _ref(rowvec(d_out)),
                                          _stream(stream)))


def burst_attn_step_bwd(shp, mask, q, k, v, d_o, lse, d, dq=None, dk=None, dv=None, accumulate_flags=0,
                        stream=None):
    _check(_lib.burst_attn_step_bwd(C.byref(shp), _ref(mask), _ref(tensor(q)), _ref(tensor(k)), _ref(tensor(v)),
                                    _ref(tensor(d_o)), _ref(rowvec(lse)), _ref(rowvec(d)), _ref(tensor(dq)),
                                    _ref(tensor(dk)), _ref(tensor(dv)), accumulate_flags, _stream(stream)))


def lm_head_shape(n_tokens, d_model, vocab, tile_tokens, grad_scale=1.0):
    return burst_lm_head_shape_t(n_tokens, d_model, vocab, tile_tokens, grad_scale, 0)


def burst_lm_head_workspace_bytes(shp):
    n = _lib.burst_lm_head_workspace_bytes(C.byref(shp))
    if n < 0:
        raise BurstError(BURST_ERR_INVALID_ARG)
    return n


def burst_lm_head_loss(shp, h_last, w_head, y, loss, workspace, lse=None, d_h=None, d_w=None, accumulate_dw=False,
                       stream=None):
    """h_last [N, d] bf16, w_head [v, d] bf16, y [N] int64, loss / lse [N] fp32, d_h [N, d] fp32 or bf16,
    d_w [v, d] fp32, workspace: one-byte tensor of burst_lm_head_workspace_bytes(shp) bytes.  Rows may be
    strided; the last dimension is contiguous."""
    for t in (h_last, w_head, d_h, d_w):
        assert t is None or (t.dim() == 2 and t.stride(1) == 1), "expected 2-D tensors with a contiguous last dim"
    assert h_last.dtype == torch.bfloat16 and w_head.dtype == torch.bfloat16 and y.dtype == torch.int64
    assert y.is_contiguous() and loss.is_contiguous() and loss.dtype == torch.float32
    assert lse is None or (lse.is_contiguous() and lse.dtype == torch.float32)
    assert d_w is None or d_w.dtype == torch.float32
    ptr = lambda t: None if t is None else C.c_void_p(t.data_ptr())
    dh_dtype = BURST_F32 if d_h is None else {torch.bfloat16: BURST_BF16, torch.float32: BURST_F32}[d_h.dtype]
    _check(_lib.burst_lm_head_loss(C.byref(shp), ptr(h_last), h_last.stride(0), ptr(w_head), w_head.stride(0), ptr(y),
                                   ptr(loss), ptr(lse), ptr(d_h), dh_dtype, 0 if d_h is None else d_h.stride(0),
                                   ptr(d_w), 0 if d_w is None else d_w.stride(0), int(accumulate_dw),
                                   ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))


def burst_lm_head_static_scratch_bytes():
    return _lib.burst_lm_head_static_scratch_bytes()


def burst_lm_head_loss_noalloc(shp, h_last, w_head, y, loss, lse=None, d_h=None, d_w=None, accumulate_dw=False,
                               stream=None):
    """burst_lm_head_loss on the library's built-in scratch array (no workspace argument, no allocation)."""
    for t in (h_last, w_head, d_h, d_w):
        assert t is None or (t.dim() == 2 and t.stride(1) == 1), "expected 2-D tensors with a contiguous last dim"
    assert h_last.dtype == torch.bfloat16 and w_head.dtype == torch.bfloat16 and y.dtype == torch.int64
    assert y.is_contiguous() and loss.is_contiguous() and loss.dtype == torch.float32
    assert lse is None or (lse.is_contiguous() and lse.dtype == torch.float32)
    assert d_w is None or d_w.dtype == torch.float32
    ptr = lambda t: None if t is None else C.c_void_p(t.data_ptr())
    dh_dtype = BURST_F32 if d_h is None else {torch.bfloat16: BURST_BF16, torch.float32: BURST_F32}[d_h.dtype]
    _check(_lib.burst_lm_head_loss_noalloc(C.byref(shp), ptr(h_last), h_last.stride(0), ptr(w_head), w_head.stride(0),
                                           ptr(y), ptr(loss), ptr(lse), ptr(d_h), dh_dtype,
                                           0 if d_h is None else d_h.stride(0), ptr(d_w),
                                           0 if d_w is None else d_w.stride(0), int(accumulate_dw), _stream(stream)))


def burst_attn_set_chunk_rows(rows):
    """Rows of the streamed axis per launch of a step kernel (diagnostics); returns the value in force."""
    return _lib.burst_attn_set_chunk_rows(int(rows))


def burst_attn_chunk_plan(mask, query_axis, max_ranges=4096):
    """Ranges the step launchers cut an axis into: list of dicts (r0, r1, nseg, seg_len, pos0, period, blk_offset)."""
    out = (C.c_int64 * (7 * max_ranges))()
    n = _lib.burst_attn_chunk_plan(C.byref(mask), int(query_axis), max_ranges, out)
    if n < 0:
        _check(n)
    keys = ("r0", "r1", "nseg", "seg_len", "pos0", "period", "blk_offset")
    return [dict(zip(keys, out[7 * i:7 * i + 7])) for i in range(min(n, max_ranges))]


def burst_attn_mfma_probe(random_operands, iterations, stream=None):
    """Enqueue the MFMA ceiling probe; returns the flop count of the launch."""
    flops = C.c_int64(0)
    _check(_lib.burst_attn_mfma_probe(int(random_operands), iterations, None, C.byref(flops), _stream(stream)))
    return flops.value


def raw():
    """The ctypes library handle, for tests that exercise the error paths with raw structs."""
    return _lib
