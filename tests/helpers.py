"""Shared plumbing of the parity tests: moving seeded host tensors to the GPU, slicing shards by
the positions a mask descriptor states, and the stated tolerances."""
import numpy as np

from paper_2509_19836_amd import workloads as wl

# Stated parity bar: max |err| <= 2e-2 * max|ref| on O / dQ / dK / dV, <= 1e-3 absolute on Lse.
REL_TOL = 2e-2
LSE_TOL = 1e-3


def mask_positions(mask, side):
    """Global token positions of the local rows of the q or k side of a burst_mask_t."""
    nseg = mask.q_nseg if side == "q" else mask.k_nseg
    seg_len = mask.q_seg_len if side == "q" else mask.k_seg_len
    seg_pos = mask.q_seg_pos if side == "q" else mask.k_seg_pos
    period = seg_pos[1] - seg_pos[0] if nseg > 1 else 0
    return np.concatenate([seg_pos[0] + s * period + np.arange(seg_len, dtype=np.int64) * mask.pos_stride
                           for s in range(nseg)])


def fill_mask(lib, kind, i, j, G, N, window=0, N_blk=0):
    """kind: full | causal (contiguous split) | zigzag | striped | block_striped; window > 0 adds a sliding window."""
    if kind == "full":
        m = lib.burst_attn_fill_contiguous_mask(i, j, G, N, False)
    elif kind == "causal":
        m = lib.burst_attn_fill_contiguous_mask(i, j, G, N, True)
    elif kind == "zigzag":
        m = lib.burst_attn_fill_zigzag_mask(i, j, G, N, True)
    elif kind == "striped":
        m = lib.burst_attn_fill_striped_mask(i, j, G, N, True)
    elif kind == "block_striped":
        m = lib.burst_attn_fill_block_striped_mask(i, j, G, N, N_blk, True)
    else:
        raise ValueError(kind)
    m.window = window
    return m


def oracle_positions(oc, kind, i, G, N, N_blk=0):
    if kind == "block_striped":
        return oc.block_striped_positions(i, G, N, N_blk)
    if kind in ("full", "causal"):
        return oc.contiguous_positions(i, G, N)
    if kind == "zigzag":
        return oc.zigzag_positions(i, G, N)
    if kind == "striped":
        return oc.striped_positions(i, G, N)
    raise ValueError(kind)


def dev_bf16(bits):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to("cuda")
    return t.view(torch.bfloat16)


def rel_err(got, ref):
    """max |got - ref| / max |ref| (the stated parity metric)."""
    ref = np.asarray(ref, np.float64)
    got = np.asarray(got, np.float64)
    denom = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (denom if denom > 0 else 1.0))


def lse_err(got, ref):
    """max |got - ref| over finite entries; -inf must match exactly."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    dead = ~np.isfinite(ref)
    assert (got[dead] == ref[dead]).all(), "-inf rows differ"
    if dead.all():
        return 0.0
    return float(np.abs(got[~dead] - ref[~dead]).max())


def widen(bits):
    return wl.bf16_bits_to_f64(bits)
