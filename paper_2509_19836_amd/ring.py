"""Simulated ring driver: the host loop of one device's pass over all KV shards.

On one GPU the ring is simulated: every KV shard already sits in HBM and device i visits them in
ring order, its own shard first and then j = (i - t) mod G (Sec. 3.4; forward algorithm lines
3-12; Alg. 1 for the backward order used here: Q_i, dO_i, Lse_i, D_i stay and dQ_i accumulates
locally while dK_j, dV_j of the visiting shard accumulate).  Nothing here computes: each step is
one call into the C ABI.
"""
from . import binding as lib


def ring_order(i, G):
    return [(i - t) % G for t in range(G)]


def fill_mask(kind, i, j, G, N, window=0, N_blk=0):
    """kind: "full" / "causal" (contiguous split), "zigzag", "striped", "block_striped" (slice i of every
    block of N_blk tokens); window > 0: sliding-window attention over the causal kinds (each token sees
    itself and the window - 1 positions before it)."""
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


def mask_positions(mask, side):
    """Global token positions of the local rows of the "q" or "k" side of a burst_mask_t."""
    import numpy as np
    nseg, seg_len, seg_pos = ((mask.q_nseg, mask.q_seg_len, mask.q_seg_pos) if side == "q" else
                              (mask.k_nseg, mask.k_seg_len, mask.k_seg_pos))
    period = seg_pos[1] - seg_pos[0] if nseg > 1 else 0
    return np.concatenate([seg_pos[0] + s * period + np.arange(seg_len, dtype=np.int64) * mask.pos_stride
                           for s in range(nseg)])


def ring_forward(i, G, N, kind, scale, q_i, k_shards, v_shards, o_acc, lse_acc, stream=None, window=0, N_blk=0):
    """o_acc / lse_acc must hold (0, -inf) on entry; they hold (O_i, Lse_i) on return."""
    B, n, Hq, d = q_i.shape
    for j in ring_order(i, G):
        k_j, v_j = k_shards[j], v_shards[j]
        shp = lib.shape(B, Hq, k_j.shape[2], d, n, k_j.shape[1], scale)
        lib.burst_attn_step_fwd(shp, fill_mask(kind, i, j, G, N, window, N_blk), q_i, k_j, v_j,
                                o_acc=o_acc, lse_acc=lse_acc, stream=stream)


def ring_backward(i, G, N, kind, scale, q_i, do_i, o_i, lse_i, d_i, k_shards, v_shards, dq_i, dk_shards,
                  dv_shards, stream=None, window=0, N_blk=0):
    """D_i once, then one backward step per shard; dq_i, dk_shards[j], dv_shards[j] are fp32
    accumulators ("+=")."""
    B, n, Hq, d = q_i.shape
    shp0 = lib.shape(B, Hq, k_shards[0].shape[2], d, n, n, scale)
    lib.burst_attn_preprocess_bwd(shp0, o_i, do_i, d_i, stream=stream)
    flags = lib.BURST_ACC_DQ | lib.BURST_ACC_DK | lib.BURST_ACC_DV
    for j in ring_order(i, G):
        k_j, v_j = k_shards[j], v_shards[j]
        shp = lib.shape(B, Hq, k_j.shape[2], d, n, k_j.shape[1], scale)
        lib.burst_attn_step_bwd(shp, fill_mask(kind, i, j, G, N, window, N_blk), q_i, k_j, v_j, do_i, lse_i, d_i,
                                dq=dq_i, dk=dk_shards[j], dv=dv_shards[j], accumulate_flags=flags,
                                stream=stream)
