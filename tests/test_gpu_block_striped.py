"""The block-striped split of block-wise sparse attention (Sec. 3.4) through the C ABI: many-piece mask
descriptors (slice i of every block of N_blk tokens), whole rings forward and backward against the
unsharded fp64 oracle, with the causal rule, a sliding window and a block pattern M_blk on top; the same
pattern under the contiguous, zigzag and striped splits; equal visible-pair counts per step."""
import numpy as np
import pytest

from oracle import burst_oracle as oc
from paper_2509_19836_amd import workloads as wl
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def _ring(lib, kind, G, N, N_blk, Hq, Hkv, d, seed, causal=True, window=0, pattern=None, devices=None):
    """All steps of the given devices: fused forward state, dQ_i, and dK_j / dV_j collected over the
    devices, against the unsharded oracle on global positions.  pattern: global block pattern over
    blocks of N_blk tokens (None: no block mask); every split used here keeps local row blocks inside
    one global block, so the step's mask is a gather of the pattern."""
    import torch
    w = wl.Workload(f"blk_{kind}", 1, Hq, Hkv, d, N // G, G, "full")
    T = wl.host_tensors(w, 7, seed_offset=seed)
    host = {n: hp.widen(T[n][1]) for n in T}
    dev = {n: hp.dev_bf16(T[n][1]) for n in T}
    glob = np.arange(N)
    vis_all = oc.visibility(glob, glob, causal, window)
    if pattern is not None:
        vis_all &= oc.block_pattern_visibility(glob, glob, pattern, N_blk)
    O, lse = oc.mha_attention_fwd(host["q"], host["k"], host["v"], w.scale, vis_all)
    dQ, dK, dV = oc.mha_attention_bwd(host["q"], host["k"], host["v"], host["do"], w.scale, vis_all)
    rows = [hp.oracle_positions(oc, "causal" if kind == "contiguous" else kind, j, G, N, N_blk) for j in range(G)]
    idx = [torch.from_numpy(r).cuda() for r in rows]
    n = rows[0].size
    shard = lambda name, j: dev[name][:, idx[j]].contiguous()
    ks, vs = [shard("k", j) for j in range(G)], [shard("v", j) for j in range(G)]
    f32 = dict(device="cuda", dtype=torch.float32)
    devices = list(range(G)) if devices is None else devices
    dks = [torch.zeros(1, n, Hkv, d, **f32) for _ in range(G)]
    dvs = [torch.zeros(1, n, Hkv, d, **f32) for _ in range(G)]
    shp = lib.shape(1, Hq, Hkv, d, n, n, w.scale)
    step_pairs = {}
    keep = []
    for i in devices:
        q_i, do_i = shard("q", i), shard("do", i)
        o_acc = torch.zeros(1, n, Hq, d, **f32)
        lse_acc = torch.full((1, Hq, n), -float("inf"), **f32)
        masks = {}
        for j in oc.ring_order(i, G):
            base = "causal" if kind == "contiguous" else kind
            m = hp.fill_mask(lib, base, i, j, G, N, window, N_blk)
            if not causal:
                m.mode = lib.BURST_MASK_FULL
            assert (hp.mask_positions(m, "q") == rows[i]).all() and (hp.mask_positions(m, "k") == rows[j]).all()
            vis_ij = vis_all[np.ix_(rows[i], rows[j])]
            step_pairs[(i, j)] = int(vis_ij.sum())
            if pattern is not None:
                R = _local_block_rows(kind, G, N, N_blk)
                bm = wl.local_block_mask(pattern, rows[i], rows[j], R, N_blk)
                keep.append(torch.from_numpy(bm).cuda())
                lib.set_block_mask(m, keep[-1], R, R)
            else:
                assert lib.burst_attn_visible_pairs(m) == step_pairs[(i, j)]
            masks[j] = m
            print(f"{kind} fwd device {i} shard {j} window {window} blocks {pattern is not None}", flush=True)
            lib.burst_attn_step_fwd(shp, m, q_i, ks[j], vs[j], o_acc=o_acc, lse_acc=lse_acc)
        d_i = torch.empty(1, Hq, n, **f32)
        lib.burst_attn_preprocess_bwd(shp, o_acc, do_i, d_i)
        dq = torch.zeros(1, n, Hq, d, **f32)
        for j in oc.ring_order(i, G):
            print(f"{kind} bwd device {i} shard {j}", flush=True)
            lib.burst_attn_step_bwd(shp, masks[j], q_i, ks[j], vs[j], do_i, lse_acc, d_i, dq=dq, dk=dks[j], dv=dvs[j],
                                    accumulate_flags=7)
        torch.cuda.synchronize()
        assert hp.rel_err(o_acc.cpu().numpy(), O[:, rows[i]]) <= hp.REL_TOL
        assert hp.lse_err(lse_acc.cpu().numpy(), lse[:, :, rows[i]]) <= hp.LSE_TOL
        assert hp.rel_err(dq.cpu().numpy(), dQ[:, rows[i]]) <= hp.REL_TOL
    if len(devices) == G:
        for j in range(G):
            assert hp.rel_err(dks[j].cpu().numpy(), dK[:, rows[j]]) <= hp.REL_TOL
            assert hp.rel_err(dvs[j].cpu().numpy(), dV[:, rows[j]]) <= hp.REL_TOL
    return step_pairs


def _local_block_rows(kind, G, N, N_blk):
    """Rows of a local block: a slice (or stripe) of a global block under the two balanced splits, a
    whole global block under the splits that keep consecutive tokens together."""
    return N_blk // G if kind in ("block_striped", "striped") else N_blk


@pytest.mark.parametrize("N_blk,window", [(512, 0), (384, 0), (512, 300), (384, 77), (2048, 0)])
def test_block_striped_causal_ring(lib, N_blk, window):
    """Pieces of 128, 96 and 512 rows (multiples of the tiles and not), 4 or more pieces a side, with and
    without a window: the many-piece tile walks and the per-element predicate across piece seams."""
    G = 4
    N = 3072 if N_blk == 384 else 4096
    _ring(lib, "block_striped", G, N, N_blk, 4, 2, 64 if N_blk == 384 else 128, seed=N_blk + window, window=window)


@pytest.mark.parametrize("kind", ["block_striped", "striped", "contiguous", "zigzag"])
@pytest.mark.parametrize("causal,window", [(False, 0), (True, 0), (True, 1500)])
def test_block_pattern_under_every_split(lib, kind, causal, window):
    """One global block pattern (blocks of N_blk tokens, diagonal open, one query block that otherwise
    sees little) under the four splits: each step's block mask is a gather of the pattern on local row
    blocks.  Under the two balanced splits and a pure block pattern every step of every device has the
    same number of visible pairs."""
    G = 4
    # local blocks must be multiples of 256 rows: slices of N_blk / G under the balanced splits
    N_blk = 1024 if kind in ("block_striped", "striped") else 256
    N = 8192 if kind in ("block_striped", "striped") else 4096
    nb = N // N_blk
    rng = np.random.Generator(np.random.PCG64(wl.BASE_SEED + 31000 + nb))
    pattern = (rng.random((nb, nb)) < 0.5).astype(np.uint8)
    np.fill_diagonal(pattern, 1)
    pattern[nb // 2, : nb // 2] = 0
    pairs = _ring(lib, kind, G, N, N_blk, 2, 2, 128, seed=50 + nb, causal=causal, window=window, pattern=pattern,
                  devices=None if kind in ("block_striped", "striped") else [1, 3])
    if kind in ("block_striped", "striped") and not causal:
        m = N_blk // G
        assert set(pairs.values()) == {int(pattern.sum()) * m * m}
