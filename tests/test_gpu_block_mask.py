"""Block-wise sparse masks (Sec. 3.4) through the C-ABI against the oracle: visibility is the mode's
predicate AND the byte of the (query block, key block) pair.  Sizes span several blocks with ragged
tails; masks include closed query-block rows and closed key-block columns."""
import numpy as np
import pytest

from oracle import burst_oracle as oc
from paper_2509_19836_amd import workloads as wl
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    return torch


def _random_blocks(rng, nq, nk, density, closed_row=None, closed_col=None):
    bm = (rng.random((nq, nk)) < density).astype(np.uint8)
    bm *= rng.integers(1, 256, size=bm.shape, dtype=np.uint8)   # any nonzero byte means open
    if closed_row is not None:
        bm[closed_row, :] = 0
    if closed_col is not None:
        bm[:, closed_col] = 0
    return bm


def _mask_cases(lib, sq, sk):
    """(name, burst_mask_t, positions of q rows, positions of k rows, causal, window)."""
    ar = np.arange
    yield "full", lib.burst_mask_t(0, 1, 1, 0, (0, 0), (0, 0), sq, sk, 1), ar(sq), ar(sk), False, 0
    yield "causal", lib.burst_mask_t(1, 1, 1, 0, (sk // 3, 0), (0, 0), sq, sk, 1), sk // 3 + ar(sq), ar(sk), True, 0
    yield "window", lib.burst_mask_t(1, 1, 1, 0, (sk // 3, 0), (0, 0), sq, sk, 1, 300), sk // 3 + ar(sq), ar(sk), True, 300
    if sq % 2 == 0 and sk % 2 == 0:   # two zigzag pieces a side
        hq, hk = sq // 2, sk // 2
        qp = np.concatenate([hk + ar(hq), 5 * hk + ar(hq)])
        kp = np.concatenate([ar(hk), 4 * hk + hq // 2 + ar(hk)])
        yield "zigzag", lib.burst_mask_t(1, 2, 2, 0, (hk, 5 * hk), (0, 4 * hk + hq // 2), hq, hk, 1), qp, kp, True, 0


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("sq,sk,bq,bk", [(700, 900, 256, 128), (1024, 1100, 512, 256), (300, 130, 256, 128)])
def test_block_sparse_single_step_forward_and_backward(lib, d, sq, sk, bq, bk):
    torch = _torch()
    B, Hq, Hkv = 2, 4, 2
    rng = np.random.Generator(np.random.PCG64(wl.BASE_SEED + 12000 + sq * 1000 + sk + d))
    qb, kb, vb, gb = (wl.f32_to_bf16_bits(rng.standard_normal(s, dtype=np.float32))
                      for s in ((B, sq, Hq, d), (B, sk, Hkv, d), (B, sk, Hkv, d), (B, sq, Hq, d)))
    scale = 1.0 / np.sqrt(d)
    Qh, Kh, Vh, Gh = hp.widen(qb), hp.widen(kb), hp.widen(vb), hp.widen(gb)
    lse_h = (oc.mha_step_fwd(Qh, Kh, Vh, scale, None)[1] + rng.uniform(0.1, 1.0, (B, Hq, sq))).astype(np.float32)
    D_h = rng.standard_normal((B, Hq, sq)).astype(np.float32)
    nq, nk = -(-sq // bq), -(-sk // bk)
    f32 = dict(device="cuda", dtype=torch.float32)
    shp = lib.shape(B, Hq, Hkv, d, sq, sk, scale)
    tol = lambda ref: hp.REL_TOL * max(np.abs(ref).max(), 1e-30)
    for n, (name, mask, qpos, kpos, causal, window) in enumerate(_mask_cases(lib, sq, sk)):
        bm = _random_blocks(rng, nq, nk, 0.5, closed_row=(n % nq) if nq > 1 else None, closed_col=n % nk)
        # a pitch wider than the row, the padding nonzero: it must never be read as a block
        bm_dev = torch.full((nq, nk + 3), 255, dtype=torch.uint8, device="cuda")
        bm_dev[:, :nk] = torch.from_numpy(bm).cuda()
        lib.set_block_mask(mask, bm_dev[:, :nk], bq, bk)
        vis = oc.apply_block_mask(oc.visibility(qpos, kpos, causal, window), bm, bq, bk)
        O_s, lse_s = oc.mha_step_fwd(Qh, Kh, Vh, scale, vis)
        o_part = torch.full((B, sq, Hq, d), 7.0, **f32)
        lse_part = torch.full((B, Hq, sq), 7.0, **f32)
        print(f"block mask fwd {name} d={d} sq={sq} sk={sk} bq={bq} bk={bk}", flush=True)
        lib.burst_attn_step_fwd(shp, mask, hp.dev_bf16(qb), hp.dev_bf16(kb), hp.dev_bf16(vb),
                                o_part=o_part, lse_part=lse_part)
        torch.cuda.synchronize()
        assert hp.rel_err(o_part.cpu().numpy(), O_s) <= hp.REL_TOL, name
        assert hp.lse_err(lse_part.cpu().numpy(), lse_s) <= hp.LSE_TOL, name

        dQ, dK, dV = oc.mha_step_bwd(Qh, Kh, Vh, Gh, lse_h.astype(np.float64), D_h.astype(np.float64), scale, vis)
        dq = torch.full((B, sq, Hq, d), float("nan"), **f32)
        dk = torch.full((B, sk, Hkv, d), 2.0, **f32)
        dv = torch.full((B, sk, Hkv, d), float("nan"), **f32)
        print(f"block mask bwd {name}", flush=True)
        lib.burst_attn_step_bwd(shp, mask, hp.dev_bf16(qb), hp.dev_bf16(kb), hp.dev_bf16(vb), hp.dev_bf16(gb),
                                torch.from_numpy(lse_h).cuda(), torch.from_numpy(D_h).cuda(),
                                dq=dq, dk=dk, dv=dv, accumulate_flags=lib.BURST_ACC_DK)
        torch.cuda.synchronize()
        assert np.abs(dq.cpu().numpy() - dQ).max() <= tol(dQ), name
        assert np.abs(dk.cpu().numpy() - 2.0 - dK).max() <= tol(dK), name
        assert np.abs(dv.cpu().numpy() - dV).max() <= tol(dV), name


def test_all_open_block_mask_equals_no_block_mask(lib):
    """An all-ones block mask changes nothing, bit for bit (same tiles, same order)."""
    torch = _torch()
    B, Hq, Hkv, d, sq, sk = 1, 4, 2, 128, 640, 768
    rng = np.random.Generator(np.random.PCG64(wl.BASE_SEED + 12500))
    q, k, v = (hp.dev_bf16(wl.f32_to_bf16_bits(rng.standard_normal(s, dtype=np.float32)))
               for s in ((B, sq, Hq, d), (B, sk, Hkv, d), (B, sk, Hkv, d)))
    shp = lib.shape(B, Hq, Hkv, d, sq, sk, 0.1)
    outs = []
    for with_blocks in (False, True):
        mask = lib.burst_mask_t(1, 1, 1, 0, (200, 0), (0, 0), sq, sk, 1)
        if with_blocks:
            bm = torch.ones((3, 6), dtype=torch.uint8, device="cuda")
            lib.set_block_mask(mask, bm, 256, 128)
        o = torch.empty((B, sq, Hq, d), device="cuda", dtype=torch.float32)
        lse = torch.empty((B, Hq, sq), device="cuda", dtype=torch.float32)
        lib.burst_attn_step_fwd(shp, mask, q, k, v, o_part=o, lse_part=lse)
        torch.cuda.synchronize()
        outs.append((o.cpu().numpy(), lse.cpu().numpy()))
    assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1])


def test_all_closed_block_mask(lib):
    """Nothing visible: the step result is (0, -inf), the running state and accumulated gradients
    stay as they were, overwritten gradients become zero."""
    torch = _torch()
    B, Hq, Hkv, d, sq, sk = 1, 2, 2, 64, 512, 384
    rng = np.random.Generator(np.random.PCG64(wl.BASE_SEED + 12600))
    q, k, v, g = (hp.dev_bf16(wl.f32_to_bf16_bits(rng.standard_normal(s, dtype=np.float32)))
                  for s in ((B, sq, Hq, d), (B, sk, Hkv, d), (B, sk, Hkv, d), (B, sq, Hq, d)))
    shp = lib.shape(B, Hq, Hkv, d, sq, sk, 0.125)
    mask = lib.burst_mask_t(0, 1, 1, 0, (0, 0), (0, 0), sq, sk, 1)
    bm = torch.zeros((2, 3), dtype=torch.uint8, device="cuda")
    lib.set_block_mask(mask, bm, 256, 128)
    f32 = dict(device="cuda", dtype=torch.float32)
    o, lse = torch.full((B, sq, Hq, d), 7.0, **f32), torch.full((B, Hq, sq), 7.0, **f32)
    o_acc, lse_acc = torch.full((B, sq, Hq, d), 3.0, **f32), torch.full((B, Hq, sq), 0.5, **f32)
    lib.burst_attn_step_fwd(shp, mask, q, k, v, o_part=o, lse_part=lse, o_acc=o_acc, lse_acc=lse_acc)
    torch.cuda.synchronize()
    assert (o == 0).all() and torch.isneginf(lse).all()
    assert (o_acc == 3.0).all() and (lse_acc == 0.5).all()
    dq, dk, dv = torch.full((B, sq, Hq, d), 1.0, **f32), torch.full((B, sk, Hkv, d), 2.0, **f32), \
        torch.full((B, sk, Hkv, d), float("nan"), **f32)
    lib.burst_attn_step_bwd(shp, mask, q, k, v, g, torch.zeros((B, Hq, sq), **f32), torch.zeros((B, Hq, sq), **f32),
                            dq=dq, dk=dk, dv=dv, accumulate_flags=lib.BURST_ACC_DQ | lib.BURST_ACC_DK)
    torch.cuda.synchronize()
    assert (dq == 1.0).all() and (dk == 2.0).all() and (dv == 0).all()


def test_block_sparse_accumulated_over_shards(lib):
    """Three key/value shards with their own block masks folded into one running state equal the
    oracle's attention over the concatenated keys with the concatenated mask."""
    torch = _torch()
    B, Hq, Hkv, d, sq, sk, G = 1, 4, 4, 128, 512, 512, 3
    bq, bk = 256, 128
    rng = np.random.Generator(np.random.PCG64(wl.BASE_SEED + 12700))
    qb = wl.f32_to_bf16_bits(rng.standard_normal((B, sq, Hq, d), dtype=np.float32))
    kbs = [wl.f32_to_bf16_bits(rng.standard_normal((B, sk, Hkv, d), dtype=np.float32)) for _ in range(G)]
    vbs = [wl.f32_to_bf16_bits(rng.standard_normal((B, sk, Hkv, d), dtype=np.float32)) for _ in range(G)]
    scale = 1.0 / np.sqrt(d)
    qpos = 2 * sk + np.arange(sq)            # the query chunk is the last of the three in position
    f32 = dict(device="cuda", dtype=torch.float32)
    o_acc = torch.zeros((B, sq, Hq, d), **f32)
    lse_acc = torch.full((B, Hq, sq), float("-inf"), **f32)
    shp = lib.shape(B, Hq, Hkv, d, sq, sk, scale)
    vis_all, keep = [], []
    for j in range(G):
        bm = _random_blocks(rng, sq // bq, sk // bk, 0.6)
        if j == G - 1:
            bm[np.arange(sq // bq), np.arange(sq // bq) * (bq // bk)] = 1   # every row keeps a causal key
        bm_dev = torch.from_numpy(bm).cuda()
        keep.append(bm_dev)
        mask = lib.burst_mask_t(1, 1, 1, 0, (2 * sk, 0), (j * sk, 0), sq, sk, 1)
        lib.set_block_mask(mask, bm_dev, bq, bk)
        lib.burst_attn_step_fwd(shp, mask, hp.dev_bf16(qb), hp.dev_bf16(kbs[j]), hp.dev_bf16(vbs[j]),
                                o_acc=o_acc, lse_acc=lse_acc)
        vis_all.append(oc.apply_block_mask(oc.visibility(qpos, j * sk + np.arange(sk), True), bm, bq, bk))
    torch.cuda.synchronize()
    K = np.concatenate([hp.widen(x) for x in kbs], axis=1)
    V = np.concatenate([hp.widen(x) for x in vbs], axis=1)
    O_ref, lse_ref = oc.mha_step_fwd(hp.widen(qb), K, V, scale, np.concatenate(vis_all, axis=1))
    assert hp.rel_err(o_acc.cpu().numpy(), O_ref) <= hp.REL_TOL
    assert hp.lse_err(lse_acc.cpu().numpy(), lse_ref) <= hp.LSE_TOL
