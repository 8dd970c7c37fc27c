"""Seeded random mask descriptors through the whole step: what the hand-picked cases of the other files might
miss.  Each seed draws a head layout (d 64 / 128, batch, GQA group), for each axis a number of equal pieces with
its own length, first position and period, a position stride, causal or full visibility, maybe a sliding window,
maybe a block-wise sparse mask, and for every other seed lowers the range length so that the launches are cut
into ranges.  One forward step (the step result, and the same step folded into a live running state) and one
backward step (overwriting or accumulating, drawn per seed) are compared element by element with the oracle on
the visibility the descriptor means (positions rebuilt here from the descriptor's fields, not by the library)."""
import numpy as np
import pytest

from oracle import burst_oracle as oc
from paper_2509_19836_amd import workloads as wl
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def _axis(rng, stride):
    nseg = int(rng.choice([1, 1, 2, 3, 5]))
    seg_len = int(rng.integers(32, 260)) if nseg > 2 else int(rng.integers(1, 640))
    if rng.random() < 0.25:
        seg_len = int(rng.choice([64, 128, 256]))
    pos0 = int(rng.integers(0, 3000))
    period = (seg_len - 1) * stride + 1 + int(rng.integers(0, 2 * seg_len * stride + 1)) if nseg > 1 else 0
    return nseg, seg_len, pos0, period


@pytest.mark.parametrize("seed", range(48))
def test_random_descriptor_step_against_the_oracle(lib, seed):
    import torch
    rng = np.random.Generator(np.random.PCG64(wl.BASE_SEED + 52000 + seed))
    d = int(rng.choice([64, 128]))
    B, Hkv, group = int(rng.choice([1, 2])), int(rng.choice([1, 2])), int(rng.choice([1, 2, 4]))
    Hq = Hkv * group
    stride = int(rng.choice([1, 1, 2, 5]))
    q_nseg, q_len, q_pos0, q_per = _axis(rng, stride)
    k_nseg, k_len, k_pos0, k_per = _axis(rng, stride)
    if rng.random() < 0.3:
        k_pos0 = q_pos0   # diagonals that start in the same place
    sq, sk = q_nseg * q_len, k_nseg * k_len
    causal = bool(rng.random() < 0.75)
    window = int(rng.integers(1, 2 * max(sq, sk) * stride)) if causal and rng.random() < 0.4 else 0
    mask = lib.burst_mask_t()
    mask.mode = lib.BURST_MASK_CAUSAL if causal else lib.BURST_MASK_FULL
    mask.q_nseg, mask.k_nseg = q_nseg, k_nseg
    mask.q_seg_pos[0], mask.q_seg_pos[1] = q_pos0, q_pos0 + q_per
    mask.k_seg_pos[0], mask.k_seg_pos[1] = k_pos0, k_pos0 + k_per
    mask.q_seg_len, mask.k_seg_len, mask.pos_stride, mask.window = q_len, k_len, stride, window
    pos_q = np.concatenate([q_pos0 + s * q_per + np.arange(q_len, dtype=np.int64) * stride for s in range(q_nseg)])
    pos_k = np.concatenate([k_pos0 + s * k_per + np.arange(k_len, dtype=np.int64) * stride for s in range(k_nseg)])
    vis = oc.visibility(pos_q, pos_k, causal, window)
    blocks = None
    if rng.random() < 0.35:
        bq, bk = int(rng.choice([256, 512])), int(rng.choice([128, 256]))
        blocks_h = (rng.random((-(-sq // bq), -(-sk // bk))) < 0.6).astype(np.uint8)
        blocks = torch.from_numpy(blocks_h).cuda()
        lib.set_block_mask(mask, blocks, bq, bk)
        vis = oc.apply_block_mask(vis, blocks_h, bq, bk)
    small_ranges = seed % 2 == 1
    desc = (f"seed {seed}: d={d} B={B} heads={Hq}/{Hkv} q={q_nseg}x{q_len}@{q_pos0}+{q_per} k={k_nseg}x{k_len}@{k_pos0}+{k_per} "
            f"stride={stride} causal={causal} window={window} blocks={blocks is not None} small_ranges={small_ranges}")
    print(desc, flush=True)

    draw = lambda *shape: wl.f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32))
    qb, kb, vb, gb = draw(B, sq, Hq, d), draw(B, sk, Hkv, d), draw(B, sk, Hkv, d), draw(B, sq, Hq, d)
    Q, K, V, G = hp.widen(qb), hp.widen(kb), hp.widen(vb), hp.widen(gb)
    q, k, v, g = hp.dev_bf16(qb), hp.dev_bf16(kb), hp.dev_bf16(vb), hp.dev_bf16(gb)
    scale = 1.0 / float(np.sqrt(d))
    shp = lib.shape(B, Hq, Hkv, d, sq, sk, scale)
    f32 = dict(device="cuda", dtype=torch.float32)
    if small_ranges:
        assert lib.burst_attn_set_chunk_rows(256) == 256
    try:
        # forward: the step's own result, and the step folded into a running state that is live for some rows
        O_ref, lse_ref = oc.mha_step_fwd(Q, K, V, scale, vis)
        o_part = torch.full((B, sq, Hq, d), 7.0, **f32)
        lse_part = torch.full((B, Hq, sq), 7.0, **f32)
        lib.burst_attn_step_fwd(shp, mask, q, k, v, o_part=o_part, lse_part=lse_part)
        O_old = rng.standard_normal((B, sq, Hq, d)).astype(np.float32)
        lse_old = rng.uniform(-2.0, 6.0, (B, Hq, sq)).astype(np.float32)
        lse_old[rng.random((B, Hq, sq)) < 0.3] = -np.inf
        O_old[np.transpose(lse_old == -np.inf, (0, 2, 1))] = 0.0
        o_acc, lse_acc = torch.from_numpy(O_old).cuda(), torch.from_numpy(lse_old).cuda()
        lib.burst_attn_step_fwd(shp, mask, q, k, v, o_acc=o_acc, lse_acc=lse_acc)
        torch.cuda.synchronize()
        assert hp.rel_err(o_part.cpu().numpy(), O_ref) <= hp.REL_TOL, desc
        assert hp.lse_err(lse_part.cpu().numpy(), lse_ref) <= hp.LSE_TOL, desc
        O_m, lse_m = oc.mha_lse_merge(O_old.astype(np.float64), lse_old.astype(np.float64), O_ref, lse_ref)
        assert hp.rel_err(o_acc.cpu().numpy(), O_m) <= hp.REL_TOL, desc
        assert hp.lse_err(lse_acc.cpu().numpy(), lse_m) <= hp.LSE_TOL, desc

        # backward with the Lse a longer ring would hand over (above this step's own) and some D
        lse_in = (oc.mha_step_fwd(Q, K, V, scale, None)[1] + rng.uniform(0.1, 1.0, (B, Hq, sq))).astype(np.float32)
        D_in = rng.standard_normal((B, Hq, sq)).astype(np.float32)
        dQ, dK, dV = oc.mha_step_bwd(Q, K, V, G, lse_in.astype(np.float64), D_in.astype(np.float64), scale, vis)
        flags = int(rng.integers(0, 8))
        start = [rng.standard_normal(s).astype(np.float32) for s in ((B, sq, Hq, d), (B, sk, Hkv, d), (B, sk, Hkv, d))]
        dq, dk, dv = (torch.from_numpy(x).cuda() if flags >> n & 1 else torch.full(x.shape, float("nan"), **f32)
                      for n, x in enumerate(start))
        lib.burst_attn_step_bwd(shp, mask, q, k, v, g, torch.from_numpy(lse_in).cuda(), torch.from_numpy(D_in).cuda(),
                                dq=dq, dk=dk, dv=dv, accumulate_flags=flags)
        torch.cuda.synchronize()
        for n, (name, got, ref) in enumerate((("dQ", dq, dQ), ("dK", dk, dK), ("dV", dv, dV))):
            prior = start[n].astype(np.float64) if flags >> n & 1 else 0.0
            err = np.abs(got.cpu().numpy() - prior - ref).max()
            assert err <= hp.REL_TOL * max(np.abs(ref).max(), 1e-30), (name, err, desc)
    finally:
        if small_ranges:
            lib.burst_attn_set_chunk_rows(32768)
