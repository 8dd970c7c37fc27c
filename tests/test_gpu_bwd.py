"""Backward parity on the GPU: burst_attn_preprocess_bwd / burst_attn_step_bwd through the C ABI
against the fp64 oracle, element by element, on the same seeded inputs."""
import numpy as np
import pytest

from oracle import burst_oracle as oc
from paper_2509_19836_amd import workloads as wl
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


def full_ring_case(lib, w, cfg_index, kind, travel="kv", window=0):
    """Whole simulated ring, every device: forward (fused merge), D, then all G*G backward steps.
    travel = "kv": Alg. 1 order (Q_i stays, dQ_i accumulates locally, dK_j/dV_j of the visiting
    chunk accumulate across devices); travel = "q": Alg. 2 order (K_i, V_i, dK_i, dV_i stay, the
    query bundles visit).  Compared with the unsharded oracle gradients."""
    torch = _torch()
    G, N = w.shards, w.seq
    T = wl.host_tensors(w, cfg_index)
    Q, K, V, dO = (hp.widen(T[n][1]) for n in ("q", "k", "v", "do"))
    causal = kind != "full"
    vis_glob = oc.visibility(np.arange(N), np.arange(N), causal, window)
    O_ref, lse_ref = oc.mha_attention_fwd(Q, K, V, w.scale, vis_glob)
    dQ_ref, dK_ref, dV_ref = oc.mha_attention_bwd(Q, K, V, dO, w.scale, vis_glob)
    D_ref = oc.mha_preprocess_bwd(dO, O_ref)
    dev = {n: hp.dev_bf16(T[n][1]) for n in ("q", "k", "v", "do")}
    rows = [hp.mask_positions(hp.fill_mask(lib, kind, i, i, G, N), "q") for i in range(G)]
    idx = [torch.from_numpy(r).cuda() for r in rows]
    n = rows[0].size
    sh = {i: {name: dev[name][:, idx[i]].contiguous() for name in dev} for i in range(G)}
    f32 = dict(device="cuda", dtype=torch.float32)
    lse, Dv = {}, {}
    for i in range(G):
        o_acc = torch.zeros(w.batch, n, w.q_heads, w.head_dim, **f32)
        lse_acc = torch.full((w.batch, w.q_heads, n), -float("inf"), **f32)
        for j in oc.ring_order(i, G):
            shp = lib.shape(w.batch, w.q_heads, w.kv_heads, w.head_dim, n, n, w.scale)
            lib.burst_attn_step_fwd(shp, hp.fill_mask(lib, kind, i, j, G, N, window), sh[i]["q"], sh[j]["k"], sh[j]["v"],
                                    o_acc=o_acc, lse_acc=lse_acc)
        d_i = torch.empty(w.batch, w.q_heads, n, **f32)
        lib.burst_attn_preprocess_bwd(lib.shape(w.batch, w.q_heads, w.kv_heads, w.head_dim, n, n, w.scale),
                                      o_acc, sh[i]["do"], d_i)
        lse[i], Dv[i] = lse_acc, d_i
        torch.cuda.synchronize()
        assert hp.lse_err(lse_acc.cpu().numpy(), lse_ref[:, :, rows[i]]) <= hp.LSE_TOL
        d_err = np.abs(d_i.cpu().numpy() - D_ref[:, :, rows[i]]).max() / np.abs(D_ref).max()
        assert d_err <= hp.REL_TOL, d_err
    dq = [torch.zeros(w.batch, n, w.q_heads, w.head_dim, **f32) for _ in range(G)]
    dk = [torch.zeros(w.batch, n, w.kv_heads, w.head_dim, **f32) for _ in range(G)]
    dv = [torch.zeros(w.batch, n, w.kv_heads, w.head_dim, **f32) for _ in range(G)]
    ALL = lib.BURST_ACC_DQ | lib.BURST_ACC_DK | lib.BURST_ACC_DV
    shp = lib.shape(w.batch, w.q_heads, w.kv_heads, w.head_dim, n, n, w.scale)
    for a in range(G):
        for t in range(G):
            # (i, j) = (query device, key device)
            i, j = (a, (a - t) % G) if travel == "kv" else ((a - t) % G, a)
            lib.burst_attn_step_bwd(shp, hp.fill_mask(lib, kind, i, j, G, N, window), sh[i]["q"], sh[j]["k"], sh[j]["v"],
                                    sh[i]["do"], lse[i], Dv[i], dq=dq[i], dk=dk[j], dv=dv[j],
                                    accumulate_flags=ALL)
    torch.cuda.synchronize()
    worst = {}
    for name, got, ref in (("dq", dq, dQ_ref), ("dk", dk, dK_ref), ("dv", dv, dV_ref)):
        full = np.zeros_like(ref)
        for i in range(G):
            full[:, rows[i]] = got[i].cpu().numpy()
        worst[name] = hp.rel_err(full, ref)
    print(f"\n[{w.name} {kind} travel={travel}] worst errors: {worst}", flush=True)
    for name, val in worst.items():
        assert val <= hp.REL_TOL, (name, val)


@pytest.mark.parametrize("kind", ["full", "causal", "zigzag"])
def test_config1_tiny_ring_backward(lib, kind):
    full_ring_case(lib, wl.WORKLOADS[1], 1, kind, travel="kv")


def test_config1_query_bundles_travel(lib):
    full_ring_case(lib, wl.WORKLOADS[1], 1, "causal", travel="q")


def test_config2_scaled_zigzag_d128_backward(lib):
    full_ring_case(lib, wl.Workload("cfg2_scaled", 1, 4, 4, 128, 512, 4, "zigzag"), 2, "zigzag")


def test_config3_scaled_gqa_backward(lib):
    full_ring_case(lib, wl.Workload("gqa_scaled", 1, 8, 2, 128, 384, 4, "zigzag"), 3, "zigzag", travel="q")


def test_config4_scaled_full_head_scales_backward(lib):
    full_ring_case(lib, wl.Workload("full_scaled", 2, 4, 4, 128, 640, 2, "full", True), 4, "full")


def test_striped_backward(lib):
    full_ring_case(lib, wl.Workload("striped", 1, 2, 2, 128, 320, 4, "striped"), 6, "striped")


@pytest.mark.parametrize("kind,window", [("causal", 1), ("causal", 100), ("causal", 300), ("zigzag", 64), ("zigzag", 200),
                                         ("striped", 37), ("striped", 500)])
def test_sliding_window_ring_backward(lib, kind, window):
    full_ring_case(lib, wl.WORKLOADS[1], 1, kind, window=window)


@pytest.mark.parametrize("d,window", [(64, 0), (128, 0), (128, 90)])
def test_zigzag_pieces_that_are_not_tile_multiples_backward(lib, d, window):
    for piece, G in ((100, 2), (150, 3)):
        w = wl.Workload(f"zigzag_piece{piece}", 1, 2, 2, d, 2 * piece, G, "zigzag")
        full_ring_case(lib, w, 6, "zigzag", window=window)


def test_sliding_window_scaled_config2_d128_backward(lib):
    w = wl.Workload("zigzag_window_d128", 1, 4, 4, 128, 512, 4, "zigzag")
    full_ring_case(lib, w, 2, "zigzag", window=w.seq // 4)


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("sq,sk,qoff", [(200, 333, 150), (1, 1, 0), (77, 64, 10), (129, 257, 300), (300, 130, 0)])
def test_ragged_single_step_backward(lib, d, sq, sk, qoff):
    """The step contract on odd sizes: any (lse, D) the caller passes, per-step outputs, overwrite
    versus accumulate, rows that see nothing."""
    torch = _torch()
    B, Hq, Hkv = 1, 4, 2
    rng = np.random.Generator(np.random.PCG64(wl.BASE_SEED + 9000 + sq * 1000 + sk + d))
    qb, kb, vb, gb = (wl.f32_to_bf16_bits(rng.standard_normal(s, dtype=np.float32))
                      for s in ((B, sq, Hq, d), (B, sk, Hkv, d), (B, sk, Hkv, d), (B, sq, Hq, d)))
    scale = 1.0 / np.sqrt(d)
    Qh, Kh, Vh, Gh = hp.widen(qb), hp.widen(kb), hp.widen(vb), hp.widen(gb)
    # lse and D as they would come out of a longer ring: larger than this step's own lse
    lse_h = (oc.mha_step_fwd(Qh, Kh, Vh, scale, None)[1] + rng.uniform(0.1, 1.0, (B, Hq, sq))).astype(np.float32)
    D_h = rng.standard_normal((B, Hq, sq)).astype(np.float32)
    f32 = dict(device="cuda", dtype=torch.float32)
    for causal in (False, True):
        mask = lib.burst_mask_t(int(causal), 1, 1, 0, (qoff, 0), (0, 0), sq, sk, 1)
        vis = oc.visibility(qoff + np.arange(sq), np.arange(sk), causal)
        dQ, dK, dV = oc.mha_step_bwd(Qh, Kh, Vh, Gh, lse_h.astype(np.float64), D_h.astype(np.float64), scale, vis)
        dq = torch.full((B, sq, Hq, d), 1.0, **f32)
        dk = torch.full((B, sk, Hkv, d), 2.0, **f32)
        dv = torch.full((B, sk, Hkv, d), float("nan"), **f32)
        shp = lib.shape(B, Hq, Hkv, d, sq, sk, scale)
        args = (shp, mask, hp.dev_bf16(qb), hp.dev_bf16(kb), hp.dev_bf16(vb), hp.dev_bf16(gb),
                torch.from_numpy(lse_h).cuda(), torch.from_numpy(D_h).cuda())
        lib.burst_attn_step_bwd(*args, dq=dq, dk=dk, dv=dv, accumulate_flags=lib.BURST_ACC_DQ | lib.BURST_ACC_DK)
        torch.cuda.synchronize()
        tol = lambda ref: hp.REL_TOL * max(np.abs(ref).max(), 1e-30)
        assert np.abs(dq.cpu().numpy() - 1.0 - dQ).max() <= tol(dQ)
        assert np.abs(dk.cpu().numpy() - 2.0 - dK).max() <= tol(dK)
        assert np.abs(dv.cpu().numpy() - dV).max() <= tol(dV)       # overwritten, NaN gone
        # dq alone, overwrite
        dq2 = torch.full((B, sq, Hq, d), float("nan"), **f32)
        lib.burst_attn_step_bwd(*args, dq=dq2)
        torch.cuda.synchronize()
        assert np.abs(dq2.cpu().numpy() - dQ).max() <= tol(dQ)


def test_backward_strided_views_and_guard_rows(lib):
    torch = _torch()
    B, S, H, d, pad = 1, 192, 2, 128, 64
    rng = np.random.Generator(np.random.PCG64(wl.BASE_SEED + 9500))
    big = {n: wl.f32_to_bf16_bits(rng.standard_normal((B, S + 2 * pad, H, d + 8), dtype=np.float32))
           for n in ("q", "k", "v", "g")}
    dev = {n: hp.dev_bf16(big[n]) for n in big}
    view = {n: dev[n][:, pad:pad + S, :, :d] for n in big}
    host = {n: hp.widen(big[n][:, pad:pad + S, :, :d]) for n in big}
    scale = 1.0 / np.sqrt(d)
    vis = oc.visibility(np.arange(S), np.arange(S), True)
    O, lse = oc.mha_attention_fwd(host["q"], host["k"], host["v"], scale, vis)
    D = oc.mha_preprocess_bwd(host["g"], O)
    dQ, dK, dV = oc.mha_step_bwd(host["q"], host["k"], host["v"], host["g"], lse, D, scale, vis)
    f32 = dict(device="cuda", dtype=torch.float32)
    outs = {n: torch.full((B, S + 2, H, d), 3.0, **f32) for n in ("dq", "dk", "dv")}
    lse_big = torch.full((B, H, S + 8), 9.0, **f32)
    d_big = torch.full((B, H, S + 8), 9.0, **f32)
    lse_big[:, :, 4:S + 4] = torch.from_numpy(lse.astype(np.float32)).cuda()
    d_big[:, :, 4:S + 4] = torch.from_numpy(D.astype(np.float32)).cuda()
    shp = lib.shape(B, H, H, d, S, S, scale)
    lib.burst_attn_step_bwd(shp, lib.burst_attn_fill_contiguous_mask(0, 0, 1, S, True), view["q"], view["k"],
                            view["v"], view["g"], lse_big[:, :, 4:S + 4], d_big[:, :, 4:S + 4],
                            dq=outs["dq"][:, 1:S + 1], dk=outs["dk"][:, 1:S + 1], dv=outs["dv"][:, 1:S + 1])
    torch.cuda.synchronize()
    for n, ref in (("dq", dQ), ("dk", dK), ("dv", dV)):
        assert hp.rel_err(outs[n][:, 1:S + 1].cpu().numpy(), ref) <= hp.REL_TOL, n
        assert (outs[n][:, 0] == 3.0).all() and (outs[n][:, S + 1] == 3.0).all(), n


def test_backward_empty_chunks(lib):
    torch = _torch()
    B, H, d = 1, 2, 64
    bf = dict(device="cuda", dtype=torch.bfloat16)
    q = torch.zeros(B, 16, H, d, **bf)
    lse = torch.zeros(B, H, 16, device="cuda")
    dq = torch.full((B, 16, H, d), 5.0, device="cuda")
    dk = torch.full((B, 16, H, d), 5.0, device="cuda")
    dv = torch.full((B, 16, H, d), 5.0, device="cuda")
    # no key rows: dq overwritten with zero, or left alone when accumulating
    shp = lib.shape(B, H, H, d, 16, 0, 0.125)
    lib.burst_attn_step_bwd(shp, None, q, q, q, q, lse, lse, dq=dq)
    torch.cuda.synchronize()
    assert (dq == 0).all()
    dq.fill_(5.0)
    lib.burst_attn_step_bwd(shp, None, q, q, q, q, lse, lse, dq=dq, accumulate_flags=lib.BURST_ACC_DQ)
    torch.cuda.synchronize()
    assert (dq == 5.0).all()
    # no query rows: dk / dv zeroed
    shp = lib.shape(B, H, H, d, 0, 16, 0.125)
    lib.burst_attn_step_bwd(shp, None, q, q, q, q, lse, lse, dk=dk, dv=dv)
    torch.cuda.synchronize()
    assert (dk == 0).all() and (dv == 0).all()
