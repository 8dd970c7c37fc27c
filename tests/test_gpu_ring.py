"""The simulated ring driver (paper_2509_19836_amd/ring.py: the host loop of one device's pass over
all KV shards, own shard first, then j = (i - t) mod G; forward algorithm and Alg. 1) on config 1,
every device, against the unsharded fp64 oracle; run-to-run determinism of the backward step; the
standalone merge's bf16 copy; a running state that starts as (garbage, -inf)."""
import numpy as np
import pytest

from oracle import burst_oracle as oc
from paper_2509_19836_amd import workloads as wl
from tests import helpers as hp

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("kind", ["full", "causal", "zigzag", "striped"])
def test_ring_driver_config1_all_devices_vs_unsharded_oracle(lib, kind):
    import torch
    from paper_2509_19836_amd import ring
    w = wl.WORKLOADS[1]
    G, N = w.shards, w.seq
    T = wl.host_tensors(w, 1)
    host = {n: hp.widen(T[n][1]) for n in T}
    dev = {n: hp.dev_bf16(T[n][1]) for n in T}
    rows = [hp.oracle_positions(oc, kind, j, G, N) for j in range(G)]
    idx = [torch.from_numpy(r).cuda() for r in rows]
    n = rows[0].size
    shard = lambda name, j: dev[name][:, idx[j]].contiguous()
    ks, vs = [shard("k", j) for j in range(G)], [shard("v", j) for j in range(G)]
    f32 = dict(device="cuda", dtype=torch.float32)
    vis = oc.visibility(np.arange(N), np.arange(N), kind != "full")
    O, lse = oc.mha_attention_fwd(host["q"], host["k"], host["v"], w.scale, vis)
    dQ, dK, dV = oc.mha_attention_bwd(host["q"], host["k"], host["v"], host["do"], w.scale, vis)
    # dK_j / dV_j travel with the shard and collect every device's contribution (Alg. 1)
    dks = [torch.zeros(w.batch, n, w.kv_heads, w.head_dim, **f32) for _ in range(G)]
    dvs = [torch.zeros(w.batch, n, w.kv_heads, w.head_dim, **f32) for _ in range(G)]
    for i in range(G):
        print(f"ring {kind} device {i}", flush=True)
        q_i, do_i = shard("q", i), shard("do", i)
        o_acc = torch.zeros(w.batch, n, w.q_heads, w.head_dim, **f32)
        lse_acc = torch.full((w.batch, w.q_heads, n), -float("inf"), **f32)
        ring.ring_forward(i, G, N, kind, w.scale, q_i, ks, vs, o_acc, lse_acc)
        d_i = torch.empty(w.batch, w.q_heads, n, **f32)
        dq = torch.zeros(w.batch, n, w.q_heads, w.head_dim, **f32)
        ring.ring_backward(i, G, N, kind, w.scale, q_i, do_i, o_acc, lse_acc, d_i, ks, vs, dq, dks, dvs)
        torch.cuda.synchronize()
        assert hp.rel_err(o_acc.cpu().numpy(), O[:, rows[i]]) <= hp.REL_TOL
        assert hp.lse_err(lse_acc.cpu().numpy(), lse[:, :, rows[i]]) <= hp.LSE_TOL
        assert hp.rel_err(dq.cpu().numpy(), dQ[:, rows[i]]) <= hp.REL_TOL
    for j in range(G):
        assert hp.rel_err(dks[j].cpu().numpy(), dK[:, rows[j]]) <= hp.REL_TOL
        assert hp.rel_err(dvs[j].cpu().numpy(), dV[:, rows[j]]) <= hp.REL_TOL


def test_backward_step_is_run_to_run_identical(lib):
    """No kernel of the backward step adds into memory that another work-group also adds into, so two
    calls on the same inputs must agree bit for bit (overwrite and accumulate-into-zero alike)."""
    import torch
    B, n, Hq, Hkv, d, G, i, j = 1, 2048, 8, 2, 128, 4, 2, 2
    N = n * G
    gen = torch.Generator(device="cuda")
    gen.manual_seed(wl.BASE_SEED + 808)
    draw = lambda heads: torch.randn(B, n, heads, d, device="cuda", generator=gen).to(torch.bfloat16)
    q, do, k, v = draw(Hq), draw(Hq), draw(Hkv), draw(Hkv)
    lse = 4.0 + torch.rand(B, Hq, n, device="cuda", generator=gen)
    dvec = torch.randn(B, Hq, n, device="cuda", generator=gen)
    mask = lib.burst_attn_fill_zigzag_mask(i, j, G, N)
    shp = lib.shape(B, Hq, Hkv, d, n, n, d ** -0.5)
    runs = []
    for rep in range(3):
        f32 = dict(device="cuda", dtype=torch.float32)
        fill = float("nan") if rep < 2 else 0.0
        dq, dk, dv = (torch.full((B, n, h_, d), fill, **f32) for h_ in (Hq, Hkv, Hkv))
        lib.burst_attn_step_bwd(shp, mask, q, k, v, do, lse, dvec, dq=dq, dk=dk, dv=dv,
                                accumulate_flags=0 if rep < 2 else 7)
        torch.cuda.synchronize()
        runs.append([t.cpu().numpy() for t in (dq, dk, dv)])
    for a, b, c in zip(*runs):
        assert np.isfinite(a).all()
        assert np.array_equal(a, b) and np.array_equal(a, c)


def test_merge_writes_the_bf16_copy_and_ignores_a_dead_running_state(lib):
    """burst_attn_lse_merge with o_out_cast, and both merge paths (standalone, fused in the step) on a
    first step whose running state is (NaN garbage, -inf): weight zero, never read as a number."""
    import torch
    w = wl.WORKLOADS[1]
    T = wl.host_tensors(w, 1, seed_offset=3)
    n = 256
    Q, K, V = (hp.widen(T[x][1])[:, :n] for x in ("q", "k", "v"))
    q, k, v = (hp.dev_bf16(T[x][1])[:, :n].contiguous() for x in ("q", "k", "v"))
    shp = lib.shape(w.batch, w.q_heads, w.kv_heads, w.head_dim, n, n, w.scale)
    mask = lib.burst_attn_fill_contiguous_mask(0, 0, 1, n, True)
    O_ref, lse_ref = oc.mha_step_fwd(Q, K, V, w.scale, oc.visibility(np.arange(n), np.arange(n), True))
    f32 = dict(device="cuda", dtype=torch.float32)
    o_part = torch.empty(w.batch, n, w.q_heads, w.head_dim, **f32)
    lse_part = torch.empty(w.batch, w.q_heads, n, **f32)
    lib.burst_attn_step_fwd(shp, mask, q, k, v, o_part=o_part, lse_part=lse_part)
    for path in ("standalone", "fused"):
        o_acc = torch.full((w.batch, n, w.q_heads, w.head_dim), float("nan"), **f32)
        lse_acc = torch.full((w.batch, w.q_heads, n), -float("inf"), **f32)
        o_bf16 = torch.full((w.batch, n, w.q_heads, w.head_dim), 7.0, device="cuda", dtype=torch.bfloat16)
        if path == "standalone":
            lib.burst_attn_lse_merge(shp, o_acc, lse_acc, o_part, lse_part, o_out_cast=o_bf16)
        else:
            lib.burst_attn_step_fwd(shp, mask, q, k, v, o_acc=o_acc, lse_acc=lse_acc)
        torch.cuda.synchronize()
        assert torch.isfinite(o_acc).all(), path
        assert hp.rel_err(o_acc.cpu().numpy(), O_ref) <= hp.REL_TOL
        assert hp.lse_err(lse_acc.cpu().numpy(), lse_ref) <= hp.LSE_TOL
        if path == "standalone":   # the bf16 copy is the merged fp32 value rounded once
            assert torch.equal(o_bf16, o_acc.to(torch.bfloat16))
    # a second merge of the same partial: (O, Lse) (+) (O, Lse) = (O, Lse + log 2), bf16 copy refreshed
    o_acc = o_part.clone()
    lse_acc = lse_part.clone()
    o_bf16 = torch.zeros(w.batch, n, w.q_heads, w.head_dim, device="cuda", dtype=torch.bfloat16)
    lib.burst_attn_lse_merge(shp, o_acc, lse_acc, o_part, lse_part, o_out_cast=o_bf16)
    torch.cuda.synchronize()
    assert hp.rel_err(o_acc.cpu().numpy(), O_ref) <= hp.REL_TOL
    assert hp.lse_err(lse_acc.cpu().numpy(), lse_ref + np.log(2.0)) <= hp.LSE_TOL
    assert torch.equal(o_bf16, o_acc.to(torch.bfloat16))
