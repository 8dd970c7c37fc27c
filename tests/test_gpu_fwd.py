"""Forward parity on the GPU: burst_attn_step_fwd / burst_attn_lse_merge through the C ABI against
the fp64 oracle, element by element, on the same seeded inputs."""
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


def ring_case(lib, w, cfg_index, kind, devices, o_part_dtype="f32", reverse=False, window=0):
    """All ring steps of the given devices: per-step partials vs oracle.step_fwd, fused running state
    and the standalone merge vs the unsharded oracle."""
    torch = _torch()
    G, N = w.shards, w.seq
    T = wl.host_tensors(w, cfg_index)
    Q, K, V = (hp.widen(T[n][1]) for n in ("q", "k", "v"))
    causal = kind != "full"
    vis_glob = oc.visibility(np.arange(N), np.arange(N), causal, window)
    O_ref, lse_ref = oc.mha_attention_fwd(Q, K, V, w.scale, vis_glob)
    qd, kd, vd = (hp.dev_bf16(T[n][1]) for n in ("q", "k", "v"))
    worst = {"o_part": 0.0, "lse_part": 0.0, "o_fused": 0.0, "lse_fused": 0.0, "o_merge": 0.0, "lse_merge": 0.0}
    for i in devices:
        m0 = hp.fill_mask(lib, kind, i, i, G, N)
        qrows = hp.mask_positions(m0, "q")
        assert (qrows == hp.oracle_positions(oc, kind, i, G, N)).all()
        n = qrows.size
        q_i = qd[:, torch.from_numpy(qrows).cuda()].contiguous()
        o_acc = torch.zeros(w.batch, n, w.q_heads, w.head_dim, device="cuda", dtype=torch.float32)
        lse_acc = torch.full((w.batch, w.q_heads, n), -float("inf"), device="cuda", dtype=torch.float32)
        o_acc2, lse_acc2 = o_acc.clone(), lse_acc.clone()
        for j in oc.ring_order(i, G, reverse):
            mask = hp.fill_mask(lib, kind, i, j, G, N, window)
            krows = hp.mask_positions(mask, "k")
            kidx = torch.from_numpy(krows).cuda()
            k_j, v_j = kd[:, kidx].contiguous(), vd[:, kidx].contiguous()
            shp = lib.shape(w.batch, w.q_heads, w.kv_heads, w.head_dim, n, krows.size, w.scale)
            o_part = torch.empty(w.batch, n, w.q_heads, w.head_dim, device="cuda",
                                 dtype=torch.float32 if o_part_dtype == "f32" else torch.bfloat16)
            lse_part = torch.empty(w.batch, w.q_heads, n, device="cuda", dtype=torch.float32)
            lib.burst_attn_step_fwd(shp, mask, q_i, k_j, v_j, o_part=o_part, lse_part=lse_part)
            lib.burst_attn_step_fwd(shp, mask, q_i, k_j, v_j, o_acc=o_acc, lse_acc=lse_acc)
            lib.burst_attn_lse_merge(shp, o_acc2, lse_acc2, o_part, lse_part)
            torch.cuda.synchronize()
            vis = oc.visibility(qrows, krows, causal, window)
            O_s, lse_s = oc.mha_step_fwd(Q[:, qrows], K[:, krows], V[:, krows], w.scale, vis)
            worst["o_part"] = max(worst["o_part"], hp.rel_err(o_part.float().cpu().numpy(), O_s))
            worst["lse_part"] = max(worst["lse_part"], hp.lse_err(lse_part.cpu().numpy(), lse_s))
        worst["o_fused"] = max(worst["o_fused"], hp.rel_err(o_acc.cpu().numpy(), O_ref[:, qrows]))
        worst["lse_fused"] = max(worst["lse_fused"], hp.lse_err(lse_acc.cpu().numpy(), lse_ref[:, :, qrows]))
        worst["o_merge"] = max(worst["o_merge"], hp.rel_err(o_acc2.cpu().numpy(), O_ref[:, qrows]))
        worst["lse_merge"] = max(worst["lse_merge"], hp.lse_err(lse_acc2.cpu().numpy(), lse_ref[:, :, qrows]))
    print(f"\n[{w.name} {kind} window {window}] worst errors: {worst}", flush=True)
    for kname, val in worst.items():
        assert val <= (hp.LSE_TOL if kname.startswith("lse") else hp.REL_TOL), (kname, val)


@pytest.mark.parametrize("kind", ["full", "causal", "zigzag"])
def test_config1_tiny_ring_all_devices(lib, kind):
    ring_case(lib, wl.WORKLOADS[1], 1, kind, devices=range(4))


def test_config1_reverse_order_and_bf16_partials(lib):
    ring_case(lib, wl.WORKLOADS[1], 1, "causal", devices=[0, 2], o_part_dtype="bf16", reverse=True)


def test_config2_scaled_zigzag_d128(lib):
    w = wl.scaled_down(wl.WORKLOADS[2], 512, q_heads=4, kv_heads=4)
    w = wl.Workload(w.name, 1, 4, 4, 128, 512, 4, "zigzag")
    ring_case(lib, w, 2, "zigzag", devices=[0, 1, 3])


def test_config3_scaled_gqa(lib):
    w = wl.Workload("gqa_scaled", 1, 8, 2, 128, 384, 4, "zigzag")
    ring_case(lib, w, 3, "zigzag", devices=[1, 2])


def test_config4_scaled_full_head_scales(lib):
    w = wl.Workload("full_scaled", 2, 4, 4, 128, 640, 2, "full", True)
    ring_case(lib, w, 4, "full", devices=[0, 1])


def test_striped_partition(lib):
    w = wl.Workload("striped", 1, 2, 2, 128, 320, 4, "striped")
    ring_case(lib, w, 6, "striped", devices=[0, 3])


@pytest.mark.parametrize("kind,window", [("causal", 1), ("causal", 100), ("causal", 300), ("zigzag", 64), ("zigzag", 200),
                                         ("striped", 37), ("striped", 500)])
def test_sliding_window_ring(lib, kind, window):
    """Sliding-window attention over the three partitions: every step's partial (some steps see
    nothing at all), the fused running state and the standalone merge, against the windowed oracle."""
    ring_case(lib, wl.WORKLOADS[1], 1, kind, range(4), window=window)


@pytest.mark.parametrize("d,window", [(64, 0), (128, 0), (128, 90)])
def test_zigzag_pieces_that_are_not_tile_multiples(lib, d, window):
    """Zigzag pieces of 100 and 150 rows: LDS tiles straddle the seam between the front and the back
    piece of a chunk, the last tile is ragged, and the tile runs of the two pieces touch."""
    for piece, G in ((100, 2), (150, 3)):
        w = wl.Workload(f"zigzag_piece{piece}", 1, 2, 2, d, 2 * piece, G, "zigzag")
        ring_case(lib, w, 6, "zigzag", range(G), window=window)


def test_sliding_window_scaled_config2_d128(lib):
    w = wl.Workload("zigzag_window_d128", 1, 4, 4, 128, 512, 4, "zigzag")
    ring_case(lib, w, 2, "zigzag", [0, 1, 3], window=w.seq // 4)


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("sq,sk,qoff", [(200, 333, 150), (1, 1, 0), (77, 64, 10), (129, 257, 300), (64, 1, 0)])
def test_ragged_single_step(lib, d, sq, sk, qoff):
    """Odd sizes: tails inside a tile, one-row chunks, queries that see no key at all."""
    torch = _torch()
    B, Hq, Hkv = 1, 4, 2
    rng = np.random.Generator(np.random.PCG64(wl.BASE_SEED + 7000 + sq * 1000 + sk + d))
    qb, kb, vb = (wl.f32_to_bf16_bits(rng.standard_normal(s, dtype=np.float32))
                  for s in ((B, sq, Hq, d), (B, sk, Hkv, d), (B, sk, Hkv, d)))
    scale = 1.0 / np.sqrt(d)
    for causal in (False, True):
        mask = lib.burst_mask_t(int(causal), 1, 1, 0, (qoff, 0), (0, 0), sq, sk, 1)
        vis = oc.visibility(qoff + np.arange(sq), np.arange(sk), causal)
        O_s, lse_s = oc.mha_step_fwd(hp.widen(qb), hp.widen(kb), hp.widen(vb), scale, vis)
        o_part = torch.full((B, sq, Hq, d), 7.0, device="cuda", dtype=torch.float32)
        lse_part = torch.full((B, Hq, sq), 7.0, device="cuda", dtype=torch.float32)
        shp = lib.shape(B, Hq, Hkv, d, sq, sk, scale)
        lib.burst_attn_step_fwd(shp, mask, hp.dev_bf16(qb), hp.dev_bf16(kb), hp.dev_bf16(vb),
                                o_part=o_part, lse_part=lse_part)
        torch.cuda.synchronize()
        assert hp.rel_err(o_part.cpu().numpy(), O_s) <= hp.REL_TOL
        assert hp.lse_err(lse_part.cpu().numpy(), lse_s) <= hp.LSE_TOL


def test_strided_views_and_guard_rows(lib):
    """Non-contiguous views (a shard sliced out of a longer buffer, heads packed with padding) and
    canaries around the outputs: nothing outside the described region may be touched."""
    torch = _torch()
    B, S, H, d, pad = 2, 192, 2, 128, 64
    rng = np.random.Generator(np.random.PCG64(wl.BASE_SEED + 8000))
    big = {n: wl.f32_to_bf16_bits(rng.standard_normal((B, S + 2 * pad, H, d + 8), dtype=np.float32)) for n in "qkv"}
    dev = {n: hp.dev_bf16(big[n]) for n in "qkv"}
    view = {n: dev[n][:, pad:pad + S, :, :d] for n in "qkv"}
    host = {n: hp.widen(big[n][:, pad:pad + S, :, :d]) for n in "qkv"}
    scale = 1.0 / np.sqrt(d)
    o_big = torch.full((B, S + 2, H, d), 3.0, device="cuda", dtype=torch.float32)
    lse_big = torch.full((B, H, S + 8), 3.0, device="cuda", dtype=torch.float32)
    shp = lib.shape(B, H, H, d, S, S, scale)
    mask = lib.burst_attn_fill_contiguous_mask(0, 0, 1, S, True)
    lib.burst_attn_step_fwd(shp, mask, view["q"], view["k"], view["v"], o_part=o_big[:, 1:S + 1],
                            lse_part=lse_big[:, :, 4:S + 4])
    torch.cuda.synchronize()
    O_s, lse_s = oc.mha_step_fwd(host["q"], host["k"], host["v"], scale, oc.visibility(np.arange(S), np.arange(S), True))
    assert hp.rel_err(o_big[:, 1:S + 1].cpu().numpy(), O_s) <= hp.REL_TOL
    assert hp.lse_err(lse_big[:, :, 4:S + 4].cpu().numpy(), lse_s) <= hp.LSE_TOL
    assert (o_big[:, 0] == 3.0).all() and (o_big[:, S + 1] == 3.0).all()
    assert (lse_big[:, :, :4] == 3.0).all() and (lse_big[:, :, S + 4:] == 3.0).all()


def test_empty_chunks(lib):
    torch = _torch()
    B, H, d = 1, 2, 64
    q = torch.zeros(B, 16, H, d, device="cuda", dtype=torch.bfloat16)
    kv = torch.zeros(B, 16, H, d, device="cuda", dtype=torch.bfloat16)
    o_part = torch.full((B, 16, H, d), 5.0, device="cuda")
    lse_part = torch.full((B, H, 16), 5.0, device="cuda")
    o_acc = torch.full((B, 16, H, d), 2.0, device="cuda")
    lse_acc = torch.full((B, H, 16), 1.0, device="cuda")
    # sk = 0: partial is (0, -inf), running state untouched
    shp = lib.shape(B, H, H, d, 16, 0, 0.125)
    lib.burst_attn_step_fwd(shp, None, q, kv, kv, o_part=o_part, lse_part=lse_part, o_acc=o_acc, lse_acc=lse_acc)
    torch.cuda.synchronize()
    assert (o_part == 0).all() and (lse_part == -float("inf")).all()
    assert (o_acc == 2.0).all() and (lse_acc == 1.0).all()
    # sq = 0: nothing to do
    shp = lib.shape(B, H, H, d, 0, 16, 0.125)
    lib.burst_attn_step_fwd(shp, None, q, kv, kv, o_part=o_part, lse_part=lse_part)
    torch.cuda.synchronize()


@pytest.mark.gpu
def test_mfma_probe_runs_and_counts_its_flops(lib):
    """The matrix-core ceiling probe: argument checks on the host, a short launch of each operand kind
    completes, and the flop count is that of the launch (512 work-groups x 4 waves x 4 chains)."""
    import torch
    raw = lib.raw()
    import ctypes as C
    assert raw.burst_attn_mfma_probe(0, 0, None, None, None) == lib.BURST_ERR_INVALID_ARG
    for random_operands in (0, 1):
        flops = lib.burst_attn_mfma_probe(random_operands, 100)
        torch.cuda.synchronize()
        assert flops == 512 * 4 * 4 * 100 * 2 * 32 * 32 * 16
