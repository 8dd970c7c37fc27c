"""The step kernels' chunked launches (a long streamed axis cut into row ranges, one launch per range, the
running forward state and the gradients accumulating in HBM between them) at sizes the oracle checks
exhaustively: the range length is lowered to 256 rows through the diagnostics call, so that chunks of a few
hundred to a few thousand rows run as 3-8 launches per kernel, forward (fused merge) and backward.  Ranges
inside a piece (contiguous, zigzag, striped), ranges of whole pieces (block-striped), ragged last ranges,
block masks whose row blocks the ranges must respect, windows, GQA."""
import numpy as np
import pytest

from paper_2509_19836_amd import workloads as wl
from tests.test_gpu_block_striped import _ring
from tests.test_gpu_bwd import full_ring_case

pytestmark = pytest.mark.gpu


@pytest.fixture
def small_chunks(lib):
    assert lib.burst_attn_set_chunk_rows(256) == 256
    yield
    lib.burst_attn_set_chunk_rows(32768)


@pytest.mark.parametrize("window", [0, 700])
def test_zigzag_gqa_ranges_inside_pieces(lib, small_chunks, window):
    # two pieces of 768 rows a side: three ranges per piece
    full_ring_case(lib, wl.Workload("chunk_zigzag", 1, 4, 2, 128, 1536, 2, "zigzag"), 2, "zigzag", window=window)


def test_full_mask_batch2_ragged_last_range(lib, small_chunks):
    full_ring_case(lib, wl.Workload("chunk_full", 2, 2, 2, 64, 1100, 2, "full", True), 4, "full")


def test_query_bundles_travel_causal(lib, small_chunks):
    full_ring_case(lib, wl.Workload("chunk_causal", 1, 2, 2, 128, 900, 3, "causal"), 1, "causal", travel="q")


def test_striped_with_window(lib, small_chunks):
    full_ring_case(lib, wl.Workload("chunk_striped", 1, 2, 2, 128, 800, 4, "striped"), 6, "striped", window=333)


@pytest.mark.parametrize("window", [0, 300])
def test_block_striped_ranges_of_whole_pieces(lib, small_chunks, window):
    # eight pieces of 128 rows a side: two pieces per range
    _ring(lib, "block_striped", 4, 4096, 512, 4, 2, 128, seed=900 + window, window=window)


@pytest.mark.parametrize("kind", ["block_striped", "zigzag", "contiguous"])
def test_block_pattern_with_ranges_on_block_boundaries(lib, small_chunks, kind):
    G = 4
    N_blk = 1024 if kind == "block_striped" else 256
    N = 8192 if kind == "block_striped" else 4096
    nb = N // N_blk
    rng = np.random.Generator(np.random.PCG64(wl.BASE_SEED + 32000 + nb))
    pattern = (rng.random((nb, nb)) < 0.5).astype(np.uint8)
    np.fill_diagonal(pattern, 1)
    _ring(lib, kind, G, N, N_blk, 2, 2, 128, seed=70 + nb, causal=True, window=0, pattern=pattern,
          devices=None if kind == "block_striped" else [0, 2])


def test_forward_ranges_fold_into_a_dead_then_a_live_running_state(lib, small_chunks):
    """The fused forward alone: five key ranges (the last ragged) folded one launch after the other into a
    running state that starts as (NaN garbage, -inf), against the oracle's step; then the same step folded
    into that result once more, which must leave O and add log 2 to Lse."""
    import torch
    from oracle import burst_oracle as oc
    from tests import helpers as hp
    w = wl.Workload("chunk_fwd", 1, 4, 2, 128, 1100, 1, "causal")
    T = wl.host_tensors(w, 1, seed_offset=11)
    n = w.shard_tokens
    Q, K, V = (hp.widen(T[x][1]) for x in ("q", "k", "v"))
    q, k, v = (hp.dev_bf16(T[x][1]).contiguous() for x in ("q", "k", "v"))
    shp = lib.shape(w.batch, w.q_heads, w.kv_heads, w.head_dim, n, n, w.scale)
    mask = lib.burst_attn_fill_contiguous_mask(0, 0, 1, n, True)
    assert len(lib.burst_attn_chunk_plan(mask, 0)) == 5
    O_ref, lse_ref = oc.mha_step_fwd(Q, K, V, w.scale, oc.visibility(np.arange(n), np.arange(n), True))
    o_acc = torch.full((w.batch, n, w.q_heads, w.head_dim), float("nan"), device="cuda", dtype=torch.float32)
    lse_acc = torch.full((w.batch, w.q_heads, n), -float("inf"), device="cuda", dtype=torch.float32)
    for extra in (0.0, np.log(2.0)):
        lib.burst_attn_step_fwd(shp, mask, q, k, v, o_acc=o_acc, lse_acc=lse_acc)
        torch.cuda.synchronize()
        assert torch.isfinite(o_acc).all()
        assert hp.rel_err(o_acc.cpu().numpy(), O_ref) <= hp.REL_TOL
        assert hp.lse_err(lse_acc.cpu().numpy(), lse_ref + extra) <= hp.LSE_TOL
