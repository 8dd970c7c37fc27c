"""The backward kernels' chunked launches (a long streamed axis cut into row ranges, one launch per range,
gradients accumulating in HBM between them) at sizes the oracle checks exhaustively: the range length is
lowered to 256 rows through the diagnostics call, so that chunks of a few hundred to a few thousand rows run
as 3-8 launches per kernel.  Ranges inside a piece (contiguous, zigzag, striped), ranges of whole pieces
(block-striped), ragged last ranges, block masks whose row blocks the ranges must respect, windows, GQA."""
import numpy as np
import pytest

from paper_2509_19836_amd import workloads as wl
from tests.test_gpu_block_striped import _ring
from tests.test_gpu_bwd import full_ring_case

pytestmark = pytest.mark.gpu


@pytest.fixture
def small_chunks(lib):
    assert lib.burst_attn_set_bwd_chunk_rows(256) == 256
    yield
    lib.burst_attn_set_bwd_chunk_rows(32768)


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
