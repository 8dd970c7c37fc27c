"""Fused LM head + cross-entropy (Alg. 3) through the C-ABI against the fp64 oracle, element by
element: loss and Lse to 1e-3 absolute, dH and dW to 2e-2 of the largest reference entry."""
import numpy as np
import pytest

from oracle import lm_head_oracle as lm
from paper_2509_19836_amd import workloads as wl
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    return torch


def _dev(bits):
    return hp.dev_bf16(bits)


def run_case(lib, seed, N, d, v, B_s, grad_scale=1.0, dh_dtype="f32", ignored=2, accumulate=False, row_pad=0):
    torch = _torch()
    Hb, Wb, Y = wl.lm_head_tensors(seed, N, d, v, ignored)
    if N > ignored + 1:
        Y[-1] = v + 5                      # outside the vocabulary: ignored as well
    H64, W64 = hp.widen(Hb), hp.widen(Wb)
    loss_ref, lse_ref, dH_ref, dW_ref = lm.lm_head_loss(H64, W64, Y, grad_scale)
    shp = lib.lm_head_shape(N, d, v, B_s, grad_scale)
    ws = torch.empty(lib.burst_lm_head_workspace_bytes(shp), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)                         # NaN patterns: nothing may depend on the workspace's old contents
    # rows wider than d, the padding poisoned, to check the leading dimensions
    h_full = torch.full((max(N, 1), d + row_pad), float("nan"), dtype=torch.bfloat16, device="cuda")
    w_full = torch.full((v, d + row_pad), float("nan"), dtype=torch.bfloat16, device="cuda")
    if N:
        h_full[:N, :d] = _dev(Hb)
    w_full[:, :d] = _dev(Wb)
    h, w = h_full[:N, :d], w_full[:, :d]
    y = torch.from_numpy(Y).cuda()
    f32 = dict(dtype=torch.float32, device="cuda")
    loss, lse = torch.full((N,), 7.0, **f32), torch.full((N,), 7.0, **f32)
    dh_full = torch.full((max(N, 1), d + row_pad), 5.0, device="cuda",
                         dtype=torch.float32 if dh_dtype == "f32" else torch.bfloat16)
    dw_full = torch.full((v, d + row_pad), 3.0 if accumulate else float("nan"), **f32)
    print(f"lm head N={N} d={d} v={v} B_s={B_s} dh={dh_dtype} acc={accumulate}", flush=True)
    lib.burst_lm_head_loss(shp, h, w, y, loss, ws, lse=lse, d_h=dh_full[:N, :d], d_w=dw_full[:, :d], accumulate_dw=accumulate)
    torch.cuda.synchronize()
    assert np.abs(loss.cpu().numpy() - loss_ref).max(initial=0) <= hp.LSE_TOL
    assert np.abs(lse.cpu().numpy() - lse_ref).max(initial=0) <= hp.LSE_TOL
    tol = lambda ref: hp.REL_TOL * max(np.abs(ref).max(initial=0), 1e-30)
    if N:
        assert np.abs(dh_full[:N, :d].float().cpu().numpy() - dH_ref).max() <= tol(dH_ref)
    dw = dw_full[:, :d].cpu().numpy() - (3.0 if accumulate else 0.0)
    assert np.abs(dw - dW_ref).max() <= tol(dW_ref) + (1e-5 if accumulate else 0)
    if row_pad:   # the padding columns were not touched
        assert (dh_full[:, d:].float() == 5.0).all()
        assert (dw_full[:, d:] == 3.0).all() if accumulate else torch.isnan(dw_full[:, d:]).all()
    return loss.cpu().numpy(), dh_full[:N, :d].float().cpu().numpy(), dw


def test_three_ragged_sequence_tiles(lib):
    run_case(lib, wl.BASE_SEED + 20001, N=700, d=256, v=1000, B_s=256)


def test_one_ragged_tile_bf16_dh_accumulated_dw_strided_rows(lib):
    run_case(lib, wl.BASE_SEED + 20002, N=300, d=512, v=2500, B_s=512, grad_scale=1.0 / 300, dh_dtype="bf16",
             accumulate=True, row_pad=8)


def test_tiny_sizes(lib):
    run_case(lib, wl.BASE_SEED + 20003, N=1, d=256, v=1, B_s=256, ignored=0)
    run_case(lib, wl.BASE_SEED + 20004, N=65, d=256, v=129, B_s=256)
    run_case(lib, wl.BASE_SEED + 20005, N=256, d=256, v=256, B_s=256)


def test_sequence_tile_size_does_not_change_the_result(lib):
    a = run_case(lib, wl.BASE_SEED + 20006, N=1100, d=256, v=1500, B_s=256)
    b = run_case(lib, wl.BASE_SEED + 20006, N=1100, d=256, v=1500, B_s=2048)
    assert np.abs(a[0] - b[0]).max() <= 1e-5               # same logits, same per-token arithmetic
    assert np.array_equal(a[1], b[1])                      # a token's dH does not depend on the tile it is in
    assert np.abs(a[2] - b[2]).max() <= 1e-3 * np.abs(b[2]).max()   # dW: only the order of the fp32 sums differs


def test_forward_only_and_no_tokens(lib):
    torch = _torch()
    N, d, v, B_s = 500, 256, 777, 256
    Hb, Wb, Y = wl.lm_head_tensors(wl.BASE_SEED + 20007, N, d, v, 3)
    loss_ref, lse_ref, _, _ = lm.lm_head_loss(hp.widen(Hb), hp.widen(Wb), Y)
    shp = lib.lm_head_shape(N, d, v, B_s)
    ws = torch.empty(lib.burst_lm_head_workspace_bytes(shp), dtype=torch.uint8, device="cuda")
    loss = torch.empty(N, dtype=torch.float32, device="cuda")
    lib.burst_lm_head_loss(shp, _dev(Hb), _dev(Wb), torch.from_numpy(Y).cuda(), loss, ws)
    torch.cuda.synchronize()
    assert np.abs(loss.cpu().numpy() - loss_ref).max() <= hp.LSE_TOL
    assert (loss[:3] == 0).all()
    # no tokens: an overwritten dW becomes zero, an accumulated one stays
    shp0 = lib.lm_head_shape(0, d, v, B_s)
    dw = torch.full((v, d), float("nan"), dtype=torch.float32, device="cuda")
    empty = torch.empty((0, d), dtype=torch.bfloat16, device="cuda")
    one = torch.empty(1, dtype=torch.float32, device="cuda")
    lib.burst_lm_head_loss(shp0, empty, _dev(Wb), torch.zeros(1, dtype=torch.int64, device="cuda")[:0], one[:0], ws, d_w=dw)
    torch.cuda.synchronize()
    assert (dw == 0).all()


def test_llama2_vocabulary_two_sequence_tiles(lib):
    """32000 words, hidden size 1024, two sequence tiles of 1024 tokens: every output element against
    the oracle (the oracle's three fp64 products take a few seconds)."""
    run_case(lib, wl.BASE_SEED + 20008, N=2048, d=1024, v=32000, B_s=1024, grad_scale=1.0 / 2048, ignored=5)


def test_benchmark_size_sampled_tokens_and_words(lib):
    """The shape bench.py --lm-head times (16384 tokens, d 4096, 32000 words, sequence tiles of 8192):
    too large for the oracle's three full products, so Lse and the loss are checked for every token
    (the oracle's logits in fp64, in chunks), dH for sampled tokens and dW for sampled words, each
    written out from the definition with the full-size Lse."""
    torch = _torch()
    N, d, v, B_s = 16384, 4096, 32000, 8192
    gs = 1.0 / N
    Hb, Wb, Y = wl.lm_head_tensors(wl.BASE_SEED + 20100, N, d, v, ignored=7)
    H64, W64 = hp.widen(Hb), hp.widen(Wb)
    rng = np.random.Generator(np.random.PCG64(wl.BASE_SEED + 20101))
    tok = np.unique(np.concatenate([[0, 6, 7, 8191, 8192, N - 1], rng.integers(0, N, 40)]))
    words = np.unique(np.concatenate([[0, v - 1], Y[tok[:8]].clip(0, v - 1), rng.integers(0, v, 40)]))
    ok = (Y >= 0) & (Y < v)
    lse_ref, tgt = np.empty(N), np.zeros(N)
    P_words = np.empty((N, words.size))            # softmax columns of the sampled words, all tokens
    for s0 in range(0, N, 2048):
        logits = H64[s0:s0 + 2048] @ W64.T
        lse_ref[s0:s0 + 2048] = lm.row_logsumexp(logits)
        rows = np.arange(s0, min(s0 + 2048, N))
        tgt[rows] = logits[rows - s0, np.where(ok[rows], Y[rows], 0)]
        P_words[rows] = np.exp(logits[:, words] - lse_ref[rows, None])
    loss_ref = np.where(ok, lse_ref - tgt, 0.0)
    E_words = (Y[:, None] == words[None, :]).astype(np.float64)
    dW_ref = (gs * (P_words - E_words) * ok[:, None]).T @ H64            # [words, d]
    P_tok = np.exp(H64[tok] @ W64.T - lse_ref[tok, None])
    E_tok = np.zeros_like(P_tok)
    E_tok[np.nonzero(ok[tok])[0], Y[tok][ok[tok]]] = 1.0
    dH_ref = (gs * (P_tok - E_tok) * ok[tok, None]) @ W64                # [tok, d]

    shp = lib.lm_head_shape(N, d, v, B_s, gs)
    ws = torch.empty(lib.burst_lm_head_workspace_bytes(shp), dtype=torch.uint8, device="cuda")
    f32 = dict(dtype=torch.float32, device="cuda")
    loss, lse = torch.empty(N, **f32), torch.empty(N, **f32)
    dh = torch.empty(N, d, dtype=torch.bfloat16, device="cuda")
    dw = torch.zeros(v, d, **f32)
    print("lm head benchmark size", flush=True)
    lib.burst_lm_head_loss(shp, _dev(Hb), _dev(Wb), torch.from_numpy(Y).cuda(), loss, ws, lse=lse, d_h=dh, d_w=dw,
                           accumulate_dw=True)
    torch.cuda.synchronize()
    assert np.abs(lse.cpu().numpy() - lse_ref).max() <= hp.LSE_TOL
    assert np.abs(loss.cpu().numpy() - loss_ref).max() <= hp.LSE_TOL
    # the tolerance is relative to the largest entry of the whole gradient; the sample's own maximum is smaller or equal
    got_dh = dh[torch.from_numpy(tok).cuda()].float().cpu().numpy()
    assert np.abs(got_dh - dH_ref).max() <= hp.REL_TOL * np.abs(dH_ref).max()
    got_dw = dw[torch.from_numpy(words).cuda()].cpu().numpy()
    assert np.abs(got_dw - dW_ref).max() <= hp.REL_TOL * np.abs(dW_ref).max()


def test_llama3_vocabulary(lib):
    """128256 words (501 vocabulary tiles of 256), hidden size 512, one ragged sequence tile: every element."""
    run_case(lib, wl.BASE_SEED + 20009, N=1500, d=512, v=128256, B_s=2048, grad_scale=1.0 / 1500, dh_dtype="bf16", ignored=4)
