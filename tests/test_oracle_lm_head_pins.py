"""Pins of the fp64 LM-head + loss oracle against things other than itself: a hand-worked example,
closed forms, invariants, finite differences, the algorithm's tiled form against the plain
definition, and an independent library routine.  CPU only."""
import math
import os

import numpy as np
import pytest

from oracle import lm_head_oracle as lm

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def case(seed, N, d, v):
    r = rng(seed)
    return r.standard_normal((N, d)), r.standard_normal((v, d)) * 0.7, r.integers(0, v, N)


def load_golden(name):
    vals = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, v = line.split()
            vals[k] = float(v)
    return vals


def test_hand_worked_two_word_example():
    g = load_golden("lm_head_two_words.txt")
    H, W, Y = np.array([[2.0]]), np.array([[0.0], [math.log(3) / 2]]), np.array([1])
    for fn in (lm.lm_head_loss, lambda *a: lm.lm_head_loss_tiled(*a, 1, 1)):
        loss, lse, dH, dW = fn(H, W, Y)
        assert lse[0] == pytest.approx(g["lse"], abs=1e-14)
        assert loss[0] == pytest.approx(g["loss"], abs=1e-14)
        assert dH[0, 0] == pytest.approx(g["dh"], abs=1e-14)
        assert dW[:, 0] == pytest.approx([g["dw0"], g["dw1"]], abs=1e-14)


def test_zero_weights_give_log_v_and_uniform_probabilities():
    N, d, v = 5, 3, 7
    H, _, Y = case(1, N, d, v)
    loss, lse, dH, dW = lm.lm_head_loss(H, np.zeros((v, d)), Y)
    assert np.allclose(loss, math.log(v), atol=1e-14) and np.allclose(lse, math.log(v), atol=1e-14)
    assert np.allclose(dH, 0)
    E = np.eye(v)[Y]
    assert np.allclose(dW, (1.0 / v - E).T @ H, atol=1e-14)


def test_loss_is_minus_log_probability_of_the_target():
    H, W, Y = case(2, 6, 4, 9)
    loss, lse, _, _ = lm.lm_head_loss(H, W, Y)
    logits = H @ W.T
    for i in range(6):   # written out per token with math.exp, no shared routine
        z = sum(math.exp(x) for x in logits[i])
        assert loss[i] == pytest.approx(-math.log(math.exp(logits[i, Y[i]]) / z), abs=1e-12)
        assert lse[i] == pytest.approx(math.log(z), abs=1e-12)


@pytest.mark.parametrize("scale", [1.0, 0.125])
def test_gradients_by_central_finite_differences(scale):
    """Fixes the sign of the one-hot term: the printed + E would fail here."""
    H, W, Y = case(3, 4, 3, 5)
    total = lambda H_, W_: scale * lm.lm_head_loss(H_, W_, Y)[0].sum()
    _, _, dH, dW = lm.lm_head_loss(H, W, Y, grad_scale=scale)
    eps = 1e-6
    for X, dX, which in ((H, dH, 0), (W, dW, 1)):
        num = np.zeros_like(X)
        for idx in np.ndindex(*X.shape):
            Xp, Xm = X.copy(), X.copy()
            Xp[idx] += eps
            Xm[idx] -= eps
            num[idx] = ((total(Xp, W) - total(Xm, W)) if which == 0 else (total(H, Xp) - total(H, Xm))) / (2 * eps)
        assert np.allclose(dX, num, atol=1e-8), which
    # the printed sign, planted: the same check must reject it
    P = np.exp(H @ W.T - lm.row_logsumexp(H @ W.T)[:, None])
    wrong_dH = scale * (P + np.eye(5)[Y]) @ W
    assert not np.allclose(wrong_dH, dH, atol=1e-3)


@pytest.mark.parametrize("N,v,B_s,B_v", [(7, 11, 3, 4), (8, 8, 8, 8), (5, 13, 1, 13), (9, 6, 4, 1), (6, 10, 100, 100)])
def test_tiled_algorithm_equals_the_definition(N, v, B_s, B_v):
    H, W, Y = case(4 + N, N, 5, v)
    Y[0] = -100          # an ignored token
    Y[-1] = v + 3        # also outside the vocabulary
    a = lm.lm_head_loss(H, W, Y, grad_scale=0.5)
    b = lm.lm_head_loss_tiled(H, W, Y, B_s, B_v, grad_scale=0.5)
    for x, y in zip(a, b):
        assert np.allclose(x, y, atol=1e-12)
    assert a[0][0] == 0 and a[0][-1] == 0 and np.all(a[2][0] == 0) and np.all(a[2][-1] == 0)


def test_invariants_of_the_gradient():
    H, W, Y = case(5, 6, 4, 8)
    loss, _, dH, dW = lm.lm_head_loss(H, W, Y)
    # rows of softmax - E sum to zero: the word gradients sum to zero over the vocabulary
    assert np.allclose(dW.sum(axis=0), 0, atol=1e-13)
    # shifting every word vector by the same c shifts each token's logits by a constant: loss unchanged
    c = rng(6).standard_normal(4)
    assert np.allclose(lm.lm_head_loss(H, W + c, Y)[0], loss, atol=1e-12)
    # a target whose logit dominates: loss -> 0, gradient -> 0
    Hs, Ws = np.array([[10.0, 0.0]]), np.array([[10.0, 0.0], [-10.0, 0.0], [0.0, 1.0]])
    l, _, dh, dw = lm.lm_head_loss(Hs, Ws, np.array([0]))
    assert l[0] < 1e-40 + math.exp(-90) and np.abs(dh).max() < 1e-30 and np.abs(dw).max() < 1e-30


def test_against_torch_cross_entropy_and_autograd():
    torch = pytest.importorskip("torch")
    H, W, Y = case(7, 10, 6, 12)
    Y[3] = -100
    Ht = torch.tensor(H, dtype=torch.float64, requires_grad=True)
    Wt = torch.tensor(W, dtype=torch.float64, requires_grad=True)
    Yt = torch.tensor(Y, dtype=torch.int64)
    per_token = torch.nn.functional.cross_entropy(Ht @ Wt.T, Yt, reduction="none", ignore_index=-100)
    (per_token.sum() / 10).backward()
    loss, _, dH, dW = lm.lm_head_loss(H, W, Y, grad_scale=0.1)
    assert np.allclose(loss, per_token.detach().numpy(), atol=1e-12)
    assert np.allclose(dH, Ht.grad.numpy(), atol=1e-12)
    assert np.allclose(dW, Wt.grad.numpy(), atol=1e-12)
