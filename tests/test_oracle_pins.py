"""Pins of the fp64 oracle against things other than itself: a hand-worked
example, closed forms, invariants, brute force, finite differences and an
independent library routine.  CPU only."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import burst_oracle as oc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def rand_qkvdo(seed, nq, nk, d):
    r = rng(seed)
    return (r.standard_normal((nq, d)), r.standard_normal((nk, d)),
            r.standard_normal((nk, d)), r.standard_normal((nq, d)))


# ----------------------------------------------------------------- worked example

def load_golden(name):
    vals = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, v = line.split()
            vals[k] = float(v)
    return vals


def test_hand_worked_two_key_example():
    g = load_golden("softmax_two_keys.txt")
    Q = np.array([[1.0]])
    K = np.array([[0.0], [math.log(3.0)]])
    V = np.array([[0.0], [4.0]])
    dO = np.array([[1.0]])
    O, lse = oc.attention_fwd(Q, K, V, 1.0)
    assert lse[0] == pytest.approx(g["lse"], abs=1e-15)
    assert O[0, 0] == pytest.approx(g["o"], abs=1e-14)
    P = oc.attention_probs(Q, K, 1.0)
    assert P[0] == pytest.approx([g["p0"], g["p1"]], abs=1e-15)
    # the step formulation and the two-step merge
    O2, lse2 = oc.step_fwd(Q, K, V, 1.0)
    assert O2[0, 0] == pytest.approx(g["o"], abs=1e-14) and lse2[0] == pytest.approx(g["lse"], abs=1e-15)
    Oa, la = oc.step_fwd(Q, K[:1], V[:1], 1.0)
    Ob, lb = oc.step_fwd(Q, K[1:], V[1:], 1.0)
    Om, lm = oc.lse_merge(*oc.lse_merge(np.zeros((1, 1)), np.full(1, -np.inf), Oa, la), Ob, lb)
    assert Om[0, 0] == pytest.approx(g["o"], abs=1e-14) and lm[0] == pytest.approx(g["lse"], abs=1e-15)
    # backward
    D = oc.preprocess_bwd(dO, O)
    assert D[0] == pytest.approx(g["D"], abs=1e-14)
    dQ, dK, dV = oc.step_bwd(Q, K, V, dO, lse, D, 1.0)
    assert dQ[0, 0] == pytest.approx(g["dq"], abs=1e-14)
    assert dK[:, 0] == pytest.approx([g["dk0"], g["dk1"]], abs=1e-14)
    assert dV[:, 0] == pytest.approx([g["dv0"], g["dv1"]], abs=1e-14)
    dQ2, dK2, dV2 = oc.attention_bwd(Q, K, V, dO, 1.0)
    assert dQ2[0, 0] == pytest.approx(g["dq"], abs=1e-14)
    assert dK2[:, 0] == pytest.approx([g["dk0"], g["dk1"]], abs=1e-14)


# ----------------------------------------------------------------- softmax / closed forms

@pytest.mark.parametrize("causal", [False, True])
def test_probability_rows_sum_to_one(causal):
    Q, K, V, _ = rand_qkvdo(1, 37, 37, 8)
    vis = oc.visibility(np.arange(37), np.arange(37), causal)
    P = oc.attention_probs(Q, K, 0.35, vis)
    assert np.abs(P.sum(axis=1) - 1.0).max() < 1e-12
    assert (P[~vis] == 0).all()


def test_equal_keys_give_uniform_attention():
    r = rng(2)
    nq, nk, d, scale = 9, 13, 6, 0.4
    Q = r.standard_normal((nq, d))
    krow = r.standard_normal(d)
    K = np.tile(krow, (nk, 1))
    V = r.standard_normal((nk, d))
    pos_q = np.arange(4, 4 + nq)
    pos_k = np.arange(nk)
    vis = oc.visibility(pos_q, pos_k, True)
    O, lse = oc.attention_fwd(Q, K, V, scale, vis)
    for rr in range(nq):
        n = int(vis[rr].sum())
        assert O[rr] == pytest.approx(V[:n].mean(axis=0), abs=1e-13)
        assert lse[rr] == pytest.approx(scale * Q[rr] @ krow + math.log(n), abs=1e-13)


def test_single_visible_key_copies_value():
    Q, K, V, _ = rand_qkvdo(3, 5, 5, 4)
    vis = np.eye(5, dtype=bool)
    O, lse = oc.attention_fwd(Q, K, V, 0.5, vis)
    assert O == pytest.approx(V, abs=1e-14)
    assert lse == pytest.approx(0.5 * (Q * K).sum(axis=1), abs=1e-14)


def test_key_shift_invariance():
    Q, K, V, _ = rand_qkvdo(4, 11, 17, 8)
    c = rng(5).standard_normal(8)
    O1, l1 = oc.attention_fwd(Q, K, V, 0.3)
    O2, l2 = oc.attention_fwd(Q, K + c, V, 0.3)
    assert O2 == pytest.approx(O1, abs=1e-12)
    assert l2 - l1 == pytest.approx(0.3 * Q @ c, abs=1e-12)


def test_scale_is_applied_to_scores():
    # a transposed operand or a dropped scale changes this closed form
    Q = np.array([[2.0, 0.0]])
    K = np.array([[1.0, 5.0], [3.0, -7.0]])
    V = np.array([[1.0, 0.0], [0.0, 1.0]])
    O, lse = oc.attention_fwd(Q, K, V, 0.5)
    # S = 0.5 * (2, 6) = (1, 3)
    z = math.exp(1.0) + math.exp(3.0)
    assert lse[0] == pytest.approx(math.log(z), abs=1e-14)
    assert O[0] == pytest.approx([math.exp(1.0) / z, math.exp(3.0) / z], abs=1e-14)


def test_all_masked_row_is_zero_and_minus_inf():
    Q, K, V, _ = rand_qkvdo(6, 4, 6, 3)
    vis = np.ones((4, 6), dtype=bool)
    vis[2] = False
    O, lse = oc.step_fwd(Q, K, V, 1.0, vis)
    assert (O[2] == 0).all() and lse[2] == -np.inf
    assert np.isfinite(lse[[0, 1, 3]]).all()
    O2, lse2 = oc.attention_fwd(Q, K, V, 1.0, vis)
    assert (O2[2] == 0).all() and lse2[2] == -np.inf


# ----------------------------------------------------------------- merge

def test_merge_identity_and_self_merge():
    Q, K, V, _ = rand_qkvdo(7, 6, 9, 4)
    O, lse = oc.step_fwd(Q, K, V, 0.5)
    zero, ninf = np.zeros_like(O), np.full(6, -np.inf)
    O1, l1 = oc.lse_merge(zero, ninf, O, lse)
    assert (O1 == O).all() and (l1 == lse).all()
    O2, l2 = oc.lse_merge(O, lse, zero, ninf)
    assert (O2 == O).all() and (l2 == lse).all()
    O3, l3 = oc.lse_merge(zero, ninf, zero, ninf)
    assert (O3 == 0).all() and (l3 == -np.inf).all()
    O4, l4 = oc.lse_merge(O, lse, O, lse)
    assert O4 == pytest.approx(O, abs=1e-14)
    assert l4 == pytest.approx(lse + math.log(2.0), abs=1e-14)


def test_merge_weights_hand_values():
    # lse_i = ln 1, lse_cur = ln 3  ->  weights 1/4 and 3/4
    O, l = oc.lse_merge(np.array([[8.0]]), np.array([0.0]), np.array([[4.0]]), np.array([math.log(3.0)]))
    assert l[0] == pytest.approx(math.log(4.0), abs=1e-15)
    assert O[0, 0] == pytest.approx(0.25 * 8.0 + 0.75 * 4.0, abs=1e-14)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("G", [1, 2, 4])
def test_ring_merge_equals_unsharded_any_order(causal, G):
    N, d, scale = 48, 8, 0.3
    Q, K, V, _ = rand_qkvdo(8 + G, N, N, d)
    pos = [oc.contiguous_positions(i, G, N) for i in range(G)]
    O_ref, lse_ref = oc.attention_fwd(Q, K, V, scale, oc.visibility(np.arange(N), np.arange(N), causal))
    Ks = [K[p] for p in pos]
    Vs = [V[p] for p in pos]
    for i in range(G):
        orders = [oc.ring_order(i, G), oc.ring_order(i, G, reverse=True)]
        if G == 4:
            orders += [list(p) for p in itertools.islice(itertools.permutations(range(G)), 5, 24, 7)]
        for order in orders:
            O, lse = oc.ring_fwd(Q[pos[i]], Ks, Vs, scale,
                                 lambda j: oc.visibility(pos[i], pos[j], causal), order)
            assert np.abs(O - O_ref[pos[i]]).max() < 1e-12
            assert np.abs(lse - lse_ref[pos[i]]).max() < 1e-12


# ----------------------------------------------------------------- partitions and masks

@pytest.mark.parametrize("G,N", [(1, 6), (2, 12), (3, 30), (4, 40)])
def test_partitions_cover_sequence_once(G, N):
    for fn in (oc.contiguous_positions, oc.zigzag_positions, oc.striped_positions):
        allpos = np.concatenate([fn(i, G, N) for i in range(G)])
        assert sorted(allpos.tolist()) == list(range(N))
        assert all(fn(i, G, N).size == N // G for i in range(G))


def test_zigzag_positions_match_equation_one_based():
    # Eq. 11 literally, 1-based tokens x_1..x_n: front k in [(i-1)P+1, iP],
    # back k in [n-iP+1, n-(i-1)P]
    G, N = 4, 40
    P = N // (2 * G)
    for i1 in range(1, G + 1):
        front = list(range((i1 - 1) * P + 1, i1 * P + 1))
        back = list(range(N - i1 * P + 1, N - (i1 - 1) * P + 1))
        expect = [k - 1 for k in front + back]
        assert oc.zigzag_positions(i1 - 1, G, N).tolist() == expect


def causal_brute(pos_q, pos_k):
    return np.array([[pq >= pk for pk in pos_k] for pq in pos_q], dtype=bool)


@pytest.mark.parametrize("G,N", [(2, 12), (3, 30), (4, 40)])
def test_zigzag_case_table_equals_position_predicate_and_global_causal(G, N):
    d, scale = 4, 0.6
    Q, K, V, _ = rand_qkvdo(20 + G, N, N, d)
    P = N // (2 * G)
    O_ref, lse_ref = oc.attention_fwd(Q, K, V, scale, causal_brute(range(N), range(N)))
    pos = [oc.zigzag_positions(i, G, N) for i in range(G)]
    total_pairs = 0
    for i in range(G):
        O_acc, lse_acc = np.zeros((2 * P, d)), np.full(2 * P, -np.inf)
        for j in oc.ring_order(i, G):
            vis = oc.visibility(pos[i], pos[j], True)
            assert (vis == causal_brute(pos[i], pos[j])).all()
            n_pairs = int(vis.sum())
            assert n_pairs == (2 * P * P + P if i == j else 2 * P * P)
            assert n_pairs == oc.visible_pairs(pos[i], pos[j], True)
            total_pairs += n_pairs
            O_pos, lse_pos = oc.step_fwd(Q[pos[i]], K[pos[j]], V[pos[j]], scale, vis)
            O_case, lse_case = oc.zigzag_step_fwd_cases(i, j, Q[pos[i]], K[pos[j]], V[pos[j]], scale)
            assert np.abs(O_pos - O_case).max() < 1e-13
            with np.errstate(invalid="ignore"):
                assert ((lse_pos == lse_case) | (np.abs(lse_pos - lse_case) < 1e-13)).all()
            O_acc, lse_acc = oc.lse_merge(O_acc, lse_acc, O_case, lse_case)
        assert np.abs(O_acc - O_ref[pos[i]]).max() < 1e-12
        assert np.abs(lse_acc - lse_ref[pos[i]]).max() < 1e-12
    assert total_pairs == N * (N + 1) // 2


@pytest.mark.parametrize("G,N", [(2, 12), (4, 24)])
def test_contiguous_and_striped_causal_steps_cover_global_causal(G, N):
    for fn in (oc.contiguous_positions, oc.striped_positions):
        pos = [fn(i, G, N) for i in range(G)]
        total = sum(oc.visible_pairs(pos[i], pos[j], True) for i in range(G) for j in range(G))
        assert total == N * (N + 1) // 2
    # striped, Eq. 14: i >= j is plain causal on local indices, i < j drops the diagonal
    pos = [oc.striped_positions(i, G, N) for i in range(G)]
    n = N // G
    for i in range(G):
        for j in range(G):
            vis = oc.visibility(pos[i], pos[j], True)
            tri = np.tril(np.ones((n, n), dtype=bool), 0 if i >= j else -1)
            assert (vis == tri).all()


# ----------------------------------------------------------------- gradients

def loss(Q, K, V, dO, scale, vis):
    return float((oc.attention_fwd(Q, K, V, scale, vis)[0] * dO).sum())


def fd_grad(f, X, h=1e-5):
    G = np.zeros_like(X)
    for idx in np.ndindex(*X.shape):
        old = X[idx]
        X[idx] = old + h
        fp = f()
        X[idx] = old - h
        fm = f()
        X[idx] = old
        G[idx] = (fp - fm) / (2 * h)
    return G


@pytest.mark.parametrize("kind", ["full", "causal", "rect_causal"])
def test_gradients_match_central_finite_differences(kind):
    nq, nk, d, scale = (16, 16, 4, 0.5) if kind != "rect_causal" else (7, 12, 3, 0.7)
    Q, K, V, dO = rand_qkvdo(30, nq, nk, d)
    if kind == "full":
        vis = None
    elif kind == "causal":
        vis = oc.visibility(np.arange(nq), np.arange(nk), True)
    else:
        vis = oc.visibility(np.arange(5, 5 + nq), np.arange(nk), True)
    dQ, dK, dV = oc.attention_bwd(Q, K, V, dO, scale, vis)
    f = lambda: loss(Q, K, V, dO, scale, vis)
    for got, X in ((dQ, Q), (dK, K), (dV, V)):
        ref = fd_grad(f, X)
        assert np.abs(got - ref).max() <= 1e-7 * max(1.0, np.abs(ref).max())
    # the step formulation with D = rowsum(dO o O) gives the same gradient
    O, lse = oc.attention_fwd(Q, K, V, scale, vis)
    dQ2, dK2, dV2 = oc.step_bwd(Q, K, V, dO, lse, oc.preprocess_bwd(dO, O), scale, vis)
    for a, b in ((dQ, dQ2), (dK, dK2), (dV, dV2)):
        assert np.abs(a - b).max() < 1e-12


def test_backward_invariants():
    nq, nk, d, scale = 24, 24, 8, 0.35
    Q, K, V, dO = rand_qkvdo(31, nq, nk, d)
    vis = oc.visibility(np.arange(nq), np.arange(nk), True)
    O, lse = oc.attention_fwd(Q, K, V, scale, vis)
    P = oc.attention_probs(Q, K, scale, vis)
    dP = dO @ V.T
    D = oc.preprocess_bwd(dO, O)
    # Eq. 7-8: rowsum(P o dP) = rowsum(dO o O)
    assert np.abs((P * dP).sum(axis=1) - D).max() < 1e-12
    dS = P * (dP - D[:, None])
    assert np.abs(dS.sum(axis=1)).max() < 1e-12
    dQ, dK, dV = oc.attention_bwd(Q, K, V, dO, scale, vis)
    assert np.abs(dV.sum(axis=0) - dO.sum(axis=0)).max() < 1e-12
    # softmax is invariant to a common shift of the keys: sum_c dK[c] = 0
    assert np.abs(dK.sum(axis=0)).max() < 1e-12


def test_partial_lse_breaks_the_D_identity():
    # feeding a step-partial Lse/O instead of the final ones must NOT give
    # the right gradient (reading: backward uses the final Lse and D)
    N, d, scale = 16, 4, 0.5
    Q, K, V, dO = rand_qkvdo(32, N, N, d)
    dQ_ref, _, _ = oc.attention_bwd(Q, K, V, dO, scale)
    O_half, lse_half = oc.step_fwd(Q, K[:8], V[:8], scale)
    dq_a, _, _ = oc.step_bwd(Q, K[:8], V[:8], dO, lse_half, oc.preprocess_bwd(dO, O_half), scale)
    dq_b, _, _ = oc.step_bwd(Q, K[8:], V[8:], dO, lse_half, oc.preprocess_bwd(dO, O_half), scale)
    assert np.abs(dq_a + dq_b - dQ_ref).max() > 1e-3


@pytest.mark.parametrize("part", ["contiguous", "zigzag", "striped"])
@pytest.mark.parametrize("causal", [False, True])
def test_both_backward_travel_orders_equal_unsharded(part, causal):
    G, N, d, scale = 3, 36, 4, 0.45
    Q, K, V, dO = rand_qkvdo(40, N, N, d)
    fn = {"contiguous": oc.contiguous_positions, "zigzag": oc.zigzag_positions,
          "striped": oc.striped_positions}[part]
    pos = [fn(i, G, N) for i in range(G)]
    vis_glob = oc.visibility(np.arange(N), np.arange(N), causal)
    O, lse = oc.attention_fwd(Q, K, V, scale, vis_glob)
    dQ_ref, dK_ref, dV_ref = oc.attention_bwd(Q, K, V, dO, scale, vis_glob)
    D = oc.preprocess_bwd(dO, O)
    vis = lambda a, b: oc.visibility(pos[a], pos[b], causal)
    Qs, dOs = [Q[p] for p in pos], [dO[p] for p in pos]
    Ks, Vs = [K[p] for p in pos], [V[p] for p in pos]
    lses, Ds = [lse[p] for p in pos], [D[p] for p in pos]
    # Alg. 2: K, V stay; Q bundles travel
    dQ2 = [np.zeros((len(p), d)) for p in pos]
    for i in range(G):
        dK_i, dV_i, contrib = oc.ring_bwd_burst(i, Qs, dOs, lses, Ds, Ks[i], Vs[i], scale, vis,
                                                oc.ring_order(i, G))
        assert np.abs(dK_i - dK_ref[pos[i]]).max() < 1e-12
        assert np.abs(dV_i - dV_ref[pos[i]]).max() < 1e-12
        for j, dq in contrib.items():
            dQ2[j] += dq
    # Alg. 1: Q stays; K, V, dK, dV travel
    dK1 = [np.zeros((len(p), d)) for p in pos]
    dV1 = [np.zeros((len(p), d)) for p in pos]
    for i in range(G):
        dQ_i, dKc, dVc = oc.ring_bwd_ring(i, Qs[i], dOs[i], O[pos[i]], lses[i], Ks, Vs, scale, vis,
                                          oc.ring_order(i, G, reverse=True))
        assert np.abs(dQ_i - dQ_ref[pos[i]]).max() < 1e-12
        assert np.abs(dQ_i - dQ2[i]).max() < 1e-12
        for j in range(G):
            dK1[j] += dKc[j]
            dV1[j] += dVc[j]
    for i in range(G):
        assert np.abs(dK1[i] - dK_ref[pos[i]]).max() < 1e-12
        assert np.abs(dV1[i] - dV_ref[pos[i]]).max() < 1e-12


# ----------------------------------------------------------------- multi-head / GQA

def test_grouped_query_wrappers_against_per_head_loops_and_fd():
    B, S, Hq, Hkv, d, scale = 2, 10, 4, 2, 3, 0.6
    r = rng(50)
    Q = r.standard_normal((B, S, Hq, d))
    K = r.standard_normal((B, S, Hkv, d))
    V = r.standard_normal((B, S, Hkv, d))
    dO = r.standard_normal((B, S, Hq, d))
    vis = oc.visibility(np.arange(S), np.arange(S), True)
    assert [oc.kv_head_of(h, 4, 2) for h in range(4)] == [0, 0, 1, 1]
    O, lse = oc.mha_attention_fwd(Q, K, V, scale, vis)
    dQ, dK, dV = oc.mha_attention_bwd(Q, K, V, dO, scale, vis)
    f = lambda: float((oc.mha_attention_fwd(Q, K, V, scale, vis)[0] * dO).sum())
    for got, X in ((dQ, Q), (dK, K), (dV, V)):
        ref = fd_grad(f, X)
        assert np.abs(got - ref).max() <= 1e-7 * max(1.0, np.abs(ref).max())
    D = oc.mha_preprocess_bwd(dO, O)
    dQ2, dK2, dV2 = oc.mha_step_bwd(Q, K, V, dO, lse, D, scale, vis)
    for a, b in ((dQ, dQ2), (dK, dK2), (dV, dV2)):
        assert np.abs(a - b).max() < 1e-12
    O2, lse2 = oc.mha_step_fwd(Q, K, V, scale, vis)
    assert np.abs(O - O2).max() < 1e-12 and np.abs(lse - lse2).max() < 1e-12
    Om, lm = oc.mha_lse_merge(np.zeros_like(O), np.full(lse.shape, -np.inf), O2, lse2)
    assert (Om == O2).all() and (lm == lse2).all()
    # a running state that is not trivial: the keys split in two halves, each head with its own state,
    # merged head by head must give back the unsharded result (a wrong head index on either side of
    # the merge mixes heads whose states differ, and fails)
    half = S // 2
    Oa, la = oc.mha_step_fwd(Q, K[:, :half], V[:, :half], scale, vis[:, :half])
    Ob, lb = oc.mha_step_fwd(Q, K[:, half:], V[:, half:], scale, vis[:, half:])
    assert np.abs(la[0, 0] - la[0, 1]).max() > 1e-3 and np.abs(Oa[:, :, 0] - Oa[:, :, 2]).max() > 1e-3
    Om, lm = oc.mha_lse_merge(Oa, la, Ob, lb)
    assert np.abs(Om - O).max() < 1e-12 and np.abs(lm - lse).max() < 1e-12
    Om2, lm2 = oc.mha_lse_merge(Ob, lb, Oa, la)     # the merge commutes
    assert np.abs(Om2 - O).max() < 1e-12 and np.abs(lm2 - lse).max() < 1e-12
    # written out for one (batch, head, row): weights e^(lse - lse') on each side
    b_, h_, r_ = 0, 3, S - 1
    lnew = np.log(np.exp(la[b_, h_, r_]) + np.exp(lb[b_, h_, r_]))
    want = np.exp(la[b_, h_, r_] - lnew) * Oa[b_, r_, h_] + np.exp(lb[b_, h_, r_] - lnew) * Ob[b_, r_, h_]
    assert np.abs(Om[b_, r_, h_] - want).max() < 1e-12 and abs(lm[b_, h_, r_] - lnew) < 1e-12


# ----------------------------------------------------------------- independent library routine

def test_against_torch_sdpa_float64_autograd():
    torch = pytest.importorskip("torch")
    B, S, Hq, Hkv, d = 1, 33, 4, 2, 8
    scale = 1.0 / math.sqrt(d)
    r = rng(60)
    Q = r.standard_normal((B, S, Hq, d))
    K = r.standard_normal((B, S, Hkv, d))
    V = r.standard_normal((B, S, Hkv, d))
    dO = r.standard_normal((B, S, Hq, d))
    for causal in (False, True):
        vis = oc.visibility(np.arange(S), np.arange(S), causal)
        O, _ = oc.mha_attention_fwd(Q, K, V, scale, vis)
        dQ, dK, dV = oc.mha_attention_bwd(Q, K, V, dO, scale, vis)
        tq = torch.tensor(Q, dtype=torch.float64, requires_grad=True)
        tk = torch.tensor(K, dtype=torch.float64, requires_grad=True)
        tv = torch.tensor(V, dtype=torch.float64, requires_grad=True)
        rep = Hq // Hkv
        out = torch.nn.functional.scaled_dot_product_attention(
            tq.permute(0, 2, 1, 3), tk.permute(0, 2, 1, 3).repeat_interleave(rep, dim=1),
            tv.permute(0, 2, 1, 3).repeat_interleave(rep, dim=1), is_causal=causal)
        out = out.permute(0, 2, 1, 3)
        out.backward(torch.tensor(dO))
        assert np.abs(out.detach().numpy() - O).max() < 1e-12
        assert np.abs(tq.grad.numpy() - dQ).max() < 1e-12
        assert np.abs(tk.grad.numpy() - dK).max() < 1e-12
        assert np.abs(tv.grad.numpy() - dV).max() < 1e-12


# ----------------------------------------------------------------- sliding window

@pytest.mark.parametrize("window", [1, 2, 5, 16, 100])
def test_window_visibility_brute_force_and_limits(window):
    """A query at position p sees exactly the keys at positions p-window+1 .. p: brute force over
    scattered positions; a window of one leaves the token itself (O = its V row, lse = its score);
    a window as long as the sequence is plain causal attention."""
    pos_q = np.array([0, 3, 4, 9, 17, 18, 40])
    pos_k = np.array([0, 1, 4, 8, 9, 16, 18, 39, 40, 41])
    vis = oc.visibility(pos_q, pos_k, True, window)
    for a, p in enumerate(pos_q):
        for b, k in enumerate(pos_k):
            assert vis[a, b] == (p - window + 1 <= k <= p)
    assert oc.visible_pairs(pos_q, pos_k, True, window) == int(vis.sum())
    n, d = 12, 4
    Q, K, V, _ = rand_qkvdo(70, n, n, d)
    pos = np.arange(n)
    if window == 1:
        O, lse = oc.attention_fwd(Q, K, V, 0.5, oc.visibility(pos, pos, True, 1))
        assert np.allclose(O, V, atol=1e-14)
        assert np.allclose(lse, 0.5 * (Q * K).sum(1), atol=1e-13)
    if window >= n:
        assert (oc.visibility(pos, pos, True, window) == oc.visibility(pos, pos, True)).all()
    with pytest.raises(ValueError):
        oc.visibility(pos, pos, False, window)


@pytest.mark.parametrize("part", ["contiguous", "zigzag", "striped"])
def test_windowed_ring_equals_unsharded_windowed_attention(part):
    """Forward ring + merge and both backward travel orders over windowed step masks reproduce
    unsharded sliding-window attention; steps wholly outside the window contribute (0, -inf)."""
    G, N, d, window, scale = 4, 48, 4, 10, 0.4
    pos_fn = {"contiguous": oc.contiguous_positions, "zigzag": oc.zigzag_positions, "striped": oc.striped_positions}[part]
    Q, K, V, dO = rand_qkvdo(71, N, N, d)
    allpos = np.arange(N)
    vis_all = oc.visibility(allpos, allpos, True, window)
    O_ref, lse_ref = oc.attention_fwd(Q, K, V, scale, vis_all)
    dQ_ref, dK_ref, dV_ref = oc.attention_bwd(Q, K, V, dO, scale, vis_all)
    pos = [pos_fn(i, G, N) for i in range(G)]
    dK_tot, dV_tot = np.zeros_like(K), np.zeros_like(V)
    saw_empty_step = False
    for i in range(G):
        order = oc.ring_order(i, G)
        vis_of = lambda j: oc.visibility(pos[i], pos[j], True, window)
        saw_empty_step |= any(not vis_of(j).any() for j in order)
        O_i, lse_i = oc.ring_fwd(Q[pos[i]], [K[p] for p in pos], [V[p] for p in pos], scale, vis_of, order)
        assert np.abs(O_i - O_ref[pos[i]]).max() < 1e-12
        assert np.abs(lse_i - lse_ref[pos[i]]).max() < 1e-12
        D_i = oc.preprocess_bwd(dO[pos[i]], O_i)
        dQ_i = np.zeros((pos[i].size, d))
        for j in order:
            dq, dk, dv = oc.step_bwd(Q[pos[i]], K[pos[j]], V[pos[j]], dO[pos[i]], lse_i, D_i, scale, vis_of(j))
            dQ_i += dq
            dK_tot[pos[j]] += dk
            dV_tot[pos[j]] += dv
        assert np.abs(dQ_i - dQ_ref[pos[i]]).max() < 1e-12
    assert np.abs(dK_tot - dK_ref).max() < 1e-12 and np.abs(dV_tot - dV_ref).max() < 1e-12
    if part == "contiguous":
        assert saw_empty_step   # N/G = 12 > window: shards two or more behind are out of reach


def test_windowed_attention_against_torch_sdpa_mask():
    torch = pytest.importorskip("torch")
    S, d, window = 29, 8, 7
    scale = 1.0 / math.sqrt(d)
    Q, K, V, dO = rand_qkvdo(72, S, S, d)
    vis = oc.visibility(np.arange(S), np.arange(S), True, window)
    O, _ = oc.attention_fwd(Q, K, V, scale, vis)
    dQ, dK, dV = oc.attention_bwd(Q, K, V, dO, scale, vis)
    idx = torch.arange(S)
    band = (idx[:, None] >= idx[None, :]) & (idx[:, None] - idx[None, :] < window)   # written out here, not taken from the oracle
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (Q, K, V))
    out = torch.nn.functional.scaled_dot_product_attention(tq[None, None], tk[None, None], tv[None, None], attn_mask=band)[0, 0]
    out.backward(torch.tensor(dO))
    assert np.abs(out.detach().numpy() - O).max() < 1e-12
    for got, want in ((tq.grad, dQ), (tk.grad, dK), (tv.grad, dV)):
        assert np.abs(got.numpy() - want).max() < 1e-12


# ----------------------------------------------------------------- block-wise sparse

def test_block_mask_brute_force_and_block_diagonal_decouples():
    """apply_block_mask against loops; and a block-diagonal mask makes every block an attention
    problem of its own: O, lse and all gradients equal those of separate per-block calls."""
    r = rng(80)
    nq, nk, bq, bk, d = 24, 30, 8, 10, 4
    M = (r.random((nq // bq, nk // bk)) < 0.5).astype(np.uint8)
    base = oc.visibility(np.arange(nq) + 6, np.arange(nk), True)
    got = oc.apply_block_mask(base, M, bq, bk)
    for a in range(nq):
        for b in range(nk):
            assert got[a, b] == (base[a, b] and M[a // bq, b // bk] != 0)
    n, blk = 24, 8
    Q, K, V, dO = rand_qkvdo(81, n, n, d)
    vis = oc.apply_block_mask(np.ones((n, n), bool), np.eye(n // blk, dtype=np.uint8), blk, blk)
    O, lse = oc.attention_fwd(Q, K, V, 0.6, vis)
    dQ, dK, dV = oc.attention_bwd(Q, K, V, dO, 0.6, vis)
    for t in range(n // blk):
        sl = slice(t * blk, (t + 1) * blk)
        O_t, lse_t = oc.attention_fwd(Q[sl], K[sl], V[sl], 0.6)
        dQ_t, dK_t, dV_t = oc.attention_bwd(Q[sl], K[sl], V[sl], dO[sl], 0.6)
        for whole, part in ((O, O_t), (lse, lse_t), (dQ, dQ_t), (dK, dK_t), (dV, dV_t)):
            assert np.abs(whole[sl] - part).max() < 1e-13


def test_block_sparse_ring_equals_unsharded():
    """Contiguous split with shard-aligned blocks: the ring over per-step block masks (sub-matrices of
    the global one) reproduces unsharded block-sparse attention, rows with no open block included."""
    G, N, d, blk, scale = 3, 36, 4, 4, 0.5
    r = rng(82)
    Q, K, V, dO = rand_qkvdo(83, N, N, d)
    Mg = (r.random((N // blk, N // blk)) < 0.4).astype(np.uint8)
    Mg[2, :] = 0   # a query block that sees nothing at all
    vis_all = oc.apply_block_mask(oc.visibility(np.arange(N), np.arange(N), True), Mg, blk, blk)
    O_ref, lse_ref = oc.attention_fwd(Q, K, V, scale, vis_all)
    n, per = N // G, N // G // blk
    for i in range(G):
        pos_i = oc.contiguous_positions(i, G, N)
        def vis_of(j):
            pos_j = oc.contiguous_positions(j, G, N)
            sub = Mg[i * per:(i + 1) * per, j * per:(j + 1) * per]
            return oc.apply_block_mask(oc.visibility(pos_i, pos_j, True), sub, blk, blk)
        O_i, lse_i = oc.ring_fwd(Q[pos_i], [K[oc.contiguous_positions(j, G, N)] for j in range(G)],
                                 [V[oc.contiguous_positions(j, G, N)] for j in range(G)], scale, vis_of, oc.ring_order(i, G))
        assert np.abs(O_i - O_ref[pos_i]).max() < 1e-12
        fin = np.isfinite(lse_ref[pos_i])
        assert (np.isfinite(lse_i) == fin).all() and np.abs(lse_i[fin] - lse_ref[pos_i][fin]).max() < 1e-12
    assert not np.isfinite(lse_ref[2 * blk:3 * blk]).any() and (O_ref[2 * blk:3 * blk] == 0).all()


@pytest.mark.parametrize("G,N,N_blk", [(2, 48, 8), (4, 96, 16), (3, 54, 18)])
def test_block_striped_split_covers_once_and_slices_every_block(G, N, N_blk):
    """Sec. 3.4, block-wise sparse attention: every device holds the same number of tokens of every
    block, and the devices together hold every token once.  Written out by loops, not via the oracle."""
    m = N_blk // G
    seen = np.zeros(N, int)
    for i in range(G):
        pos = oc.block_striped_positions(i, G, N, N_blk)
        want = [b * N_blk + i * m + t for b in range(N // N_blk) for t in range(m)]
        assert pos.tolist() == want
        assert (np.diff(pos) > 0).all()                       # local row order is position order
        seen[pos] += 1
        for b in range(N // N_blk):
            assert ((pos // N_blk) == b).sum() == m
        # local row block a of m rows lies inside global block a: the step's block mask is M_blk itself
        assert ((pos // N_blk) == np.arange(pos.size) // m).all()
        # the same holds for the striped split of Eq. 13 (tokens i + G*t), the other way to deal out a block
        spos = oc.striped_positions(i, G, N)
        assert ((spos // N_blk) == np.arange(spos.size) // m).all()
    assert (seen == 1).all()
    with pytest.raises(ValueError):
        oc.block_striped_positions(0, G, N, N_blk + 1)


@pytest.mark.parametrize("split", ["block_striped", "striped"])
def test_block_sparse_steps_are_balanced_and_ring_equals_unsharded(split):
    """Under either way of dealing blocks out, (1) the step's visibility by the definition on global
    positions equals the global pattern applied to LOCAL row blocks of N_blk/G rows, (2) every step
    of every device has the same number of visible pairs under a pure block pattern ("exactly the
    same compute workload"), and (3) ring + merge over the steps gives unsharded block-sparse
    attention, also with the causal rule and a window on top."""
    G, N, N_blk, d, scale = 3, 72, 12, 4, 0.5
    m = N_blk // G
    r = rng(84)
    Q, K, V, dO = rand_qkvdo(85, N, N, d)
    Mg = (r.random((N // N_blk, N // N_blk)) < 0.5).astype(np.uint8)
    np.fill_diagonal(Mg, 1)
    pos_of = (lambda i: oc.block_striped_positions(i, G, N, N_blk)) if split == "block_striped" else \
             (lambda i: oc.striped_positions(i, G, N))
    glob = np.arange(N)
    counts = set()
    for causal, window in ((False, 0), (True, 0), (True, 20)):
        vis_all = oc.block_pattern_visibility(glob, glob, Mg, N_blk) & oc.visibility(glob, glob, causal, window)
        O_ref, lse_ref = oc.attention_fwd(Q, K, V, scale, vis_all)
        ring_pairs = []
        for i in range(G):
            pos_i = pos_of(i)
            def vis_of(j):
                pos_j = pos_of(j)
                by_definition = oc.block_pattern_visibility(pos_i, pos_j, Mg, N_blk) & oc.visibility(pos_i, pos_j, causal, window)
                local = oc.apply_block_mask(oc.visibility(pos_i, pos_j, causal, window), Mg, m, m)
                assert (by_definition == local).all()
                return local
            if not causal:
                for j in range(G):
                    counts.add(int(vis_of(j).sum()))
            ring_pairs.append(sum(int(vis_of(j).sum()) for j in range(G)))
            O_i, lse_i = oc.ring_fwd(Q[pos_i], [K[pos_of(j)] for j in range(G)], [V[pos_of(j)] for j in range(G)], scale,
                                     vis_of, oc.ring_order(i, G))
            assert np.abs(O_i - O_ref[pos_i]).max() < 1e-12
            assert np.abs(lse_i - lse_ref[pos_i]).max() < 1e-12
        if causal and not window and split == "striped":
            # token stripes stay balanced under the causal rule as well: devices differ by O(rows), not O(rows^2)
            assert max(ring_pairs) - min(ring_pairs) <= (N // N_blk) * m * G
    assert counts == {int(Mg.sum()) * m * m}


# ----------------------------------------------------------------- planted mistakes are caught

def test_planted_mistakes_fail_the_pins(monkeypatch):
    """Each plausible slip, planted in a copy of the oracle's arithmetic on
    the CPU, must move a pinned quantity by far more than the pin's tolerance."""
    Q, K, V, dO = rand_qkvdo(70, 12, 12, 4)
    scale = 0.5
    vis = oc.visibility(np.arange(12), np.arange(12), True)
    dQ, dK, dV = oc.attention_bwd(Q, K, V, dO, scale, vis)
    f = lambda: loss(Q, K, V, dO, scale, vis)
    fdQ, fdK, fdV = fd_grad(f, Q), fd_grad(f, K), fd_grad(f, V)
    P = oc.attention_probs(Q, K, scale, vis)
    dP = dO @ V.T
    O = P @ V
    D = (dO * O).sum(1)
    dS = P * (dP - D[:, None])
    slips = {
        "dropped scale in dQ": (dS @ K, fdQ),
        "transposed dS in dK": (scale * (dS @ Q), fdK),
        "sign of D": (scale * ((P * (dP + D[:, None])) @ K), fdQ),
        "dV from P not P^T": (P @ dO, fdV),
        "strict causal": (oc.attention_bwd(Q, K, V, dO, scale,
                                           np.tril(np.ones((12, 12), bool), -1) | np.eye(12, dtype=bool)[:, ::-1])[0], fdQ),
    }
    for name, (wrong, ref) in slips.items():
        assert np.abs(wrong - ref).max() > 1e-3, name
    for good, ref in ((dQ, fdQ), (dK, fdK), (dV, fdV)):
        assert np.abs(good - ref).max() < 1e-7
