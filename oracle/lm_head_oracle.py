"""fp64 CPU oracle for the sequence-level fusion of the LM head and the loss
function (Sec. 3.3, Eq. 9, Alg. 3).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module;
only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg do.  It
shares no code with the HIP library and never imports it.

Two forms are given.  `lm_head_loss` is the plain definition the method reaches
exactly: logits, row-wise log-sum-exp, cross-entropy, and the textbook gradient
of the cross-entropy through the softmax and the two matrix products.
`lm_head_loss_tiled` takes the algorithm's steps in its order and notation
(sequence tiles of B_s rows, vocabulary tiles of B_v rows, a running Lse per
sequence tile, the loss from the indexed target rows, then the backward sweep
over the same vocabulary tiles) so the two can be held against each other.

H_last is N x d, W_head is v x d, Y holds N integer targets.

Readings of the paper taken here (the paper is silent or inconsistent):
  * the algorithm prints the one-hot matrix E ADDED to exp(Logits - Lse); the
    gradient of  L = Lse - Logits[y]  with respect to the logits is
    softmax - E, so E is SUBTRACTED here (pinned by finite differences);
  * the index set of vocabulary tile j is printed 1-based; 0-based here;
  * the loss is returned per token (L_i = Lse_i - <H_i, W_head[Y_i]>, the row
    form of the algorithm's loss line); how tokens are reduced is the caller's
    choice, expressed by `grad_scale`, the gradient of the caller's scalar with
    respect to every token's loss (1 for a sum, 1/N for a mean);
  * a target outside [0, v) marks an ignored token: loss 0 and no gradient
    (the paper has no such case; this fixes the behaviour instead of reading
    out of bounds).

Pins: tests/test_oracle_lm_head_pins.py (run with -m "not gpu").
"""
import numpy as np


def row_logsumexp(X):
    """log sum_j exp(X[i, j]) per row; -inf for an empty or all -inf row."""
    if X.shape[1] == 0:
        return np.full(X.shape[0], -np.inf)
    m = X.max(axis=1)
    safe = np.where(np.isfinite(m), m, 0.0)
    with np.errstate(divide="ignore"):
        return safe + np.log(np.exp(X - safe[:, None]).sum(axis=1))


def _valid(Y, v):
    Y = np.asarray(Y, dtype=np.int64)
    return Y, (Y >= 0) & (Y < v)


def lm_head_loss(H, W, Y, grad_scale=1.0):
    """Eq. 9 and its gradient.  Returns (loss[N], lse[N], dH[N, d], dW[v, d])."""
    H, W = np.asarray(H, np.float64), np.asarray(W, np.float64)
    N, v = H.shape[0], W.shape[0]
    Y, ok = _valid(Y, v)
    logits = H @ W.T
    lse = row_logsumexp(logits)
    P = np.exp(logits - lse[:, None])
    E = np.zeros((N, v))
    rows = np.nonzero(ok)[0]
    E[rows, Y[rows]] = 1.0
    loss = np.where(ok, lse - (logits * E).sum(axis=1), 0.0)
    dlogits = grad_scale * (P - E) * ok[:, None]
    return loss, lse, dlogits @ W, dlogits.T @ H


def lm_head_loss_tiled(H, W, Y, B_s, B_v, grad_scale=1.0):
    """Alg. 3 step by step.  Returns (loss[N], lse[N], dH[N, d], dW[v, d])."""
    H, W = np.asarray(H, np.float64), np.asarray(W, np.float64)
    N, v = H.shape[0], W.shape[0]
    Y, ok = _valid(Y, v)
    W_target = W[np.where(ok, Y, 0)]                # index operation, N x d
    loss, lse_all = np.zeros(N), np.zeros(N)
    dH, dW = np.zeros_like(H), np.zeros_like(W)
    for s0 in range(0, N, B_s):
        s1 = min(s0 + B_s, N)
        H_i, Y_i, ok_i = H[s0:s1], Y[s0:s1], ok[s0:s1]
        Lse_i = np.full(s1 - s0, -np.inf)
        logits_i = {}                               # kept for the backward sweep of this sequence tile
        for v0 in range(0, v, B_v):
            W_j = W[v0:min(v0 + B_v, v)]
            Logits_ij = H_i @ W_j.T
            Lse_ij = row_logsumexp(Logits_ij)
            Lse_i = np.logaddexp(Lse_i, Lse_ij)
            logits_i[v0] = Logits_ij
        loss[s0:s1] = np.where(ok_i, -(H_i * W_target[s0:s1]).sum(axis=1) + Lse_i, 0.0)
        lse_all[s0:s1] = Lse_i
        for v0 in range(0, v, B_v):
            v1 = min(v0 + B_v, v)
            W_j = W[v0:v1]
            dLogits_ij = np.exp(logits_i[v0] - Lse_i[:, None])
            Index_j = np.arange(v0, v1)
            E = (Index_j[None, :] == Y_i[:, None]).astype(np.float64)
            G = grad_scale * (dLogits_ij - E) * ok_i[:, None]
            dH[s0:s1] += G @ W_j
            dW[v0:v1] += G.T @ H_i
    return loss, lse_all, dH, dW
