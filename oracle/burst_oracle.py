"""fp64 CPU oracle for the per-device compute step of BurstAttention.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module;
only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg do.  It
shares no code with the HIP library and never imports it.

Everything here is plain numpy in float64, written to be checked against the
paper by eye: no tiling, no fusion, no re-ordering.  The only library
primitives used as steps are numpy's matmul, exp, log and max.

Single-head functions take 2-D arrays (rows = tokens, columns = head_dim).
Multi-head wrappers at the bottom loop over (batch, head) and apply the
grouped-query mapping  kv_head = q_head // (Hq // Hkv).

Readings of the paper taken here (the paper is silent or inconsistent):
  * the 1/sqrt(d) factor ("scale") is applied in backward as in forward,
    although both backward algorithms print S = Q K^T without it
    (Alg. 1 / Alg. 2 vs Eq. 4, Eq. 5, forward algorithm);
  * a masked score is excluded from the softmax (treated as -inf), as the
    causal formula Eq. 10 shows, not multiplied by zero as the sentence in
    Sec. 2.2 (4) suggests; the diagonal is visible;
  * D is the per-row scalar rowsum(dO o O) (Alg. 2), broadcast over
    keys, not the N x N product the derivation Eq. 7-8 literally prints;
  * a query row that sees no key in a step emits (O = 0, Lse = -inf) and the
    merge treats exp(-inf) as 0, so merging it is the identity.

Pins: tests/test_oracle_*.py (run with -m "not gpu").
"""
import numpy as np

NEG_INF = -np.inf


# ---------------------------------------------------------------------------
# Partitions of the sequence over G devices: global token positions of the
# rows a device holds, in local row order.
# ---------------------------------------------------------------------------

def contiguous_positions(i, G, N):
    """Device i (0-based) holds tokens [i*N/G, (i+1)*N/G)  (Sec. 3.1)."""
    n = N // G
    return np.arange(i * n, (i + 1) * n, dtype=np.int64)


def zigzag_positions(i, G, N):
    """Zigzag split, Eq. 11, rewritten 0-based: with P = N/(2G), device i
    holds the front piece [i*P, (i+1)*P) followed by the back piece
    [N-(i+1)*P, N-i*P)."""
    P = N // (2 * G)
    front = np.arange(i * P, (i + 1) * P, dtype=np.int64)
    back = np.arange(N - (i + 1) * P, N - i * P, dtype=np.int64)
    return np.concatenate([front, back])


def striped_positions(i, G, N):
    """Striped split, Eq. 13, 0-based: device i holds tokens i + G*m."""
    return np.arange(i, N, G, dtype=np.int64)


def block_striped_positions(i, G, N, N_blk):
    """Block-striped split for block-wise sparse attention (Sec. 3.4, "a strategy similar to
    striped-way workload balance", drawn only in a figure): the sequence is cut into blocks of N_blk
    tokens, N_blk a multiple of G, and every block is dealt to the G devices in G slices of
    N_blk/G consecutive tokens; device i holds slice i of every block, blocks in order.  Every device
    then holds the same number of tokens of every block.  (The other way to deal a block out, token
    i + G*m of every block to device i, is the striped split of Eq. 13 itself, because N_blk is a
    multiple of G: striped_positions.)"""
    if N % N_blk or N_blk % G:
        raise ValueError("N must be a multiple of N_blk and N_blk a multiple of G")
    m = N_blk // G
    starts = np.arange(0, N, N_blk, dtype=np.int64) + i * m
    return (starts[:, None] + np.arange(m, dtype=np.int64)[None, :]).reshape(-1)


def block_pattern_visibility(pos_q, pos_k, pattern, N_blk):
    """Block-wise sparse attention by its definition (Sec. 3.4): with the sequence cut into blocks
    of N_blk tokens, the token at global position p may attend to the token at position p' iff
    M_blk[p // N_blk, p' // N_blk] = 1."""
    pos_q = np.asarray(pos_q, dtype=np.int64)
    pos_k = np.asarray(pos_k, dtype=np.int64)
    pattern = np.asarray(pattern)
    return pattern[(pos_q // N_blk)[:, None], (pos_k // N_blk)[None, :]] != 0


def visibility(pos_q, pos_k, causal, window=0):
    """Boolean [len(pos_q), len(pos_k)]: may query row r use key row c?
    Causal (Eq. 10): a token attends to keys 1..i, itself included.
    window > 0 (sliding-window attention, the sparse pattern of Sec. 3.4 /
    the SWA row of the sparse-attention table): of those keys only the last
    `window` positions, i.e. keys at positions p-window+1 .. p for a query at
    position p.  The paper states no formula for the window; this is the
    usual definition, with the token itself counted in the window."""
    pos_q = np.asarray(pos_q, dtype=np.int64)
    pos_k = np.asarray(pos_k, dtype=np.int64)
    if not causal:
        if window:
            raise ValueError("a window needs a causal mask")
        return np.ones((pos_q.size, pos_k.size), dtype=bool)
    diff = pos_q[:, None] - pos_k[None, :]
    vis = diff >= 0
    if window:
        vis &= diff < window
    return vis


def apply_block_mask(vis, block_mask, q_block_rows, k_block_rows):
    """Block-wise sparse attention (Sec. 3.4): the rows of the query chunk and of
    the key chunk are cut into blocks of q_block_rows / k_block_rows local rows,
    and block_mask[a, b] != 0 says that the queries of block a may attend to the
    keys of block b.  A pair stays visible if `vis` (full, causal or windowed)
    allows it AND its block pair is open.  The blocks are those of the device's
    local rows: under a split that keeps whole global blocks together (the
    striped-like balance of Sec. 3.4) they are the global blocks."""
    vis = np.asarray(vis, dtype=bool)
    block_mask = np.asarray(block_mask)
    nq, nk = vis.shape
    qb = np.arange(nq) // q_block_rows
    kb = np.arange(nk) // k_block_rows
    return vis & (block_mask[qb][:, kb] != 0)


# ---------------------------------------------------------------------------
# The plain definition (Eq. 1 with the exclusion mask of Eq. 10) and its
# textbook gradient.  This is what ring + merge must reproduce.
# ---------------------------------------------------------------------------

def _masked_scores(Q, K, scale, vis):
    S = scale * (np.asarray(Q, np.float64) @ np.asarray(K, np.float64).T)
    if vis is not None:
        S = np.where(vis, S, NEG_INF)
    return S


def row_logsumexp(S):
    """Eq. 6: natural-log logsumexp of every row; -inf for an all-masked row."""
    m = S.max(axis=1) if S.shape[1] else np.full(S.shape[0], NEG_INF)
    safe_m = np.where(np.isfinite(m), m, 0.0)
    with np.errstate(divide="ignore"):
        return safe_m + np.log(np.exp(S - safe_m[:, None]).sum(axis=1))


def attention_probs(Q, K, scale, vis=None):
    """P = Softmax(S) over the visible keys (Eq. 1); all-masked rows are 0."""
    S = _masked_scores(Q, K, scale, vis)
    m = S.max(axis=1) if S.shape[1] else np.full(S.shape[0], NEG_INF)
    safe_m = np.where(np.isfinite(m), m, 0.0)
    E = np.exp(S - safe_m[:, None])
    tot = E.sum(axis=1)
    return E / np.where(tot > 0, tot, 1.0)[:, None]


def attention_fwd(Q, K, V, scale, vis=None):
    """O = Softmax(Q K^T * scale) V and the row logsumexp (Eq. 1, Eq. 6)."""
    P = attention_probs(Q, K, scale, vis)
    O = P @ np.asarray(V, np.float64)
    lse = row_logsumexp(_masked_scores(Q, K, scale, vis))
    return O, lse


def attention_bwd(Q, K, V, dO, scale, vis=None):
    """Gradient of L = sum(O o dO) w.r.t. Q, K, V through the softmax
    Jacobian  dS = P o dP - P o rowsum(P o dP)  (first line of Eq. 7)."""
    Q = np.asarray(Q, np.float64)
    K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64)
    dO = np.asarray(dO, np.float64)
    P = attention_probs(Q, K, scale, vis)
    dV = P.T @ dO
    dP = dO @ V.T
    dS = P * dP - P * (P * dP).sum(axis=1, keepdims=True)
    dQ = scale * (dS @ K)
    dK = scale * (dS.T @ Q)
    return dQ, dK, dV


# ---------------------------------------------------------------------------
# The sharded method, step by step, in the paper's notation.
# ---------------------------------------------------------------------------

def step_fwd(Qi, Kj, Vj, scale, vis=None):
    """One local attention step (Eq. 5-6; forward algorithm):
    S_ij = Q_i K_j^T * scale, Lse = LSE(S_ij), P_ij = exp(S_ij - Lse),
    O_ij = P_ij V_j.  Returns (O_ij, Lse_current)."""
    S = _masked_scores(Qi, Kj, scale, vis)
    lse = row_logsumexp(S)
    safe = np.where(np.isfinite(lse), lse, 0.0)
    P = np.exp(S - safe[:, None])
    P = np.where(np.isfinite(lse)[:, None], P, 0.0)
    return P @ np.asarray(Vj, np.float64), lse


def lse_merge(O_i, lse_i, O_ij, lse_cur):
    """Fold a step's (O_ij, Lse_current) into the running (O_i, Lse_i)
    (forward algorithm):
      Lse' = log(exp(Lse_i) + exp(Lse_current))
      O_i  = exp(Lse_current - Lse') O_ij + exp(Lse_i - Lse') O_i
    with exp(-inf) = 0 and (-inf, -inf) merging to (0, -inf)."""
    O_i = np.asarray(O_i, np.float64)
    O_ij = np.asarray(O_ij, np.float64)
    a = np.asarray(lse_i, np.float64)
    b = np.asarray(lse_cur, np.float64)
    m = np.maximum(a, b)
    dead = ~np.isfinite(m)
    safe_m = np.where(dead, 0.0, m)
    with np.errstate(divide="ignore"):
        new = safe_m + np.log(np.exp(a - safe_m) + np.exp(b - safe_m))
    new = np.where(dead, NEG_INF, new)
    safe_new = np.where(dead, 0.0, new)
    w_old = np.where(dead, 0.0, np.exp(a - safe_new))
    w_cur = np.where(dead, 0.0, np.exp(b - safe_new))
    return w_cur[:, None] * O_ij + w_old[:, None] * O_i, new


def ring_order(i, G, reverse=False):
    """Order in which device i meets the KV shards: its own first, then the
    ring neighbours one after the other (Sec. 3.4: local attention first,
    then communicate)."""
    if reverse:
        return [(i + t) % G for t in range(G)]
    return [(i - t) % G for t in range(G)]


def ring_fwd(Qi, K_shards, V_shards, scale, vis_of_shard, order):
    """Forward algorithm on one device: initialise O_i = 0, Lse_i = -inf,
    then for every shard j in `order` run step_fwd and lse_merge.
    vis_of_shard(j) returns the visibility matrix of Q_i against shard j
    (or None for a full mask)."""
    n, d = np.asarray(Qi).shape[0], np.asarray(V_shards[0]).shape[1]
    O = np.zeros((n, d))
    lse = np.full(n, NEG_INF)
    for j in order:
        O_ij, lse_cur = step_fwd(Qi, K_shards[j], V_shards[j], scale, vis_of_shard(j))
        O, lse = lse_merge(O, lse, O_ij, lse_cur)
    return O, lse


def preprocess_bwd(dO, O):
    """D = rowsum(dO o O), once per ring (Alg. 2)."""
    return (np.asarray(dO, np.float64) * np.asarray(O, np.float64)).sum(axis=1)


def step_bwd(Q, K, V, dO, lse, D, scale, vis=None):
    """One backward step (Alg. 2, same arithmetic as the local step of
    Alg. 1) for query rows Q (with their FINAL Lse and D) against key/value
    rows K, V.  Returns this step's contributions (dQ, dK, dV):
      S = Q K^T * scale;  P = exp(S - Lse);  dV = P^T dO;  dP = dO V^T;
      dS = P o (dP - D);  dK = scale dS^T Q;  dQ = scale dS K."""
    Q = np.asarray(Q, np.float64)
    K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64)
    dO = np.asarray(dO, np.float64)
    lse = np.asarray(lse, np.float64)
    D = np.asarray(D, np.float64)
    S = _masked_scores(Q, K, scale, vis)
    alive = np.isfinite(lse)
    P = np.exp(S - np.where(alive, lse, 0.0)[:, None])
    P = np.where(alive[:, None], P, 0.0)
    dV = P.T @ dO
    dP = dO @ V.T
    dS = P * (dP - D[:, None])
    dK = scale * (dS.T @ Q)
    dQ = scale * (dS @ K)
    return dQ, dK, dV


def ring_bwd_burst(i, Q_shards, dO_shards, lse_shards, D_shards, Ki, Vi, scale,
                   vis_of_pair, order):
    """Alg. 2 as seen from device i: K_i, V_i, dK_i, dV_i stay; the bundles
    (Q_j, dQ_j, dO_j, D_j, Lse_j) visit in `order`.  Returns (dK_i, dV_i,
    {j: device i's contribution to dQ_j}).  vis_of_pair(j, i) is the
    visibility of Q_j's rows against K_i's rows."""
    dK = np.zeros_like(np.asarray(Ki, np.float64))
    dV = np.zeros_like(np.asarray(Vi, np.float64))
    dQ_contrib = {}
    for j in order:
        dq, dk, dv = step_bwd(Q_shards[j], Ki, Vi, dO_shards[j], lse_shards[j],
                              D_shards[j], scale, vis_of_pair(j, i))
        dK += dk
        dV += dv
        dQ_contrib[j] = dq
    return dK, dV, dQ_contrib


def ring_bwd_ring(i, Qi, dOi, Oi, lse_i, K_shards, V_shards, scale, vis_of_pair, order):
    """Alg. 1 as seen from device i: Q_i, dO_i, O_i, Lse_i stay and dQ_i is
    accumulated locally; (K_j, V_j, dK_j, dV_j) visit in `order`, and D_i is
    recomputed every round (Alg. 1).  Returns (dQ_i, {j: device i's
    contribution to dK_j}, {j: ... dV_j})."""
    dQ = np.zeros_like(np.asarray(Qi, np.float64))
    dK_contrib, dV_contrib = {}, {}
    for j in order:
        D_i = preprocess_bwd(dOi, Oi)
        dq, dk, dv = step_bwd(Qi, K_shards[j], V_shards[j], dOi, lse_i, D_i, scale,
                              vis_of_pair(i, j))
        dQ += dq
        dK_contrib[j] = dk
        dV_contrib[j] = dv
    return dQ, dK_contrib, dV_contrib


# ---------------------------------------------------------------------------
# Zigzag step written as the case table Eq. 12 with explicit slices (no
# positions involved), to pin the position predicate against.
# ---------------------------------------------------------------------------

def zigzag_step_fwd_cases(i, j, Qi, Kj, Vj, scale):
    """O_ij and Lse_current of device i against shard j under the zigzag
    split, by the three cases of Eq. 12.  Local rows are ordered front piece
    then back piece; P = rows // 2.  Rows outside the case's query set keep
    (0, -inf)."""
    Qi = np.asarray(Qi, np.float64)
    P = Qi.shape[0] // 2
    d = np.asarray(Vj).shape[1]
    O = np.zeros((2 * P, d))
    lse = np.full(2 * P, NEG_INF)
    if i == j:
        # causal attention on the device's own pair of pieces: local row
        # order is also position order, so the mask is lower-triangular.
        tri = np.tril(np.ones((2 * P, 2 * P), dtype=bool))
        O, lse = step_fwd(Qi, Kj, Vj, scale, tri)
    elif i < j:
        # only the back queries, against both key pieces, unmasked
        O[P:], lse[P:] = step_fwd(Qi[P:], Kj, Vj, scale, None)
    else:
        # all queries, against the front key piece only, unmasked
        O, lse = step_fwd(Qi, Kj[:P], Vj[:P], scale, None)
    return O, lse


# ---------------------------------------------------------------------------
# Multi-head wrappers.  Tensors are [batch, seq, heads, head_dim].
# ---------------------------------------------------------------------------

def kv_head_of(h, Hq, Hkv):
    """Grouped-query mapping (not in the paper, which treats one head):
    consecutive groups of Hq/Hkv query heads share one KV head."""
    return h // (Hq // Hkv)


def mha_step_fwd(Q, K, V, scale, vis=None):
    B, Sq, Hq, d = Q.shape
    Hkv = K.shape[2]
    O = np.zeros((B, Sq, Hq, V.shape[3]))
    lse = np.full((B, Hq, Sq), NEG_INF)
    for b in range(B):
        for h in range(Hq):
            g = kv_head_of(h, Hq, Hkv)
            O[b, :, h], lse[b, h] = step_fwd(Q[b, :, h], K[b, :, g], V[b, :, g], scale, vis)
    return O, lse


def mha_lse_merge(O_acc, lse_acc, O_part, lse_part):
    B, Sq, Hq, d = O_acc.shape
    O = np.empty((B, Sq, Hq, d))
    lse = np.empty((B, Hq, Sq))
    for b in range(B):
        for h in range(Hq):
            O[b, :, h], lse[b, h] = lse_merge(O_acc[b, :, h], lse_acc[b, h],
                                              O_part[b, :, h], lse_part[b, h])
    return O, lse


def mha_preprocess_bwd(dO, O):
    B, Sq, Hq, d = O.shape
    D = np.empty((B, Hq, Sq))
    for b in range(B):
        for h in range(Hq):
            D[b, h] = preprocess_bwd(dO[b, :, h], O[b, :, h])
    return D


def mha_step_bwd(Q, K, V, dO, lse, D, scale, vis=None):
    """dK and dV of a KV head are summed over the query heads of its group."""
    B, Sq, Hq, d = Q.shape
    Hkv = K.shape[2]
    dQ = np.zeros(Q.shape)
    dK = np.zeros(K.shape)
    dV = np.zeros(V.shape)
    for b in range(B):
        for h in range(Hq):
            g = kv_head_of(h, Hq, Hkv)
            dq, dk, dv = step_bwd(Q[b, :, h], K[b, :, g], V[b, :, g], dO[b, :, h],
                                  lse[b, h], D[b, h], scale, vis)
            dQ[b, :, h] = dq
            dK[b, :, g] += dk
            dV[b, :, g] += dv
    return dQ, dK, dV


def mha_attention_fwd(Q, K, V, scale, vis=None):
    B, Sq, Hq, d = Q.shape
    Hkv = K.shape[2]
    O = np.zeros((B, Sq, Hq, V.shape[3]))
    lse = np.full((B, Hq, Sq), NEG_INF)
    for b in range(B):
        for h in range(Hq):
            g = kv_head_of(h, Hq, Hkv)
            O[b, :, h], lse[b, h] = attention_fwd(Q[b, :, h], K[b, :, g], V[b, :, g], scale, vis)
    return O, lse


def mha_attention_bwd(Q, K, V, dO, scale, vis=None):
    B, Sq, Hq, d = Q.shape
    Hkv = K.shape[2]
    dQ = np.zeros(Q.shape)
    dK = np.zeros(K.shape)
    dV = np.zeros(V.shape)
    for b in range(B):
        for h in range(Hq):
            g = kv_head_of(h, Hq, Hkv)
            dq, dk, dv = attention_bwd(Q[b, :, h], K[b, :, g], V[b, :, g], dO[b, :, h], scale, vis)
            dQ[b, :, h] = dq
            dK[b, :, g] += dk
            dV[b, :, g] += dv
    return dQ, dK, dV


# ---------------------------------------------------------------------------
# Work counting (the benchmark's FLOP convention): visible (q, k) pairs.
# ---------------------------------------------------------------------------

def visible_pairs(pos_q, pos_k, causal, window=0):
    return int(visibility(pos_q, pos_k, causal, window).sum())
