"""The chunk-by-chunk method of the paper, step by step, in numpy fp64.

TEST INFRASTRUCTURE ONLY.  This is the *method* (Sec. 4.1, Fig. 5 for the
forward; Sec. 4.2, Fig. 7 for the backward), written in the paper's order and
notation: the sequence is cut into u chunks; query chunk q_m visits the
key/value chunks k_i, v_i with i <= m one at a time; every visit yields an
intermediate result that is rescaled when the next chunk is folded in ("online
attention").  It exists to cross-check the unchunked definition in
fpdt_oracle.c -- the two are written in different languages from different
formulas (per-pair local softmax + log-sum-exp merge here, one two-pass softmax
per row there) and must agree to rounding.

Tensors: Q, O, dO, dQ [S, Hq, D]; K, V, dK, dV [S, Hkv, D]; LSE [Hq, S].
"""
import numpy as np


def _pair_scores(q, k, scale, diagonal):
    """scale * q k^T for one chunk pair and one head; -inf above the diagonal
    of a diagonal pair (a query never attends a later key, Sec. 4.2)."""
    s = scale * (q @ k.T)
    if diagonal:
        C = q.shape[0]
        s = np.where(np.arange(C)[None, :] > np.arange(C)[:, None], -np.inf, s)
    return s


def pair_partial(q, k, v, scale, diagonal):
    """Attention of one query chunk against ONE key/value chunk: the partial
    output normalised by that chunk's own softmax, and that chunk's LSE."""
    s = _pair_scores(q, k, scale, diagonal)
    m = s.max(axis=1, keepdims=True)
    e = np.exp(s - m)
    l = e.sum(axis=1, keepdims=True)
    return (e / l) @ v, (m + np.log(l))[:, 0]


def merge(o_a, lse_a, o_b, lse_b):
    """Fold two partial results over disjoint key sets into one (the rescale of
    the intermediate result, Sec. 4.1)."""
    lse = np.logaddexp(lse_a, lse_b)
    o = o_a * np.exp(lse_a - lse)[:, None] + o_b * np.exp(lse_b - lse)[:, None]
    return o, lse


def forward(Q, K, V, chunk, scale, max_inner=None):
    """Forward schedule: outer loop over query chunks m, inner loop over key
    chunks i = 0..m (earlier chunks first, diagonal last).

    max_inner, if given, stops every inner loop after that many key chunks --
    the result must then equal attention restricted to the visited chunks.
    Returns O [S,Hq,D], LSE [Hq,S], and the list of visited (m, i) pairs.
    """
    S, Hq, D = Q.shape
    Hkv = K.shape[1]
    g = Hq // Hkv
    assert S % chunk == 0 and Hq % Hkv == 0
    u = S // chunk
    O = np.zeros((S, Hq, D))
    LSE = np.full((Hq, S), -np.inf)
    visited = []
    for m in range(u):
        rq = slice(m * chunk, (m + 1) * chunk)
        inner = list(range(m + 1))
        if max_inner is not None:
            inner = inner[:max_inner]
        for h in range(Hq):
            o_acc, lse_acc = None, None
            for i in inner:
                rk = slice(i * chunk, (i + 1) * chunk)
                o_p, lse_p = pair_partial(Q[rq, h], K[rk, h // g], V[rk, h // g], scale, i == m)
                if o_acc is None:
                    o_acc, lse_acc = o_p, lse_p
                else:
                    o_acc, lse_acc = merge(o_acc, lse_acc, o_p, lse_p)
            O[rq, h] = o_acc
            LSE[h, rq] = lse_acc
        visited += [(m, i) for i in inner]
    return O, LSE, visited


def backward(Q, K, V, O, LSE, dO, chunk, scale, order="kv_outer", max_pairs=None):
    """Backward schedule over chunk pairs.

    order "kv_outer": outer loop over key/value chunks j, inner over query
    chunks i = j..u-1 (the paper's nested loop, Sec. 4.2); "q_outer": outer
    over query chunks i, inner over j = 0..i.  Every pair adds its share to
    dQ_i, dK_j and dV_j.  max_pairs stops after that many pairs (to check which
    gradients are already final).  Returns dQ, dK, dV and the visited pairs.
    """
    S, Hq, D = Q.shape
    Hkv = K.shape[1]
    g = Hq // Hkv
    u = S // chunk
    Delta = np.einsum("shd,shd->hs", dO, O)
    dQ = np.zeros_like(Q)
    dK = np.zeros_like(K)
    dV = np.zeros_like(V)
    if order == "kv_outer":
        pairs = [(i, j) for j in range(u) for i in range(j, u)]
    elif order == "q_outer":
        pairs = [(i, j) for i in range(u) for j in range(i + 1)]
    else:
        raise ValueError(order)
    if max_pairs is not None:
        pairs = pairs[:max_pairs]
    for (i, j) in pairs:
        rq = slice(i * chunk, (i + 1) * chunk)
        rk = slice(j * chunk, (j + 1) * chunk)
        for h in range(Hq):
            kv = h // g
            s = _pair_scores(Q[rq, h], K[rk, kv], scale, i == j)
            p = np.exp(s - LSE[h, rq][:, None])
            dV[rk, kv] += p.T @ dO[rq, h]
            dP = dO[rq, h] @ V[rk, kv].T
            dS = p * (dP - Delta[h, rq][:, None])
            dQ[rq, h] += scale * (dS @ K[rk, kv])
            dK[rk, kv] += scale * (dS.T @ Q[rq, h])
    return dQ, dK, dV, pairs
