"""Pins for the fp64 oracle: everything here checks oracle/ against something
other than itself -- hand-derived closed forms, a library autodiff, brute-force
finite differences, invariants of the mathematics, and the step-by-step chunked
method against the one-shot definition."""
import json
import math
import os

import numpy as np
import pytest
import torch

from oracle import chunked, definition

HERE = os.path.dirname(os.path.abspath(__file__))


def rand(S, Hq, Hkv, D, seed):
    r = np.random.default_rng(seed)
    return (r.standard_normal((S, Hq, D)), r.standard_normal((S, Hkv, D)),
            r.standard_normal((S, Hkv, D)), r.standard_normal((S, Hq, D)))


def torch_reference(Q, K, V, dO, scale, allowed=None):
    """Library pin: masked softmax + autograd in fp64 (no formula of ours).
    allowed: optional [S,S] boolean matrix ANDed with the causal mask."""
    q = torch.tensor(Q, requires_grad=True)
    k = torch.tensor(K, requires_grad=True)
    v = torch.tensor(V, requires_grad=True)
    S, Hq, D = Q.shape
    g = Hq // K.shape[1]
    kk = k.repeat_interleave(g, dim=1)
    vv = v.repeat_interleave(g, dim=1)
    s = scale * torch.einsum("ihd,jhd->hij", q, kk)
    mask = torch.ones(S, S, dtype=torch.bool).tril()
    if allowed is not None:
        mask = mask & torch.tensor(allowed)
    s = s.masked_fill(~mask, float("-inf"))
    lse = torch.logsumexp(s, dim=-1)
    o = torch.einsum("hij,jhd->ihd", torch.softmax(s, dim=-1), vv)
    (o * torch.tensor(dO)).sum().backward()
    return (o.detach().numpy(), lse.detach().numpy(), q.grad.numpy(), k.grad.numpy(),
            v.grad.numpy())


def _expr(x):
    if isinstance(x, (int, float)):
        return float(x)
    return float(eval(x, {"__builtins__": {}}, {"ln2": math.log(2), "ln3": math.log(3),
                                                 "ln6": math.log(6)}))


def test_golden_closed_form_s3():
    g = json.load(open(os.path.join(HERE, "golden", "closed_form_s3.json")))
    col = lambda name: np.array([_expr(x) for x in g[name]]).reshape(g["S"], 1, 1)
    r = definition.attn_fwd_bwd(col("Q"), col("K"), col("V"), col("dO"), g["scale"])
    for name in ("O", "dQ", "dK", "dV"):
        np.testing.assert_allclose(r[name], col(name), rtol=0, atol=1e-14, err_msg=name)
    np.testing.assert_allclose(r["LSE"][0], [_expr(x) for x in g["LSE"]], rtol=0, atol=1e-14)
    # the chunked method on the same fixture (chunk = 1: three chunks)
    O, LSE, _ = chunked.forward(col("Q"), col("K"), col("V"), 1, g["scale"])
    np.testing.assert_allclose(O, col("O"), atol=1e-14)
    dQ, dK, dV, _ = chunked.backward(col("Q"), col("K"), col("V"), O, LSE, col("dO"), 1,
                                     g["scale"])
    np.testing.assert_allclose(dQ, col("dQ"), atol=1e-14)
    np.testing.assert_allclose(dK, col("dK"), atol=1e-14)
    np.testing.assert_allclose(dV, col("dV"), atol=1e-14)


@pytest.mark.parametrize("S,Hq,Hkv,D", [(33, 1, 1, 8), (48, 4, 2, 16), (40, 8, 1, 5),
                                        (17, 2, 2, 64)])
def test_against_torch_autograd(S, Hq, Hkv, D):
    Q, K, V, dO = rand(S, Hq, Hkv, D, 1)
    scale = 0.37
    r = definition.attn_fwd_bwd(Q, K, V, dO, scale)
    O, LSE, dQ, dK, dV = torch_reference(Q, K, V, dO, scale)
    for name, ref in (("O", O), ("LSE", LSE), ("dQ", dQ), ("dK", dK), ("dV", dV)):
        np.testing.assert_allclose(r[name], ref, rtol=1e-11, atol=1e-12, err_msg=name)


@pytest.mark.parametrize("S,Hq,Hkv,D", [(6, 1, 1, 3), (9, 2, 1, 4), (7, 4, 2, 2)])
def test_gradients_by_finite_differences(S, Hq, Hkv, D):
    """Brute force: L = sum(O * W); every element of dQ, dK, dV by central differences."""
    Q, K, V, W = rand(S, Hq, Hkv, D, 2)
    scale = 1.0 / math.sqrt(D)
    r = definition.attn_fwd_bwd(Q, K, V, W, scale)
    loss = lambda q, k, v: float((definition.attn_fwd(q, k, v, scale)[0] * W).sum())
    eps = 1e-6
    for name, X, idx in (("dQ", Q, 0), ("dK", K, 1), ("dV", V, 2)):
        num = np.zeros_like(X)
        for pos in np.ndindex(*X.shape):
            args = [Q.copy(), K.copy(), V.copy()]
            args[idx][pos] += eps
            up = loss(*args)
            args[idx][pos] -= 2 * eps
            num[pos] = (up - loss(*args)) / (2 * eps)
        np.testing.assert_allclose(r[name], num, rtol=1e-6, atol=1e-8, err_msg=name)


def test_forward_closed_forms():
    S, Hq, Hkv, D = 64, 4, 2, 8
    Q, K, V, dO = rand(S, Hq, Hkv, D, 3)
    scale = 0.5
    O, LSE = definition.attn_fwd(Q, K, V, scale)
    # row 0 sees only key 0
    np.testing.assert_allclose(O[0], np.repeat(V[0], 2, axis=0), atol=1e-15)
    np.testing.assert_allclose(LSE[:, 0], scale * np.einsum("hd,hd->h", Q[0],
                                                            np.repeat(K[0], 2, axis=0)), atol=1e-14)
    # K == 0: uniform causal average, LSE_i = log(i + 1)
    O0, LSE0 = definition.attn_fwd(Q, np.zeros_like(K), V, scale)
    cum = np.cumsum(V, axis=0) / np.arange(1, S + 1)[:, None, None]
    np.testing.assert_allclose(O0, np.repeat(cum, 2, axis=1), atol=1e-14)
    np.testing.assert_allclose(LSE0, np.tile(np.log(np.arange(1, S + 1)), (Hq, 1)), atol=1e-14)
    # V constant along the sequence: rows of p sum to one, so O is that constant
    Vc = np.broadcast_to(V[:1], V.shape).copy()
    Oc, _ = definition.attn_fwd(Q, K, Vc, scale)
    np.testing.assert_allclose(Oc, np.broadcast_to(np.repeat(V[:1], 2, axis=1), Oc.shape),
                               atol=1e-14)
    # exp(LSE) equals the direct sum where that does not overflow
    h, i = 3, 40
    direct = np.exp(scale * K[: i + 1, h // 2] @ Q[i, h]).sum()
    assert abs(math.exp(LSE[h, i]) - direct) <= 1e-12 * direct


def test_backward_invariants():
    S, Hq, Hkv, D = 96, 4, 2, 8
    g = Hq // Hkv
    Q, K, V, dO = rand(S, Hq, Hkv, D, 4)
    scale = 0.41
    r = definition.attn_fwd_bwd(Q, K, V, dO, scale)
    # rows of p sum to one: sum_j dV_j = sum over the group's heads and rows of dO
    want = dO.reshape(S, Hkv, g, D).sum(axis=(0, 2))
    np.testing.assert_allclose(r["dV"].sum(axis=0), want, rtol=1e-12, atol=1e-12)
    # gauge identity: Q K^T is invariant under Q -> Q A, K -> K A^-T, hence
    # sum_h Q_h^T dQ_h = dK^T K per KV head (D x D matrices)
    for kv in range(Hkv):
        lhs = sum(Q[:, h].T @ r["dQ"][:, h] for h in range(kv * g, (kv + 1) * g))
        rhs = r["dK"][:, kv].T @ K[:, kv]
        np.testing.assert_allclose(lhs, rhs, rtol=1e-11, atol=1e-11)
    # K constant along the sequence: sum_j dS_ij = 0 makes dQ vanish
    Kc = np.broadcast_to(K[:1], K.shape).copy()
    rc = definition.attn_fwd_bwd(Q, Kc, V, dO, scale)
    assert np.abs(rc["dQ"]).max() < 1e-13
    # V constant along the sequence: dP_ij = Delta_i, so dS = 0 and dQ = dK = 0
    Vc = np.broadcast_to(V[:1], V.shape).copy()
    rv = definition.attn_fwd_bwd(Q, K, Vc, dO, scale)
    assert np.abs(rv["dQ"]).max() < 1e-13 and np.abs(rv["dK"]).max() < 1e-13
    # Delta is rowsum(dO * O)
    np.testing.assert_allclose(r["Delta"], np.einsum("shd,shd->hs", dO, r["O"]), atol=1e-13)


@pytest.mark.parametrize("S,chunk,Hq,Hkv,D", [(128, 128, 2, 2, 8), (128, 32, 4, 1, 16),
                                              (96, 32, 4, 2, 8), (120, 24, 2, 1, 12),
                                              (64, 1, 1, 1, 4)])
@pytest.mark.parametrize("order", ["kv_outer", "q_outer"])
def test_chunked_method_equals_definition(S, chunk, Hq, Hkv, D, order):
    Q, K, V, dO = rand(S, Hq, Hkv, D, 5)
    scale = 1.0 / math.sqrt(D)
    r = definition.attn_fwd_bwd(Q, K, V, dO, scale)
    O, LSE, visited = chunked.forward(Q, K, V, chunk, scale)
    u = S // chunk
    assert len(visited) == u * (u + 1) // 2
    tol = lambda ref: 1e-12 * (1 + np.abs(ref).max())
    assert np.abs(O - r["O"]).max() <= tol(r["O"])
    assert np.abs(LSE - r["LSE"]).max() <= tol(r["LSE"])
    dQ, dK, dV, pairs = chunked.backward(Q, K, V, O, LSE, dO, chunk, scale, order)
    assert len(pairs) == u * (u + 1) // 2
    for name, got in (("dQ", dQ), ("dK", dK), ("dV", dV)):
        assert np.abs(got - r[name]).max() <= tol(r[name]), name


def test_chunked_single_chunk_is_deterministic():
    Q, K, V, dO = rand(64, 2, 1, 8, 6)
    a = chunked.forward(Q, K, V, 64, 0.3)
    b = chunked.forward(Q, K, V, 64, 0.3)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_merge_of_disjoint_key_sets():
    """Two partial softmaxes over disjoint keys, merged, equal the one-shot one."""
    r = np.random.default_rng(7)
    q, k, v = r.standard_normal((16, 8)), r.standard_normal((40, 8)), r.standard_normal((40, 8))
    oa, la = chunked.pair_partial(q, k[:16], v[:16], 0.6, False)
    ob, lb = chunked.pair_partial(q, k[16:], v[16:], 0.6, False)
    o, l = chunked.merge(oa, la, ob, lb)
    s = torch.tensor(0.6 * q @ k.T)
    np.testing.assert_allclose(o, (torch.softmax(s, -1) @ torch.tensor(v)).numpy(), atol=1e-14)
    np.testing.assert_allclose(l, torch.logsumexp(s, -1).numpy(), atol=1e-14)


def test_truncated_forward_is_attention_over_visited_chunks():
    """After the first k inner steps a query chunk holds attention restricted to
    the visited key chunks; chunk 0 is final after one step (Sec. 4.1)."""
    S, chunk, Hq, Hkv, D = 128, 32, 2, 1, 8
    Q, K, V, dO = rand(S, Hq, Hkv, D, 8)
    scale = 0.35
    full, _ = definition.attn_fwd(Q, K, V, scale)
    O2, LSE2, _ = chunked.forward(Q, K, V, chunk, scale, max_inner=2)
    # chunks 0 and 1 have at most two inner steps: already final
    np.testing.assert_allclose(O2[: 2 * chunk], full[: 2 * chunk], atol=1e-13)
    # chunk 3 has seen key chunks 0 and 1 only, unmasked
    m = 3
    rows = np.arange(m * chunk, (m + 1) * chunk)
    for h in range(Hq):
        s = torch.tensor(scale * Q[rows, h] @ K[: 2 * chunk, 0].T)
        ref = (torch.softmax(s, -1) @ torch.tensor(V[: 2 * chunk, 0])).numpy()
        np.testing.assert_allclose(O2[rows, h], ref, atol=1e-13)


def test_backward_schedule_finality():
    """KV-outer order: dq_0 is final after the first inner step, dk_0 and dv_0
    after the first outer iteration (Sec. 4.2)."""
    S, chunk, Hq, Hkv, D = 128, 32, 2, 2, 8
    u = S // chunk
    Q, K, V, dO = rand(S, Hq, Hkv, D, 9)
    scale = 0.35
    r = definition.attn_fwd_bwd(Q, K, V, dO, scale)
    dQ, dK, dV, pairs = chunked.backward(Q, K, V, r["O"], r["LSE"], dO, chunk, scale,
                                         "kv_outer", max_pairs=1)
    assert pairs == [(0, 0)]
    np.testing.assert_allclose(dQ[:chunk], r["dQ"][:chunk], atol=1e-13)
    dQ, dK, dV, pairs = chunked.backward(Q, K, V, r["O"], r["LSE"], dO, chunk, scale,
                                         "kv_outer", max_pairs=u)
    assert pairs == [(i, 0) for i in range(u)]
    np.testing.assert_allclose(dK[:chunk], r["dK"][:chunk], atol=1e-13)
    np.testing.assert_allclose(dV[:chunk], r["dV"][:chunk], atol=1e-13)
    assert np.abs(dK[chunk:]).max() == 0.0
    # Q-outer order: after the first i+1 pairs of query chunk i its dq is final
    dQ, _, _, pairs = chunked.backward(Q, K, V, r["O"], r["LSE"], dO, chunk, scale,
                                       "q_outer", max_pairs=3)
    assert pairs == [(0, 0), (1, 0), (1, 1)]
    np.testing.assert_allclose(dQ[: 2 * chunk], r["dQ"][: 2 * chunk], atol=1e-13)


def test_sampled_rows_and_tail_window_match_full():
    S, Hq, Hkv, D = 200, 4, 2, 8
    Q, K, V, dO = rand(S, Hq, Hkv, D, 10)
    scale = 0.3
    r = definition.attn_fwd_bwd(Q, K, V, dO, scale)
    idx = np.array([0, 1, 63, 64, 65, 199, 128])
    s = definition.rows(Q[idx], K, V, idx, scale, dOr=dO[idx])
    assert np.array_equal(s["O"], r["O"][idx]) and np.array_equal(s["dQ"], r["dQ"][idx])
    assert np.array_equal(s["LSE"], r["LSE"][:, idx])
    w = 37
    t = definition.tail_window(Q[S - w:], dO[S - w:], K, V, w, scale)
    np.testing.assert_allclose(t["dK"], r["dK"][S - w:], rtol=0, atol=1e-14)
    np.testing.assert_allclose(t["dV"], r["dV"][S - w:], rtol=0, atol=1e-14)


def test_oracle_rejects_bad_arguments():
    Q, K, V, dO = rand(8, 3, 2, 4, 11)   # Hq not a multiple of Hkv
    with pytest.raises(ValueError):
        definition.attn_fwd(Q, K, V, 1.0)
    Q, K, V, dO = rand(8, 2, 2, 4, 11)
    with pytest.raises(ValueError):
        definition.rows(Q[:1], K, V, np.array([8]), 1.0)


# ---- block-sparse variant (Sec. 5.5): a chunk-level mask on top of the causal one ----
def _chunk_masks(u, seed):
    r = np.random.default_rng(seed)
    m = np.tril(r.random((u, u)) < 0.5)
    np.fill_diagonal(m, True)
    return m


@pytest.mark.parametrize("S,chunk,Hq,Hkv,D", [(48, 8, 2, 1, 8), (40, 10, 4, 2, 5), (36, 12, 1, 1, 16)])
def test_blocksparse_against_torch_autograd(S, chunk, Hq, Hkv, D):
    Q, K, V, dO = rand(S, Hq, Hkv, D, 11)
    cm = _chunk_masks(S // chunk, 12)
    assert not cm[np.tril_indices(S // chunk)].all()  # something below the diagonal is dropped
    allowed = np.kron(cm, np.ones((chunk, chunk), dtype=bool))
    r = definition.attn_fwd_bwd(Q, K, V, dO, 0.41, chunk=chunk, chunk_mask=cm)
    O, LSE, dQ, dK, dV = torch_reference(Q, K, V, dO, 0.41, allowed=allowed)
    for name, ref in (("O", O), ("LSE", LSE), ("dQ", dQ), ("dK", dK), ("dV", dV)):
        np.testing.assert_allclose(r[name], ref, rtol=1e-11, atol=1e-12, err_msg=name)


def test_blocksparse_full_mask_is_the_dense_definition():
    S, chunk = 64, 16
    Q, K, V, dO = rand(S, 4, 2, 8, 13)
    dense = definition.attn_fwd_bwd(Q, K, V, dO, 0.3)
    full = definition.attn_fwd_bwd(Q, K, V, dO, 0.3, chunk=chunk, chunk_mask=np.ones((4, 4)))
    for name in ("O", "LSE", "Delta", "dQ", "dK", "dV"):
        assert np.array_equal(dense[name], full[name]), name
    # entries above the diagonal are never read
    junk = np.tril(np.ones((4, 4))) + np.triu(np.ones((4, 4)), 1) * 7
    r = definition.attn_fwd_bwd(Q, K, V, dO, 0.3, chunk=chunk, chunk_mask=junk)
    assert np.array_equal(dense["dK"], r["dK"])


def test_blocksparse_reduces_to_dense_attention_over_the_kept_chunks():
    """Rows of query chunk m equal dense causal attention over the concatenation of the key
    chunks it keeps (they all precede it, so only its own chunk is masked inside)."""
    S, chunk, Hq, Hkv, D = 60, 12, 2, 2, 6
    u = S // chunk
    Q, K, V, dO = rand(S, Hq, Hkv, D, 14)
    cm = _chunk_masks(u, 15)
    sp = definition.rows(Q, K, V, np.arange(S), 0.5, dOr=dO, chunk=chunk, chunk_mask=cm)
    for m in range(u):
        kept = [i for i in range(m + 1) if cm[m, i]]
        sel = np.concatenate([np.arange(i * chunk, (i + 1) * chunk) for i in kept])
        rows_m = np.arange(m * chunk, (m + 1) * chunk)
        local = np.arange((len(kept) - 1) * chunk, len(kept) * chunk)  # chunk m comes last
        d = definition.rows(Q[rows_m], K[sel], V[sel], local, 0.5, dOr=dO[rows_m])
        np.testing.assert_allclose(sp["O"][rows_m], d["O"], atol=1e-14)
        np.testing.assert_allclose(sp["LSE"][:, rows_m], d["LSE"], atol=1e-14)
        np.testing.assert_allclose(sp["dQ"][rows_m], d["dQ"], atol=1e-13)


def test_blocksparse_closed_form_and_invariants():
    S, chunk, Hq, Hkv, D = 40, 8, 2, 1, 4
    u = S // chunk
    Q, K, V, dO = rand(S, Hq, Hkv, D, 16)
    cm = _chunk_masks(u, 17)
    # K == 0: uniform average over the allowed keys, LSE = log(their number)
    O0, LSE0 = (lambda r: (r["O"], r["LSE"]))(definition.rows(Q, np.zeros_like(K), V, np.arange(S), 0.7,
                                                                chunk=chunk, chunk_mask=cm))
    allowed = np.kron(cm, np.ones((chunk, chunk), dtype=bool)) & np.tril(np.ones((S, S), dtype=bool))
    cnt = allowed.sum(axis=1)
    mean = (allowed[:, :, None, None] * V[None]).sum(axis=1) / cnt[:, None, None]
    np.testing.assert_allclose(O0, np.repeat(mean, Hq, axis=1), atol=1e-14)
    np.testing.assert_allclose(LSE0, np.tile(np.log(cnt), (Hq, 1)), atol=1e-14)
    # rows of P still sum to one: sum_j dV_j = sum_i dO_i per KV head; a key chunk nobody but
    # its own diagonal reads gets gradient only from its own chunk's rows
    r = definition.attn_fwd_bwd(Q, K, V, dO, 0.7, chunk=chunk, chunk_mask=cm)
    np.testing.assert_allclose(r["dV"].sum(axis=0)[0], dO.sum(axis=(0, 1)), atol=1e-12)
    lonely = [j for j in range(u) if not cm[j + 1:, j].any()]
    assert lonely
    j = lonely[0]
    rows_j = np.arange(j * chunk, (j + 1) * chunk)
    Q2, dO2 = Q.copy(), dO.copy()
    other = np.setdiff1d(np.arange(S), rows_j)
    Q2[other] += 1.0
    dO2[other] *= -3.0
    r2 = definition.attn_fwd_bwd(Q2, K, V, dO2, 0.7, chunk=chunk, chunk_mask=cm)
    np.testing.assert_array_equal(r["dK"][rows_j], r2["dK"][rows_j])
    np.testing.assert_array_equal(r["dV"][rows_j], r2["dV"][rows_j])


def test_blocksparse_oracle_rejects_bad_masks():
    Q, K, V, dO = rand(16, 1, 1, 4, 18)
    bad = np.ones((4, 4))
    bad[2, 2] = 0  # a dropped diagonal entry would leave rows without any key
    with pytest.raises(ValueError):
        definition.rows(Q, K, V, np.arange(16), 1.0, chunk=4, chunk_mask=bad)
    with pytest.raises(AssertionError):
        definition.rows(Q, K, V, np.arange(16), 1.0, chunk=5, chunk_mask=np.ones((3, 3)))
