"""fp64 oracle of the token-wise chunked neighbours (Sec. 5.4): plain definitions in numpy.

TEST INFRASTRUCTURE ONLY.  Chunking does not change what these operations compute, so the
oracle is the unchunked definition; inputs are the stored bits widened to fp64.
"""
import numpy as np


def cross_entropy(H, W, target, grad_scale=1.0):
    """logits = H W^T; lse_r = log sum_v exp(logits_r[v]) (max-subtracted); loss_r = lse_r -
    logits_r[target_r]; gradient of sum_r grad_scale * loss_r with respect to H and W.
    Returns dict loss [rows], lse [rows], dH [rows, hidden], dW [vocab, hidden]."""
    H = np.asarray(H, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    t = np.asarray(target, dtype=np.int64)
    logits = H @ W.T
    m = logits.max(axis=1, keepdims=True)
    lse = (m + np.log(np.exp(logits - m).sum(axis=1, keepdims=True)))[:, 0]
    rows = np.arange(H.shape[0])
    loss = lse - logits[rows, t]
    G = np.exp(logits - lse[:, None])
    G[rows, t] -= 1.0
    G *= grad_scale
    return {"loss": loss, "lse": lse, "dH": G @ W, "dW": G.T @ H}
