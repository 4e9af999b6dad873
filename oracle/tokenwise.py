"""fp64 oracle of the token-wise chunked neighbours (Sec. 5.4): plain definitions in numpy.

TEST INFRASTRUCTURE ONLY.  Chunking does not change what these operations compute, so the
oracle is the unchunked definition; inputs are the stored bits widened to fp64.
"""
import math

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


def linear(X, W, dY=None):
    """Y = X W^T (Sec. 4.1, the projection of one sequence chunk); with dY also dX = dY W and
    dW = dY^T X.  Returns dict Y [, dX, dW]."""
    X = np.asarray(X, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    out = {"Y": X @ W.T}
    if dY is not None:
        dY = np.asarray(dY, dtype=np.float64)
        out["dX"] = dY @ W
        out["dW"] = dY.T @ X
    return out


_erf = np.vectorize(math.erf, otypes=[np.float64])


def ffn(X, W1, W2, W3=None, dY=None):
    """Feed-forward block.  W3 is None: Y = gelu(X W1^T) W2^T with gelu(a) = a Phi(a), Phi the
    standard normal CDF.  Otherwise Y = (silu(X W1^T) * (X W3^T)) W2^T, silu(a) = a / (1 + e^-a).
    With dY also the gradients of sum(Y * dY): dX, dW1, dW2 (and dW3)."""
    X = np.asarray(X, dtype=np.float64)
    W1 = np.asarray(W1, dtype=np.float64)
    W2 = np.asarray(W2, dtype=np.float64)
    A = X @ W1.T
    if W3 is None:
        Phi = 0.5 * (1.0 + _erf(A / math.sqrt(2.0)))
        Hh = A * Phi
    else:
        W3 = np.asarray(W3, dtype=np.float64)
        B = X @ W3.T
        sg = 1.0 / (1.0 + np.exp(-A))
        Hh = A * sg * B
    out = {"Y": Hh @ W2.T}
    if dY is None:
        return out
    dY = np.asarray(dY, dtype=np.float64)
    dHh = dY @ W2
    out["dW2"] = dY.T @ Hh
    if W3 is None:
        phi = np.exp(-0.5 * A * A) / math.sqrt(2.0 * math.pi)
        dA = dHh * (Phi + A * phi)
        out["dX"] = dA @ W1
    else:
        dA = dHh * B * (sg + A * sg * (1.0 - sg))
        dB = dHh * A * sg
        out["dX"] = dA @ W1 + dB @ W3
        out["dW3"] = dB.T @ X
    out["dW1"] = dA.T @ X
    return out
