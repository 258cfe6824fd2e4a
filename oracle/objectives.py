"""TEST INFRASTRUCTURE ONLY — the local stochastic gradients g_i(x_i) of the
synthetic objectives, in fp64.

The paper leaves f_i abstract ("Application Layer": each worker sees only a
stochastic gradient oracle of its own loss); these are textbook losses whose
gradients are written out directly.  Row i of X is worker i's model.
"""
from __future__ import annotations

import numpy as np


def grad_lstsq(X, A, b) -> np.ndarray:
    """f_i(x) = 1/2 ||A_i x - b_i||^2  ->  grad = A_i^T (A_i x - b_i).
    X (n,d), A (n,m,d), b (n,m)."""
    X = np.asarray(X, np.float64)
    A = np.asarray(A, np.float64)
    b = np.asarray(b, np.float64)
    G = np.empty_like(X)
    for i in range(X.shape[0]):
        r = A[i] @ X[i] - b[i]
        G[i] = A[i].T @ r
    return G


def grad_quadratic_diag(X, h, b, noise=None, sigma: float = 0.0) -> np.ndarray:
    """f_i(x) = 1/2 sum_c h_c (x_c - b_ic)^2  ->  grad = h * (x - b_i),
    plus sigma * noise (an unbiased, bounded-variance oracle as the "oracle
    class" assumption asks).  h is (d,) shared or (n,d) per worker."""
    X = np.asarray(X, np.float64)
    G = np.asarray(h, np.float64) * (X - np.asarray(b, np.float64))
    if noise is not None and sigma != 0.0:
        G = G + sigma * np.asarray(noise, np.float64)
    return G


def _log_softmax(logits: np.ndarray) -> np.ndarray:
    z = logits - logits.max(axis=1, keepdims=True)
    return z - np.log(np.exp(z).sum(axis=1, keepdims=True))


def softmax_loss(x_row, feats, labels, F: int, C: int) -> float:
    """Mean cross-entropy of multinomial logistic regression for one worker.
    x_row holds C*F weights (class-major) followed by C biases."""
    x_row = np.asarray(x_row, np.float64)
    Wt = x_row[:C * F].reshape(C, F)
    bias = x_row[C * F:C * F + C]
    logits = np.asarray(feats, np.float64) @ Wt.T + bias
    lp = _log_softmax(logits)
    return float(-lp[np.arange(len(labels)), labels].mean())


def grad_softmax(X, feats, labels, batch_idx, F: int, C: int):
    """Mini-batch gradient of the mean cross-entropy, every worker on its own
    batch: dW_c = mean_s (p_sc - [y_s = c]) x_s,  db_c = mean_s (p_sc - [y_s = c]).
    X (n, C*F+C), feats (n,S,F), labels (n,S), batch_idx (n,B).
    Returns (G (n, C*F+C), loss (n,))."""
    X = np.asarray(X, np.float64)
    n = X.shape[0]
    G = np.zeros_like(X)
    loss = np.zeros(n)
    for i in range(n):
        idx = np.asarray(batch_idx[i], np.int64)
        xs = np.asarray(feats[i][idx], np.float64)
        ys = np.asarray(labels[i][idx], np.int64)
        B = len(idx)
        Wt = X[i, :C * F].reshape(C, F)
        bias = X[i, C * F:C * F + C]
        lp = _log_softmax(xs @ Wt.T + bias)
        delta = np.exp(lp)
        delta[np.arange(B), ys] -= 1.0
        G[i, :C * F] = (delta.T @ xs / B).reshape(-1)
        G[i, C * F:C * F + C] = delta.sum(axis=0) / B
        loss[i] = -lp[np.arange(B), ys].mean()
    return G, loss


def round_bf16(x) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even) and return
    them widened to float32: the storage format of the reduced-precision state."""
    a = np.ascontiguousarray(x, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    bias = np.uint64(0x7FFF) + ((bits >> np.uint64(16)) & np.uint64(1))
    rounded = ((bits + bias) >> np.uint64(16)) << np.uint64(16)
    out = (rounded & np.uint64(0xFFFFFFFF)).astype(np.uint32).view(np.float32)
    nan = np.isnan(a)
    if nan.any():
        out = out.copy()
        out[nan] = np.nan
    return out.reshape(np.shape(x))
