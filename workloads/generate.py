"""Seeded input generators (numbers and index lists only, no method arithmetic).

Every function is a pure function of its arguments and a seed, so the CPU
oracle and the HIP path can be fed bit-identical arrays.  Host arrays come
from numpy's PCG64; arrays that are too large to build on the host are drawn
on the device by torch's seeded generator and sampled back as data.
"""
from __future__ import annotations

import numpy as np


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([int(seed), int(stream)]))


# --------------------------------------------------------------------------
# graphs: undirected simple edge lists, vertices 0..n-1
# --------------------------------------------------------------------------
def edges_ring(n: int) -> np.ndarray:
    """Cycle graph: i -- (i+1) mod n.  n=2 gives the single edge, n=1 none."""
    if n < 2:
        return np.zeros((0, 2), dtype=np.int64)
    e = {(min(i, (i + 1) % n), max(i, (i + 1) % n)) for i in range(n)}
    return np.array(sorted(e), dtype=np.int64)


def edges_torus(rows: int, cols: int) -> np.ndarray:
    """2-D torus: vertex r*cols+c joined to (r±1, c) and (r, c±1), wrapping."""
    e = set()
    for r in range(rows):
        for c in range(cols):
            v = r * cols + c
            for w in (((r + 1) % rows) * cols + c, r * cols + (c + 1) % cols):
                if w != v:
                    e.add((min(v, w), max(v, w)))
    return np.array(sorted(e), dtype=np.int64)


def edges_path(n: int) -> np.ndarray:
    return np.array([(i, i + 1) for i in range(n - 1)], dtype=np.int64).reshape(-1, 2)


def edges_random_regular(n: int, degree: int, seed: int) -> np.ndarray:
    """Simple connected `degree`-regular graph (degree even): the union of
    degree/2 random Hamiltonian cycles, redrawn until no edge repeats."""
    if degree % 2 or degree < 2 or n <= degree:
        raise ValueError("need even degree >= 2 and n > degree")
    rng = _rng(seed, 101)
    while True:
        e = set()
        ok = True
        for _ in range(degree // 2):
            p = rng.permutation(n)
            for a, b in zip(p, np.roll(p, -1)):
                key = (int(min(a, b)), int(max(a, b)))
                if key in e:
                    ok = False
                    break
                e.add(key)
            if not ok:
                break
        if ok:
            return np.array(sorted(e), dtype=np.int64)


# --------------------------------------------------------------------------
# state matrices and objectives (host, float32)
# --------------------------------------------------------------------------
def state(n: int, d: int, seed: int, scale: float = 1.0, stream: int = 1) -> np.ndarray:
    """n x d matrix of N(0, scale^2) entries, float32."""
    return (_rng(seed, stream).standard_normal((n, d)) * scale).astype(np.float32)


def lstsq_problem(n: int, m: int, d: int, seed: int, shift: float):
    """Worker i holds A_i (m x d) ~ N(0, 1/m) and b_i (m) ~ N(i - shift, 1)."""
    rng = _rng(seed, 2)
    A = (rng.standard_normal((n, m, d)) / np.sqrt(m)).astype(np.float32)
    mu = (np.arange(n, dtype=np.float64) - shift)[:, None]
    b = (rng.standard_normal((n, m)) + mu).astype(np.float32)
    return A, b


def quadratic_problem(n: int, d: int, seed: int, b_mean: str = "0",
                      b_std: float = 1.0, h_lo: float = 1e-3, h_hi: float = 1.0):
    """Shared curvature h (d), log-uniform in [h_lo, h_hi]; offsets b (n x d)
    with b[i] ~ N(mean_i, b_std^2), mean_i = i/n for "i/n" and 0 for "0"."""
    rng = _rng(seed, 3)
    h = np.exp(rng.uniform(np.log(h_lo), np.log(h_hi), size=d)).astype(np.float32)
    mean = (np.arange(n) / n if b_mean == "i/n" else np.zeros(n))[:, None]
    b = (rng.standard_normal((n, d)) * b_std + mean).astype(np.float32)
    return h, b


def gaussian(n: int, d: int, seed: int, step: int) -> np.ndarray:
    """Explicit standard-normal noise array for one step (small parity runs)."""
    return _rng(seed, 1000 + step).standard_normal((n, d)).astype(np.float32)


def softmax_problem(n: int, S: int, F: int, C: int, seed: int):
    """Label-sorted shards: worker i holds S samples whose labels are drawn
    only from {i mod C, (i+1) mod C}; features ~ N(class mean, I) with class
    means ~ N(0, I).  Returns features (n,S,F) float32 and labels (n,S) int32."""
    rng = _rng(seed, 4)
    means = rng.standard_normal((C, F))
    labels = np.empty((n, S), dtype=np.int32)
    feats = np.empty((n, S, F), dtype=np.float32)
    for i in range(n):
        pick = rng.integers(0, 2, size=S)
        labels[i] = np.where(pick == 0, i % C, (i + 1) % C)
        feats[i] = (means[labels[i]] + rng.standard_normal((S, F))).astype(np.float32)
    return feats, labels


def batch_indices(n: int, S: int, B: int, seed: int, step: int) -> np.ndarray:
    """Per worker, B distinct sample indices for this step: (n,B) int32."""
    rng = _rng(seed, 5000 + step)
    return np.stack([rng.choice(S, size=B, replace=False) for _ in range(n)]).astype(np.int32)


# --------------------------------------------------------------------------
# device-side draws for the matrices too large for the host
# --------------------------------------------------------------------------
def device_normal(n: int, d: int, ld: int, seed: int, stream: int, device,
                  mean: float = 0.0, std: float = 1.0, dtype=None):
    """n x ld torch tensor on `device`; columns [0,d) are N(mean, std^2) drawn
    by torch's seeded generator, the padding columns [d,ld) are zero."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) * 1_000_003 + int(stream))
    out = torch.zeros((n, ld), dtype=torch.float32, device=device)
    out[:, :d].normal_(mean, std, generator=g)
    if dtype is not None and dtype != torch.float32:
        out = out.to(dtype)
    return out


def device_log_uniform(d: int, ld: int, seed: int, stream: int, device,
                       lo: float = 1e-3, hi: float = 1.0):
    """Length-ld vector, entries [0,d) log-uniform in [lo,hi], padding zero."""
    import math
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) * 1_000_003 + int(stream))
    u = torch.zeros(ld, dtype=torch.float32, device=device)
    u[:d].uniform_(math.log(lo), math.log(hi), generator=g)
    u[:d].exp_()
    return u
