"""TEST ORACLE - exact average consensus by factor matrices, and DeFacto.

Lemma 1 of the paper: on a connected graph there are R <= 2D matrices, each
with the graph's sparsity, whose product is the average-consensus matrix
11^T/n.  The construction used here is the spanning-tree one the paper's
supplementary material describes (GATHER-PROPAGATE): every node hands its
accumulated value to its parent, level by level, until the root holds the
sum; then every node, level by level from the root, keeps its share of what
it holds and hands each child the share of that child's subtree.  DeFacto
(Algorithm 1) alternates R iterations of gradient accumulation with R
iterations of communication through these matrices.  fp64, dense, slow.
Test infrastructure only.
"""
from __future__ import annotations

from collections import deque

import numpy as np


def spanning_tree(n: int, edges, root: int):
    """Breadth-first spanning tree: (parent, level) arrays; parent[root] = -1.
    Neighbours are visited in increasing index order."""
    adj = [[] for _ in range(n)]
    for a, b in edges:
        adj[a].append(b)
        adj[b].append(a)
    parent = [-1] * n
    level = [-1] * n
    level[root] = 0
    q = deque([root])
    while q:
        u = q.popleft()
        for v in sorted(set(adj[u])):
            if level[v] < 0:
                level[v], parent[v] = level[u] + 1, u
                q.append(v)
    if min(level) < 0:
        raise ValueError("graph is not connected")
    return parent, level


def gather_propagate_factors(n: int, edges, root: int = 0):
    """The matrices A_0, ..., A_{R-1} (dense n x n), R = 2*depth, acting on the vector of the workers' values
    of one coordinate from the left: x <- A_r x.  In the notation of Algorithm 1, whose update is
    x_i <- sum_j x_j [W_r]_ji, W_r = A_r^T.  A_{R-1} ... A_0 = 11^T/n."""
    parent, level = spanning_tree(n, edges, root)
    depth = max(level)
    size = [1] * n                                   # d_v: number of nodes in the subtree of v
    for lv in range(depth, 0, -1):
        for v in range(n):
            if level[v] == lv:
                size[parent[v]] += size[v]
    factors = []
    for lv in range(depth, 0, -1):                   # gather: level lv gives everything to its parents
        A = np.eye(n)
        for v in range(n):
            if level[v] == lv:
                A[v, v] = 0.0
                A[parent[v], v] = 1.0
        factors.append(A)
    for lv in range(depth):                          # propagate: level lv keeps its share, children get theirs
        A = np.eye(n)
        for v in range(n):
            if level[v] == lv + 1:
                u = parent[v]
                A[v, v] = 0.0
                A[v, u] = size[v] / size[u]
                A[u, u] = 1.0 / size[u]              # (d_u - sum of the children's d) / d_u
        factors.append(A)
    return factors


def average_consensus(X, factors):
    Z = np.asarray(X, np.float64)
    for A in factors:
        Z = A @ Z
    return Z


def defacto(grad, X0, factors, alpha: float, T: int, B: int = 1):
    """Algorithm 1 iteration by iteration.  Iteration t is step r = t mod 2R of round k = t div 2R: for r < R,
    B gradient queries at the round-start model are added to the gradient buffer; for r >= R the model copy is
    multiplied by factor r - R; the last iteration of a round sets x = copy - alpha * g / R, clears the buffer
    and copies x.  grad(t, q, X) -> n x d.  An unfinished round leaves X at the last round end.
    Returns (X, rounds completed)."""
    R = len(factors)
    X = np.array(X0, np.float64)
    Xt = X.copy()
    g = np.zeros_like(X)
    rounds = 0
    for t in range(T):
        r = t % (2 * R)
        if r < R:
            for q in range(B):
                g = g + np.asarray(grad(t, q, X), np.float64)
        else:
            Xt = factors[r - R] @ Xt
        if r == 2 * R - 1:
            X = Xt - alpha * g / R
            g = np.zeros_like(X)
            Xt = X.copy()
            rounds += 1
    return X, rounds
