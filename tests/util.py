"""Shared helpers for the parity tests."""
import numpy as np

# Tolerances of the parity bar: max relative error against the fp64 oracle.
TOL_F32 = 1e-5
TOL_BF16 = 2e-2


# An output entry is a signed sum of fp32 terms as large as the operands, so even
# a correctly rounded fp32 evaluation carries an ABSOLUTE error of a few
# 2^-24 * S per gossip round, S = the largest magnitude among inputs and outputs,
# whatever the entry's own magnitude: entries far below S cannot meet a purely
# relative bound.  The relative error is therefore floored at S/16 — small
# entries must be right to 1e-5/16 of S (about ten fp32 ulps of it), the others
# to 1e-5 of themselves.  Whole runs of T steps, where rounding noise of every
# step feeds the next, are judged normwise (floor = 1): max |error| / S.
FLOOR = 1.0 / 16.0


def rel_err(got, ref, scale: float = 0.0, floor: float = FLOOR) -> float:
    """max_ij |got - ref| / max(|ref_ij|, floor * S),  S = max(||ref||_inf, scale).
    `scale` is the largest magnitude among the inputs of the operation."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    S = max(float(np.abs(ref).max()), float(scale))
    if S == 0.0:
        return float(np.abs(got).max())
    return float((np.abs(got - ref) / np.maximum(np.abs(ref), floor * S)).max())


def amax(*arrays) -> float:
    return max(float(np.abs(np.asarray(a, np.float64)).max()) for a in arrays)


def dense_from_csr(n, rowptr, colidx, vals):
    """W[j, i] from CSR rows that list (j, W_ji) for worker i."""
    W = np.zeros((n, n))
    for i in range(n):
        for k in range(rowptr[i], rowptr[i + 1]):
            W[colidx[k], i] = vals[k]
    return W
