"""Shared helpers for the parity tests."""
import os

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


# Every comparison made through rel_err is also measured under tighter floors, so that the margin of the gate is
# on record: (test id, asserted floor) -> worst figures seen in that test's comparisons under that floor.  tests/conftest.py prints the table at the end of a run.
MARGINS: dict = {}


def _record(err: np.ndarray, ref_abs: np.ndarray, S: float, floor: float, gate: float):
    test = os.environ.get("PYTEST_CURRENT_TEST", "?").split(" ")[0]
    rinf = float(ref_abs.max())
    fig = {
        "gate": gate,                                                               # what the test asserts on
        "floor_S/16": float((err / np.maximum(ref_abs, S / 16.0)).max()),
        "floor_S/64": float((err / np.maximum(ref_abs, S / 64.0)).max()),
        "floor_1e-3_ref": float((err / np.maximum(ref_abs, 1e-3 * rinf)).max()) if rinf > 0 else 0.0,
        "normwise_S": float(err.max() / S),
        "normwise_ref": float(err.max() / rinf) if rinf > 0 else 0.0,
    }
    slot = MARGINS.setdefault((test, floor), {"floor": floor, "count": 0})
    slot["count"] += 1
    for k, v in fig.items():
        slot[k] = max(slot.get(k, 0.0), v)


def rel_err(got, ref, scale: float = 0.0, floor: float = FLOOR) -> float:
    """max_ij |got - ref| / max(|ref_ij|, floor * S),  S = max(||ref||_inf, scale).
    `scale` is the largest magnitude among the inputs of the operation."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    S = max(float(np.abs(ref).max()), float(scale))
    if S == 0.0:
        return float(np.abs(got).max())
    err, ref_abs = np.abs(got - ref), np.abs(ref)
    gate = float((err / np.maximum(ref_abs, floor * S)).max())
    _record(err, ref_abs, S, floor, gate)
    return gate


def amax(*arrays) -> float:
    return max(float(np.abs(np.asarray(a, np.float64)).max()) for a in arrays)


def dense_from_csr(n, rowptr, colidx, vals):
    """W[j, i] from CSR rows that list (j, W_ji) for worker i."""
    W = np.zeros((n, n))
    for i in range(n):
        for k in range(rowptr[i], rowptr[i + 1]):
            W[colidx[k], i] = vals[k]
    return W
