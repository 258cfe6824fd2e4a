"""Pins for oracle/objectives.py and oracle/noise.py: finite differences of the
written-out losses, textbook identities, torch's own bf16 conversion, and the
published known-answer vectors of Philox-4x32-10."""
import os

import numpy as np
import pytest
import torch

from oracle import noise as N
from oracle import objectives as O
from workloads import generate as gen


def _fd(f, x, eps=1e-6):
    g = np.zeros_like(x)
    for k in range(x.size):
        e = np.zeros_like(x); e[k] = eps
        g[k] = (f(x + e) - f(x - e)) / (2 * eps)
    return g


def test_lstsq_gradient_matches_finite_differences():
    n, m, d = 3, 4, 7
    A, b = gen.lstsq_problem(n, m, d, seed=2, shift=1.0)
    X = gen.state(n, d, seed=1).astype(np.float64)
    Gr = O.grad_lstsq(X, A, b)
    for i in range(n):
        f = lambda x: 0.5 * np.sum((A[i].astype(np.float64) @ x - b[i]) ** 2)
        assert np.allclose(Gr[i], _fd(f, X[i]), atol=1e-6)


def test_quadratic_gradient_and_noise_term():
    n, d = 4, 9
    h, b = gen.quadratic_problem(n, d, seed=3)
    X = gen.state(n, d, seed=1).astype(np.float64)
    Gr = O.grad_quadratic_diag(X, h, b)
    for i in range(n):
        f = lambda x: 0.5 * np.sum(h.astype(np.float64) * (x - b[i]) ** 2)
        assert np.allclose(Gr[i], _fd(f, X[i]), atol=1e-7)
    assert np.allclose(O.grad_quadratic_diag(b, h, b), 0.0)        # minimiser of f_i is b_i
    z = gen.gaussian(n, d, seed=5, step=0)
    assert np.allclose(O.grad_quadratic_diag(X, h, b, z, 0.1) - Gr, 0.1 * z.astype(np.float64), atol=1e-15)
    hw = np.tile(h, (n, 1)) * np.arange(1, n + 1)[:, None]          # per-worker curvature
    assert np.allclose(O.grad_quadratic_diag(X, hw, b)[2], 3 * Gr[2], atol=1e-12)


def test_softmax_gradient_matches_finite_differences_and_sums_to_zero():
    n, S, F, C, B = 2, 12, 5, 4, 6
    feats, labels = gen.softmax_problem(n, S, F, C, seed=1)
    idx = gen.batch_indices(n, S, B, seed=1, step=0)
    X = 0.3 * gen.state(n, C * F + C, seed=4).astype(np.float64)
    Gr, loss = O.grad_softmax(X, feats, labels, idx, F, C)
    for i in range(n):
        f = lambda x: O.softmax_loss(x, feats[i][idx[i]], labels[i][idx[i]], F, C)
        assert loss[i] == pytest.approx(f(X[i]), rel=1e-12)
        assert np.allclose(Gr[i], _fd(f, X[i]), atol=1e-7)
        # sum over classes of (p_c - y_c) is zero: weight block and bias block both sum to 0 over c
        assert np.allclose(Gr[i, :C * F].reshape(C, F).sum(0), 0.0, atol=1e-13)
        assert abs(Gr[i, C * F:].sum()) < 1e-13
    # zero weights: p = 1/C, loss = log C
    _, l0 = O.grad_softmax(np.zeros_like(X), feats, labels, idx, F, C)
    assert np.allclose(l0, np.log(C))


def test_softmax_shards_are_label_sorted():
    feats, labels = gen.softmax_problem(12, 50, 3, 10, seed=0)
    for i in range(12):
        assert set(np.unique(labels[i])) <= {i % 10, (i + 1) % 10}
    idx = gen.batch_indices(12, 50, 16, seed=0, step=3)
    assert all(len(set(r)) == 16 for r in idx) and idx.max() < 50


def test_round_bf16_matches_torch():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-20, 20, 20000),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, np.inf, -np.inf,
                         1e-40, 65280.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8]]).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    got = O.round_bf16(x)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    assert np.isnan(O.round_bf16(np.array([np.nan], np.float32))[0])
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert O.round_bf16(np.float32(1 + 2 ** -8)) == 1.0
    assert O.round_bf16(np.float32(1 + 3 * 2 ** -8)) == np.float32(1 + 2 ** -6)


def test_philox_known_answers(golden_dir):
    rows = [ln.split() for ln in open(os.path.join(golden_dir, "philox4x32_10_kat.txt"))
            if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(t, 16) for t in r]
        out = N.philox4x32_10(v[0:4], v[4:6])
        assert [int(o) for o in out] == v[6:10]


def test_philox_is_vectorised_consistently():
    q = np.arange(1000, dtype=np.uint64)
    a = N.philox4x32_10((q, 0 * q, 0 * q + 3, 0 * q + 7), (11, 0))
    for k in (0, 17, 999):
        b = N.philox4x32_10((k, 0, 3, 7), (11, 0))
        assert [int(x[k]) for x in a] == [int(x) for x in b]


def test_normal_noise_layout_and_box_muller():
    n, d = 3, 64
    z = N.normal_noise(seed=5, step=2, n=n, cols=np.arange(d))
    # any column subset reproduces the same numbers (columns are addressable)
    sub = np.array([63, 5, 4, 17, 0])
    assert np.array_equal(N.normal_noise(5, 2, n, sub), z[:, sub])
    # Box-Muller: z0^2 + z1^2 = -2 ln u with u from the first word of the block
    r = N.philox4x32_10((np.uint64(3), 0, 1, 2), (5, 0))        # block q=3 -> columns 12..15, worker 1
    u0 = ((int(r[0]) >> 9) + 0.5) / 2 ** 23
    assert z[1, 12] ** 2 + z[1, 13] ** 2 == pytest.approx(-2 * np.log(u0), rel=1e-12)
    u3 = ((int(r[3]) >> 9) + 0.5) / 2 ** 23
    assert np.arctan2(z[1, 15], z[1, 14]) % (2 * np.pi) == pytest.approx(2 * np.pi * u3, rel=1e-9)
    # the same for the first pair of the block: radius from word 2, angle (cosine first) from word 1
    u1 = ((int(r[1]) >> 9) + 0.5) / 2 ** 23
    assert np.arctan2(z[1, 13], z[1, 12]) % (2 * np.pi) == pytest.approx(2 * np.pi * u1, rel=1e-9)
    u2 = ((int(r[2]) >> 9) + 0.5) / 2 ** 23
    assert z[1, 14] ** 2 + z[1, 15] ** 2 == pytest.approx(-2 * np.log(u2), rel=1e-12)
    # different step / worker / seed -> different streams
    assert not np.array_equal(z, N.normal_noise(5, 3, n, np.arange(d)))
    assert not np.array_equal(z[0], z[1])
    assert not np.array_equal(z, N.normal_noise(6, 2, n, np.arange(d)))


def test_normal_noise_moments():
    z = N.normal_noise(seed=1, step=0, n=4, cols=np.arange(200_000)).ravel()
    m = len(z)
    assert abs(z.mean()) < 4 / np.sqrt(m)
    assert abs(z.var() - 1) < 4 * np.sqrt(2 / m)
    assert abs((z ** 3).mean()) < 4 * np.sqrt(15 / m)
    assert abs((z ** 4).mean() - 3) < 4 * np.sqrt(96 / m)
    # neighbouring outputs of one block are uncorrelated
    zz = z.reshape(-1, 4)
    for a in range(4):
        for b in range(a + 1, 4):
            assert abs((zz[:, a] * zz[:, b]).mean()) < 4 / np.sqrt(len(zz))
