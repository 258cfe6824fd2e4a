"""bf16-MFMA softmax-regression gradient against the fp64 oracle, on the
label-sorted shards that stand in for the paper's unshuffled-data experiment."""
import os

import numpy as np
import pytest
import torch

import paper_2006_08085_amd as D
from oracle import gossip as OG
from oracle import objectives as OO
from oracle import topology as OT
from tests.util import TOL_F32, amax, rel_err
from workloads import CONFIGS, generate as gen

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module", autouse=True)
def _built():
    if not os.path.exists(D.LIB_PATH):
        from paper_2006_08085_amd.build import build
        build(verbose=False)
    assert torch.cuda.is_available()


def _problem(n, S, F, C, seed):
    feats32, labels = gen.softmax_problem(n, S, F, C, seed)
    feats_bf = torch.from_numpy(feats32).to(torch.bfloat16)           # the stored data
    feats_ref = feats_bf.to(torch.float32).numpy().astype(np.float64)   # what the oracle sees
    return feats_bf.to(DEV), feats_ref, labels


@pytest.mark.parametrize("n,S,F,C,B", [(3, 80, 64, 10, 32), (4, 200, 160, 7, 64), (2, 300, 96, 2, 256)])
def test_softmax_gradient_small(n, S, F, C, B):
    d = C * F + C
    ld = D.padded_ld(d) + 3                      # odd pitch
    feats_dev, feats_ref, labels = _problem(n, S, F, C, seed=1)
    idx = gen.batch_indices(n, S, B, seed=1, step=0)
    X = 0.2 * gen.state(n, d, seed=2)
    ctx = D.detag_create(D.Topology.ring(), n, d, ld)
    Xd = torch.zeros(n, ld); Xd[:, :d] = torch.from_numpy(X); Xd = Xd.to(DEV)
    Gd = torch.full((n, ld), 777.0, device=DEV)
    loss = torch.zeros(n, device=DEV)
    ctx.grad_softmax_bf16(Xd, feats_dev, torch.from_numpy(labels).to(DEV), torch.from_numpy(idx).to(DEV), C, Gd, loss)
    torch.cuda.synchronize()
    Gr, lr = OO.grad_softmax(X, feats_ref, labels, idx, F, C)
    got = Gd.cpu().numpy()[:, :d].astype(np.float64)
    # the gradient is a mean of B products delta*x with |delta| <= 1: its own scale, not X's, is the operand scale
    S_ = max(amax(Gr), np.abs(feats_ref).max() / B)
    assert rel_err(got, Gr, S_) < TOL_F32
    assert np.abs(loss.cpu().numpy() - lr).max() < 1e-5 * max(1.0, np.abs(lr).max())
    assert np.all(Gd.cpu().numpy()[:, d:] == 777.0)
    # sum over classes of (p - y) is zero
    assert np.abs(got[:, :C * F].reshape(n, C, F).sum(1)).max() < 1e-6


def test_softmax_limits_are_statuses():
    ctx = D.detag_create(D.Topology.ring(), 2, 11 * 32 + 11, 512)
    X = D.new_matrix(2, 11 * 32 + 11, 512, device=DEV)
    feats = torch.zeros(2, 40, 32, dtype=torch.bfloat16, device=DEV)
    lab = torch.zeros(2, 40, dtype=torch.int32, device=DEV)
    bat = torch.zeros(2, 32, dtype=torch.int32, device=DEV)
    with pytest.raises(D.DetagError) as ei:
        ctx.grad_softmax_bf16(X, feats, lab, bat, 11, X.clone())     # C > 10
    assert ei.value.status == D.DETAG_EUNSUPPORTED
    ctx2 = D.detag_create(D.Topology.ring(), 2, 100, 128)
    with pytest.raises(D.DetagError) as ei:
        ctx2.grad_softmax_bf16(D.new_matrix(2, 100, 128, device=DEV), feats, lab, bat, 10, D.new_matrix(2, 100, 128, device=DEV))
    assert ei.value.status == D.DETAG_EINVAL                          # d != C*F + C


def test_config3_run_matches_oracle():
    """n=32 ring, 3072 features, 10 classes, 1,562 label-sorted samples per worker,
    batch 128, K=8, lr=0.01: gradient + phase for a few steps at full size."""
    cfg = CONFIGS[3]
    n, d, K, alpha = cfg.n, cfg.d, cfg.K, cfg.lr
    F, C, S, B = (cfg.extra[k] for k in ("F", "C", "S", "B"))
    T = 3
    ld = D.padded_ld(d)
    feats_dev, feats_ref, labels = _problem(n, S, F, C, seed=cfg.seed)
    lab_dev = torch.from_numpy(labels).to(DEV)
    ctx = D.detag_create(D.Topology.ring(), n, d, ld)
    W = OT.mixing_matrix(n, gen.edges_ring(n))
    eta = OT.eta_from_lambda(OT.spectrum(W)[2])
    Xd, Yd, Ga, Gb = (D.new_matrix(n, d, ld, device=DEV) for _ in range(4))
    loss = torch.zeros(n, device=DEV)
    X = np.zeros((n, d)); Y = np.zeros((n, d)); Gold = np.zeros((n, d))
    for t in range(T):
        idx = gen.batch_indices(n, S, B, seed=cfg.seed, step=t)
        ctx.grad_softmax_bf16(Xd, feats_dev, lab_dev, torch.from_numpy(idx).to(DEV), C, Ga, loss)
        if t == 0:
            torch.cuda.synchronize()
            assert np.allclose(loss.cpu().numpy(), np.log(C), atol=1e-6)      # zero weights: loss = log C
        ctx.step(Xd, Yd, Ga, Gb, alpha, K)
        Ga, Gb = Gb, Ga
        Gnew, lr = OO.grad_softmax(X, feats_ref, labels, idx, F, C)
        if t == 0:
            torch.cuda.synchronize()
            assert rel_err(Gb.cpu().numpy()[:, :d], Gnew, np.abs(feats_ref).max() / B) < TOL_F32
        X, Y = OG.detag_step(X, Y, Gnew, Gold, W, alpha, K, eta)
        Gold = Gnew
    torch.cuda.synchronize()
    assert np.abs(loss.cpu().numpy() - lr).max() < 1e-5
    S_ = amax(X, Y, Gold)
    assert rel_err(Xd.cpu().numpy()[:, :d], X, S_, floor=1.0) < TOL_F32
    assert rel_err(Yd.cpu().numpy()[:, :d], Y, S_, floor=1.0) < TOL_F32
