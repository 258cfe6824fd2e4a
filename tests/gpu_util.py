"""Helpers shared by the GPU parity tests: host <-> device matrices with
sentinel-filled padding, and matching (library context, dense oracle W) pairs."""
import os

import numpy as np
import pytest
import torch

import paper_2006_08085_amd as D
from oracle import topology as OT
from workloads import generate as gen

DEV = "cuda:0"
SENTINEL = 12345.0


@pytest.fixture(scope="module", autouse=True)
def _built():
    if not os.path.exists(D.LIB_PATH):
        from paper_2006_08085_amd.build import build
        build(verbose=False)
    assert torch.cuda.is_available(), "these tests need the GPU"


def to_dev(a, ld, dtype=torch.float32):
    """Host (n,d) array -> device n x ld matrix, padding filled with a sentinel."""
    n, d = a.shape
    t = torch.full((n, ld), SENTINEL, dtype=torch.float32)
    t[:, :d] = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(dtype).to(DEV)


def to_host(t, d):
    torch.cuda.synchronize()
    return t.float().cpu().numpy()[:, :d].astype(np.float64)


def padding_ok(t, d):
    pad = t.float().cpu().numpy()[:, d:]
    return pad.size == 0 or np.all(pad == np.float32(torch.tensor(SENTINEL).to(t.dtype).float().item()))


def make_ctx(kind, n, d, ld, dtype=D.DETAG_F32):
    if kind == "ring":
        topo, W = D.Topology.ring(), OT.mixing_matrix(n, gen.edges_ring(n))
    elif kind == "torus88":
        topo, W = D.Topology.torus(8, 8), OT.mixing_matrix(64, gen.edges_torus(8, 8))
    elif kind == "torus44":
        topo, W = D.Topology.torus(4, 4), OT.mixing_matrix(16, gen.edges_torus(4, 4))
    elif kind == "torus48":
        topo, W = D.Topology.torus(4, 8), OT.mixing_matrix(32, gen.edges_torus(4, 8))
    elif kind == "asym":
        W = 0.5 * np.eye(n) + 0.5 * np.roll(np.eye(n), 1, axis=1)
        topo = D.Topology.from_dense(W)
    elif kind == "rr":
        e = gen.edges_random_regular(n, 4, seed=1)
        topo, W = D.Topology.from_edges(e, D.DETAG_W_METROPOLIS), OT.mixing_matrix(n, e, "metropolis")
    elif kind == "ring_slack":
        topo, W = D.Topology.ring(kappa=0.3), OT.slack(OT.mixing_matrix(n, gen.edges_ring(n)), 0.3)
    else:
        raise ValueError(kind)
    return D.detag_create(topo, n, d, ld, dtype), W
