"""The entry point for callers that cannot allocate: detag_consensus_error_static
must give exactly what detag_consensus_error gives (same kernels, same reduction
order), on calls in a row that share the library-resident partial sums."""
import numpy as np
import pytest
import torch

import paper_2006_08085_amd as D
from tests.gpu_util import DEV, _built, to_dev  # noqa: F401
from oracle import gossip as OG

pytestmark = pytest.mark.gpu


def _case(n, d, dtype, seed):
    rng = np.random.default_rng(seed)
    ld = D.padded_ld(d)
    X = rng.standard_normal((n, d)) * 3.0 + rng.standard_normal(d)[None, :]
    tdt = torch.bfloat16 if dtype == D.DETAG_BF16 else torch.float32
    Xd = to_dev(X, ld, tdt)
    Xh = Xd.float().cpu().numpy()[:, :d].astype(np.float64)   # the values the device holds
    return ld, Xd, Xh


def test_static_partials_match_the_allocating_entry_point_on_calls_in_a_row():
    # the second call is smaller than the first: it must not see the first call's partial sums
    shapes = [(64, 70_001, D.DETAG_F32), (16, 1_031, D.DETAG_F32), (8, 257, D.DETAG_BF16), (64, 70_001, D.DETAG_F32)]
    out_s = torch.full((1,), -1.0, dtype=torch.float64, device=DEV)
    for k, (n, d, dtype) in enumerate(shapes):
        ld, Xd, Xh = _case(n, d, dtype, seed=k)
        ctx = D.detag_create(D.Topology.ring(), n, d, ld, dtype)
        ctx.consensus_error_static(Xd, out_s)
        got = out_s.item()
        want = ctx.consensus_error(Xd).item()
        assert got == want, (n, d, got, want)                          # bit for bit
        assert got == pytest.approx(OG.consensus_error(Xh), rel=1e-10)  # and both agree with the oracle
        ctx.close()


def test_static_partials_reject_what_does_not_fit():
    n, d = 2, 256 * 65536 + 1
    ctx = D.detag_create(D.Topology.ring(), n, d, d)
    X = torch.zeros((n, d), dtype=torch.float32, device=DEV)
    out = torch.zeros(1, dtype=torch.float64, device=DEV)
    with pytest.raises(D.DetagError) as e:
        ctx.consensus_error_static(X, out)
    assert e.value.status == D.DETAG_EUNSUPPORTED
    ctx.consensus_error(X, out)          # the allocating entry point still takes it
    assert out.item() == 0.0
    ctx.close()
