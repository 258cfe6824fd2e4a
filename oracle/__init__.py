"""TEST INFRASTRUCTURE ONLY — plain, slow, fp64 CPU oracle of the DeTAG hot path.

Written from the paper (Algorithms 2 and 3, the gossip equation of the
"Protocol Layer" subsection, and the matrix form used in the proof of
Theorem 3).  Nothing here is imported, linked or executed by the product
path; only the tests, the smoke check and the benchmark's CPU-baseline leg use
it.  It shares no code with the HIP library: only seeded input arrays are
common to both.

Pinned by tests/test_oracle_*.py to closed forms, invariants and brute force.
Not pinned (no data in the paper to pin to): the training-loss curves of the
"Experiments" section — parity unpinned for those; they are not reproduced.
"""
from .topology import (mixing_matrix, slack, spectrum, eta_from_lambda,  # noqa: F401
                       neighbour_lists, check_gossip_matrix, phase_length)
from .gossip import (accelerated_gossip, tracking_update, detag_step,  # noqa: F401
                     worker_mean, consensus_error, dpsgd_step)
from .objectives import (grad_lstsq, grad_quadratic_diag, grad_softmax,  # noqa: F401
                         softmax_loss, round_bf16)
from .noise import philox4x32_10, normal_noise  # noqa: F401
