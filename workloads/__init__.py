"""Seeded synthetic inputs shared by the CPU oracle and the HIP path.

This package only draws numbers and lays out index lists.  None of the
method's arithmetic (mixing weights, spectra, gossip, tracking, gradients)
lives here: both sides receive these arrays as plain data.
"""
from .configs import CONFIGS, WorkloadConfig  # noqa: F401
from . import generate  # noqa: F401
