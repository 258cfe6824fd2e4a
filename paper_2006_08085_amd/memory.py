"""Device-memory plumbing for the n x ld state matrices (PyTorch allocates,
the library computes)."""
from __future__ import annotations


def padded_ld(d: int, multiple: int = 64) -> int:
    """Row pitch >= d rounded up so every row starts on a 256-byte (fp32) or
    128-byte (bf16) boundary."""
    return (d + multiple - 1) // multiple * multiple


def new_matrix(n: int, d: int, ld: int | None = None, dtype=None, device="cuda"):
    """Zero-filled n x ld matrix (row i = worker i); ld defaults to padded_ld(d)."""
    import torch
    ld = padded_ld(d) if ld is None else ld
    return torch.zeros((n, ld), dtype=dtype or torch.float32, device=device)
