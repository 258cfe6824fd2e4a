"""ctypes binding of libdetag.so: argument marshalling only.

Every function mirrors one entry point of include/detag.h (same name, same
argument order) and takes torch tensors where the C call takes device
pointers.  PyTorch is used for device memory and the current HIP stream and
for nothing else: every step of the method runs in the library's kernels.
There is no fallback: if the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("DETAG_LIB") or os.path.join(_HERE, "libdetag.so")

# enums of detag.h
DETAG_OK, DETAG_EINVAL, DETAG_ENOT_DOUBLY_STOCHASTIC, DETAG_EDISCONNECTED, DETAG_EUNSUPPORTED, DETAG_ENOMEM, DETAG_EHIP = range(7)
DETAG_F32, DETAG_BF16 = 0, 1
DETAG_TOPO_RING, DETAG_TOPO_TORUS2D, DETAG_TOPO_RANDOM_REGULAR, DETAG_TOPO_EDGES, DETAG_TOPO_CSR = range(5)
DETAG_W_UNIFORM, DETAG_W_METROPOLIS = 0, 1
DETAG_VARIANT_ATC, DETAG_VARIANT_ALG2 = 0, 1
DETAG_PATH_AUTO, DETAG_PATH_PER_ROUND, DETAG_PATH_FUSED, DETAG_PATH_DENSE = 0, 1, 2, 3
DETAG_KERNEL_PER_ROUND, DETAG_KERNEL_REGISTER_TILE, DETAG_KERNEL_LDS_TILE, DETAG_KERNEL_DENSE = 0, 1, 2, 3

_STATUS_NAMES = ["DETAG_OK", "DETAG_EINVAL", "DETAG_ENOT_DOUBLY_STOCHASTIC", "DETAG_EDISCONNECTED",
                 "DETAG_EUNSUPPORTED", "DETAG_ENOMEM", "DETAG_EHIP"]

EXPORTS = ["detag_create", "detag_destroy", "detag_get_spectrum", "detag_get_csr", "detag_set_path",
           "detag_get_phase_length", "detag_get_gossip_polynomial", "detag_has_fused", "detag_get_kernel", "detag_reserve_gossip", "detag_reserve_gradient", "detag_gossip_accel", "detag_track", "detag_step", "detag_dpsgd_step", "detag_gossip_round", "detag_accumulate", "detag_phase_end",
           "detag_factors_create", "detag_factors_destroy", "detag_factors_count", "detag_factors_get_csr",
           "detag_factors_get_program",
           "detag_factor_apply", "detag_average_consensus", "detag_defacto_update",
           "detag_mean", "detag_consensus_error", "detag_consensus_error_static", "detag_grad_quadratic_diag", "detag_step_quadratic", "detag_grad_lstsq",
           "detag_grad_softmax_bf16", "detag_last_error", "detag_version"]


class DetagError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS_NAMES[status] if 0 <= status < len(_STATUS_NAMES) else status}: {message}")
        self.status = status
        self.message = message


class _Topology(C.Structure):
    _fields_ = [("kind", C.c_int32), ("weights", C.c_int32), ("rows", C.c_int32), ("cols", C.c_int32),
                ("degree", C.c_int32), ("seed", C.c_uint64), ("kappa", C.c_double), ("n_edges", C.c_int64),
                ("edges", C.POINTER(C.c_int32)), ("rowptr", C.POINTER(C.c_int32)),
                ("colidx", C.POINTER(C.c_int32)), ("vals", C.POINTER(C.c_double))]


_lib = None


def lib() -> C.CDLL:
    """Load libdetag.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2006_08085_amd.build`")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, f64, f32, u64, u32 = C.c_void_p, C.c_int32, C.c_int64, C.c_double, C.c_float, C.c_uint64, C.c_uint32
    L.detag_create.argtypes = [C.POINTER(_Topology), i32, i64, i64, C.c_int, C.POINTER(vp)]
    L.detag_create.restype = C.c_int
    L.detag_destroy.argtypes = [vp]
    L.detag_destroy.restype = None
    L.detag_get_spectrum.argtypes = [vp] + [C.POINTER(f64)] * 4
    L.detag_get_spectrum.restype = C.c_int
    L.detag_get_phase_length.argtypes = [vp, f64, C.POINTER(i32)]
    L.detag_get_phase_length.restype = C.c_int
    L.detag_get_gossip_polynomial.argtypes = [vp, i32, f64, C.POINTER(f64)]
    L.detag_get_gossip_polynomial.restype = C.c_int
    L.detag_get_csr.argtypes = [vp, C.POINTER(i32), C.POINTER(i64), C.POINTER(C.POINTER(i32)),
                                C.POINTER(C.POINTER(i32)), C.POINTER(C.POINTER(f64))]
    L.detag_get_csr.restype = C.c_int
    L.detag_set_path.argtypes = [vp, C.c_int]
    L.detag_set_path.restype = C.c_int
    L.detag_get_kernel.argtypes = [vp, C.POINTER(i32)]
    L.detag_get_kernel.restype = C.c_int
    L.detag_has_fused.argtypes = [vp]
    L.detag_has_fused.restype = i32
    L.detag_reserve_gossip.argtypes = [vp, C.c_int, i32, f64]
    L.detag_reserve_gossip.restype = C.c_int
    L.detag_reserve_gradient.argtypes = [vp, i32, i32, i32, i32]
    L.detag_reserve_gradient.restype = C.c_int
    L.detag_gossip_accel.argtypes = [vp, vp, i32, f64, vp]
    L.detag_gossip_accel.restype = C.c_int
    L.detag_track.argtypes = [vp, vp, vp, vp, vp]
    L.detag_track.restype = C.c_int
    L.detag_step.argtypes = [vp, vp, vp, vp, vp, f64, i32, f64, C.c_int, vp]
    L.detag_step.restype = C.c_int
    L.detag_dpsgd_step.argtypes = [vp, vp, vp, f64, vp]
    L.detag_dpsgd_step.restype = C.c_int
    L.detag_gossip_round.argtypes = [vp, vp, vp, vp, f64, vp]
    L.detag_gossip_round.restype = C.c_int
    L.detag_accumulate.argtypes = [vp, vp, vp, f64, vp]
    L.detag_accumulate.restype = C.c_int
    L.detag_phase_end.argtypes = [vp, vp, vp, vp, vp, vp, f64, vp]
    L.detag_phase_end.restype = C.c_int
    L.detag_factors_create.argtypes = [vp, i32, C.POINTER(vp)]
    L.detag_factors_create.restype = C.c_int
    L.detag_factors_destroy.argtypes = [vp]
    L.detag_factors_destroy.restype = None
    L.detag_factors_count.argtypes = [vp, C.POINTER(i32)]
    L.detag_factors_count.restype = C.c_int
    L.detag_factors_get_csr.argtypes = [vp, i32, C.POINTER(i64), C.POINTER(C.POINTER(i32)), C.POINTER(C.POINTER(i32)),
                                        C.POINTER(C.POINTER(f64))]
    L.detag_factors_get_csr.restype = C.c_int
    L.detag_factors_get_program.argtypes = [vp, C.POINTER(i64), C.POINTER(C.POINTER(C.c_uint32))]
    L.detag_factors_get_program.restype = C.c_int
    L.detag_factor_apply.argtypes = [vp, vp, i32, vp, vp, vp]
    L.detag_factor_apply.restype = C.c_int
    L.detag_average_consensus.argtypes = [vp, vp, vp, vp]
    L.detag_average_consensus.restype = C.c_int
    L.detag_defacto_update.argtypes = [vp, vp, vp, vp, f64, vp]
    L.detag_defacto_update.restype = C.c_int
    L.detag_mean.argtypes = [vp, vp, vp, vp]
    L.detag_mean.restype = C.c_int
    L.detag_consensus_error.argtypes = [vp, vp, vp, vp]
    L.detag_consensus_error.restype = C.c_int
    L.detag_consensus_error_static.argtypes = [vp, vp, vp, vp]
    L.detag_consensus_error_static.restype = C.c_int
    L.detag_grad_quadratic_diag.argtypes = [vp, vp, vp, i32, vp, vp, f32, u64, u32, vp, vp]
    L.detag_grad_quadratic_diag.restype = C.c_int
    L.detag_step_quadratic.argtypes = [vp, vp, vp, vp, vp, i32, vp, f32, u64, u32, f64, i32, f64, i32, vp]
    L.detag_step_quadratic.restype = C.c_int
    L.detag_grad_lstsq.argtypes = [vp, vp, vp, vp, i32, vp, vp]
    L.detag_grad_lstsq.restype = C.c_int
    L.detag_grad_softmax_bf16.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp, vp]
    L.detag_grad_softmax_bf16.restype = C.c_int
    L.detag_last_error.argtypes = [vp]
    L.detag_last_error.restype = C.c_char_p
    L.detag_version.argtypes = []
    L.detag_version.restype = C.c_char_p
    _lib = L
    return L


@dataclass
class Topology:
    """Host description of the gossip graph / matrix (detag_topology)."""
    kind: int
    weights: int = DETAG_W_UNIFORM
    rows: int = 0
    cols: int = 0
    degree: int = 0
    seed: int = 0
    kappa: float = 1.0
    edges: Optional[np.ndarray] = None
    rowptr: Optional[np.ndarray] = None
    colidx: Optional[np.ndarray] = None
    vals: Optional[np.ndarray] = None
    _keep: list = field(default_factory=list, repr=False)

    @staticmethod
    def ring(kappa: float = 1.0) -> "Topology":
        return Topology(DETAG_TOPO_RING, kappa=kappa)

    @staticmethod
    def torus(rows: int, cols: int, kappa: float = 1.0) -> "Topology":
        return Topology(DETAG_TOPO_TORUS2D, rows=rows, cols=cols, kappa=kappa)

    @staticmethod
    def random_regular(degree: int, seed: int, weights: int = DETAG_W_METROPOLIS) -> "Topology":
        return Topology(DETAG_TOPO_RANDOM_REGULAR, weights=weights, degree=degree, seed=seed)

    @staticmethod
    def from_edges(edges, weights: int = DETAG_W_METROPOLIS, kappa: float = 1.0) -> "Topology":
        return Topology(DETAG_TOPO_EDGES, weights=weights, kappa=kappa,
                        edges=np.ascontiguousarray(edges, dtype=np.int32).reshape(-1, 2))

    @staticmethod
    def from_dense(W, kappa: float = 1.0) -> "Topology":
        """Complete matrix W (n x n, W[j, i] is the weight worker i gives worker j's value)."""
        W = np.asarray(W, dtype=np.float64)
        n = W.shape[0]
        rowptr, colidx, vals = [0], [], []
        for i in range(n):
            for j in range(n):
                if W[j, i] != 0.0 or j == i:
                    colidx.append(j)
                    vals.append(W[j, i])
            rowptr.append(len(colidx))
        return Topology(DETAG_TOPO_CSR, kappa=kappa, rowptr=np.array(rowptr, np.int32),
                        colidx=np.array(colidx, np.int32), vals=np.array(vals, np.float64))

    def _as_struct(self) -> _Topology:
        t = _Topology()
        t.kind, t.weights, t.rows, t.cols, t.degree = self.kind, self.weights, self.rows, self.cols, self.degree
        t.seed, t.kappa = self.seed, self.kappa
        self._keep.clear()

        def ptr(a, ctype):
            if a is None:
                return None
            self._keep.append(a)
            return a.ctypes.data_as(C.POINTER(ctype))

        t.n_edges = 0 if self.edges is None else len(self.edges)
        t.edges = ptr(self.edges, C.c_int32)
        t.rowptr = ptr(self.rowptr, C.c_int32)
        t.colidx = ptr(self.colidx, C.c_int32)
        t.vals = ptr(self.vals, C.c_double)
        return t


class Factors:
    """Owns one detag_factors: the matrices of the exact average consensus on a context's graph."""

    def __init__(self, ctx: "Context", root: int = 0):
        h = C.c_void_p()
        ctx._check(lib().detag_factors_create(ctx._h, root, C.byref(h)))
        self._h, self.ctx = h, ctx
        R = C.c_int32()
        ctx._check(lib().detag_factors_count(self._h, C.byref(R)))
        self.R = R.value

    def close(self):
        if self._h:
            lib().detag_factors_destroy(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def dense(self, r: int) -> np.ndarray:
        """Factor r as a dense n x n array A (z <- A z), rebuilt from detag_factors_get_csr."""
        n = self.ctx.n
        nnz = C.c_int64()
        rp, ci, va = C.POINTER(C.c_int32)(), C.POINTER(C.c_int32)(), C.POINTER(C.c_double)()
        self.ctx._check(lib().detag_factors_get_csr(self._h, r, C.byref(nnz), C.byref(rp), C.byref(ci), C.byref(va)))
        A = np.zeros((n, n))
        for i in range(n):
            for k in range(rp[i], rp[i + 1]):
                A[i, ci[k]] = va[k]
        return A

    def program(self) -> np.ndarray:
        """The on-chip form of the sequence as a (batches, 4, 8) uint32 array (detag_factors_get_program); no
        batches if the sequence is not run that way."""
        nb, words = C.c_int64(), C.POINTER(C.c_uint32)()
        self.ctx._check(lib().detag_factors_get_program(self._h, C.byref(nb), C.byref(words)))
        if nb.value == 0:
            return np.zeros((0, 4, 8), np.uint32)
        return np.ctypeslib.as_array(words, shape=(nb.value, 4, 8)).copy()

    def apply(self, r: int, Z_in, Z_out):
        c = self.ctx
        c._check(lib().detag_factor_apply(c._h, self._h, r, c._state(Z_in, "Z_in"), c._state(Z_out, "Z_out"),
                                          c._stream()))


    def average(self, Z):
        """Z <- A_{R-1} ... A_0 Z in place: every row becomes the column mean."""
        c = self.ctx
        c._check(lib().detag_average_consensus(c._h, self._h, c._state(Z, "Z"), c._stream()))


class Context:
    """Owns one detag_ctx.  Methods map one-to-one onto the C entry points."""

    def __init__(self, handle: int, n: int, d: int, ld: int, dtype: int):
        self._h = C.c_void_p(handle)
        self.n, self.d, self.ld, self.dtype = n, d, ld, dtype

    def close(self):
        if self._h:
            lib().detag_destroy(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- helpers -------------------------------------------------------------
    def _check(self, status: int):
        if status != DETAG_OK:
            raise DetagError(status, lib().detag_last_error(self._h).decode())

    def _state(self, t, name="state"):
        import torch
        want = torch.bfloat16 if self.dtype == DETAG_BF16 else torch.float32
        return self._mat(t, want, name)

    def _mat(self, t, want_dtype, name):
        if not t.is_cuda:
            raise ValueError(f"{name} must be a GPU tensor")
        if t.dtype != want_dtype:
            raise ValueError(f"{name} must be {want_dtype}, got {t.dtype}")
        if t.dim() != 2 or t.shape[0] != self.n or t.shape[1] < self.d or t.stride(1) != 1 or t.stride(0) != self.ld:
            raise ValueError(f"{name} must be an n x ld row-major matrix with pitch {self.ld} (n={self.n}, d={self.d}); "
                             f"got shape {tuple(t.shape)} strides {t.stride()}")
        return C.c_void_p(t.data_ptr())

    @staticmethod
    def _stream():
        import torch
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)

    # -- queries -------------------------------------------------------------
    def spectrum(self):
        v = [C.c_double() for _ in range(4)]
        self._check(lib().detag_get_spectrum(self._h, *[C.byref(x) for x in v]))
        return dict(lambda2=v[0].value, lambdan=v[1].value, lam=v[2].value, eta=v[3].value)

    def phase_length(self, outer_ratio: float = 0.0) -> int:
        R = C.c_int32()
        self._check(lib().detag_get_phase_length(self._h, outer_ratio, C.byref(R)))
        return R.value

    def gossip_polynomial(self, K: int, eta: float = -1.0) -> np.ndarray:
        """P with AG_K(Z) = P Z (detag_get_gossip_polynomial), n x n fp64."""
        P = np.empty((self.n, self.n), np.float64)
        self._check(lib().detag_get_gossip_polynomial(self._h, K, eta, P.ctypes.data_as(C.POINTER(C.c_double))))
        return P

    def csr(self):
        n, nnz = C.c_int32(), C.c_int64()
        rp, ci, va = C.POINTER(C.c_int32)(), C.POINTER(C.c_int32)(), C.POINTER(C.c_double)()
        self._check(lib().detag_get_csr(self._h, C.byref(n), C.byref(nnz), C.byref(rp), C.byref(ci), C.byref(va)))
        rowptr = np.ctypeslib.as_array(rp, shape=(n.value + 1,)).copy()
        colidx = np.ctypeslib.as_array(ci, shape=(nnz.value,)).copy()
        vals = np.ctypeslib.as_array(va, shape=(nnz.value,)).copy()
        return rowptr, colidx, vals

    def dense_W(self) -> np.ndarray:
        """W as a dense n x n array rebuilt from detag_get_csr (data for the oracle)."""
        rowptr, colidx, vals = self.csr()
        W = np.zeros((self.n, self.n))
        for i in range(self.n):
            for k in range(rowptr[i], rowptr[i + 1]):
                W[colidx[k], i] = vals[k]
        return W

    def set_path(self, path: int):
        self._check(lib().detag_set_path(self._h, path))

    def kernel(self) -> int:
        """detag_get_kernel: the kernel family (DETAG_KERNEL_*) the gossip and phase calls use with the current path."""
        k = C.c_int32()
        self._check(lib().detag_get_kernel(self._h, C.byref(k)))
        return k.value

    def has_fused(self) -> bool:
        return bool(lib().detag_has_fused(self._h))

    def reserve_gossip(self, path: int, K: int = 1, eta: float = -1.0):
        self._check(lib().detag_reserve_gossip(self._h, path, K, eta))

    def reserve_gradient(self, m: int = 0, F: int = 0, C_classes: int = 0, B: int = 0):
        self._check(lib().detag_reserve_gradient(self._h, m, F, C_classes, B))

    # -- hot path ------------------------------------------------------------
    def gossip_accel(self, Z, K: int, eta: float = -1.0):
        self._check(lib().detag_gossip_accel(self._h, self._state(Z, "Z"), K, eta, self._stream()))

    def track(self, Y, G_new, G_old):
        import torch
        self._check(lib().detag_track(self._h, self._state(Y, "Y"), self._mat(G_new, torch.float32, "G_new"),
                                      self._mat(G_old, torch.float32, "G_old"), self._stream()))

    def step(self, X, Y, G_new, G_old, alpha: float, K: int, eta: float = -1.0, variant: int = DETAG_VARIANT_ATC):
        import torch
        self._check(lib().detag_step(self._h, self._state(X, "X"), self._state(Y, "Y"),
                                     self._mat(G_new, torch.float32, "G_new"), self._mat(G_old, torch.float32, "G_old"),
                                     alpha, K, eta, variant, self._stream()))

    def dpsgd_step(self, X, G, alpha: float):
        import torch
        self._check(lib().detag_dpsgd_step(self._h, self._state(X, "X"), self._mat(G, torch.float32, "G"), alpha,
                                           self._stream()))

    # -- Algorithm 2 iteration by iteration ---------------------------------------
    def gossip_round(self, Z_cur, Z_prev, Z_out, eta: float = -1.0):
        self._check(lib().detag_gossip_round(self._h, self._state(Z_cur, "Z_cur"), self._state(Z_prev, "Z_prev"),
                                             self._state(Z_out, "Z_out"), eta, self._stream()))

    def accumulate(self, G_acc, g, scale: float = 1.0):
        import torch
        self._check(lib().detag_accumulate(self._h, self._mat(G_acc, torch.float32, "G_acc"),
                                           self._mat(g, torch.float32, "g"), scale, self._stream()))

    def phase_end(self, X, X_tilde, Y, G_k, G_km1, alpha: float):
        import torch
        self._check(lib().detag_phase_end(self._h, self._state(X, "X"), self._state(X_tilde, "X_tilde"),
                                          self._state(Y, "Y"), self._mat(G_k, torch.float32, "G_k"),
                                          self._mat(G_km1, torch.float32, "G_km1"), alpha, self._stream()))

    def defacto_update(self, X, X_tilde, G, scale: float):
        import torch
        self._check(lib().detag_defacto_update(self._h, self._state(X, "X"), self._state(X_tilde, "X_tilde"),
                                               self._mat(G, torch.float32, "G"), scale, self._stream()))

    # -- diagnostics -----------------------------------------------------------
    def mean(self, X, out=None):
        import torch
        if out is None:
            out = torch.empty(self.d, dtype=torch.float32, device=X.device)
        if out.dtype != torch.float32 or out.numel() < self.d or not out.is_contiguous():
            raise ValueError("out must be a contiguous float32 vector of length >= d")
        self._check(lib().detag_mean(self._h, self._state(X, "X"), C.c_void_p(out.data_ptr()), self._stream()))
        return out

    def consensus_error(self, X, out=None):
        import torch
        if out is None:
            out = torch.empty(1, dtype=torch.float64, device=X.device)
        self._check(lib().detag_consensus_error(self._h, self._state(X, "X"), C.c_void_p(out.data_ptr()),
                                                self._stream()))
        return out

    def consensus_error_static(self, X, out):
        """detag_consensus_error_static: `out` (one float64 on the GPU) is required, since this call is for
        callers that may not allocate."""
        import torch
        if out.dtype != torch.float64 or not out.is_cuda or out.numel() < 1:
            raise ValueError("out must be a float64 GPU tensor with at least one element")
        self._check(lib().detag_consensus_error_static(self._h, self._state(X, "X"), C.c_void_p(out.data_ptr()),
                                                       self._stream()))
        return out

    # -- gradients ---------------------------------------------------------------
    def grad_quadratic_diag(self, X, h, b, G, noise=None, sigma: float = 0.0, seed: int = 0, step: int = 0):
        import torch
        per_worker = 1 if h.dim() == 2 else 0
        if per_worker:
            hp = self._mat(h, torch.float32, "h")
        else:
            if h.dtype != torch.float32 or not h.is_cuda or h.numel() < self.d or not h.is_contiguous():
                raise ValueError("h must be a contiguous float32 GPU vector of length >= d")
            hp = C.c_void_p(h.data_ptr())
        npz = None if noise is None else self._mat(noise, torch.float32, "noise")
        self._check(lib().detag_grad_quadratic_diag(self._h, self._state(X, "X"), hp, per_worker,
                                                    self._mat(b, torch.float32, "b"), npz, sigma, seed, step,
                                                    self._mat(G, torch.float32, "G"), self._stream()))

    def step_quadratic(self, X, Y, G, h, b, alpha: float, K: int, sigma: float = 0.0, seed: int = 0, step: int = 0,
                       eta: float = -1.0, variant: int = DETAG_VARIANT_ATC):
        """h: a float32 vector of length >= d shared by the workers, or an n x ld matrix with one row per worker."""
        import torch
        per_worker = 1 if h.dim() == 2 else 0
        if per_worker:
            hp = self._mat(h, torch.float32, "h")
        else:
            if h.dtype != torch.float32 or not h.is_cuda or h.dim() != 1 or h.numel() < self.d or not h.is_contiguous():
                raise ValueError("h must be a contiguous float32 GPU vector of length >= d")
            hp = C.c_void_p(h.data_ptr())
        self._check(lib().detag_step_quadratic(self._h, self._state(X, "X"), self._state(Y, "Y"),
                                               self._mat(G, torch.float32, "G"), hp, per_worker,
                                               self._mat(b, torch.float32, "b"), sigma, seed, step, alpha, K, eta,
                                               variant, self._stream()))

    def grad_lstsq(self, X, A, b, G):
        import torch
        if A.dtype != torch.float32 or not A.is_cuda or not A.is_contiguous() or A.dim() != 3 \
                or A.shape[0] != self.n or A.shape[2] != self.d:
            raise ValueError("A must be a contiguous float32 GPU tensor of shape (n, m, d)")
        m = A.shape[1]
        if b.dtype != torch.float32 or not b.is_cuda or not b.is_contiguous() or tuple(b.shape) != (self.n, m):
            raise ValueError("b must be a contiguous float32 GPU tensor of shape (n, m)")
        self._check(lib().detag_grad_lstsq(self._h, self._state(X, "X"), C.c_void_p(A.data_ptr()),
                                           C.c_void_p(b.data_ptr()), m, self._mat(G, torch.float32, "G"),
                                           self._stream()))

    def grad_softmax_bf16(self, X, feats, labels, batch, C_classes: int, G, loss=None):
        import torch
        if feats.dtype != torch.bfloat16 or not feats.is_cuda or not feats.is_contiguous() or feats.dim() != 3 \
                or feats.shape[0] != self.n:
            raise ValueError("feats must be a contiguous bfloat16 GPU tensor of shape (n, S, F)")
        S, F = feats.shape[1], feats.shape[2]
        if labels.dtype != torch.int32 or not labels.is_cuda or not labels.is_contiguous() or tuple(labels.shape) != (self.n, S):
            raise ValueError("labels must be a contiguous int32 GPU tensor of shape (n, S)")
        if batch.dtype != torch.int32 or not batch.is_cuda or not batch.is_contiguous() or batch.dim() != 2 \
                or batch.shape[0] != self.n:
            raise ValueError("batch must be a contiguous int32 GPU tensor of shape (n, B)")
        B = batch.shape[1]
        lp = None
        if loss is not None:
            if loss.dtype != torch.float32 or not loss.is_cuda or loss.numel() < self.n or not loss.is_contiguous():
                raise ValueError("loss must be a contiguous float32 GPU vector of length >= n")
            lp = C.c_void_p(loss.data_ptr())
        self._check(lib().detag_grad_softmax_bf16(self._h, self._state(X, "X"), C.c_void_p(feats.data_ptr()),
                                                  C.c_void_p(labels.data_ptr()), C.c_void_p(batch.data_ptr()),
                                                  S, F, C_classes, B, self._mat(G, torch.float32, "G"), lp,
                                                  self._stream()))


def detag_create(topology: Topology, n: int, d: int, ld: Optional[int] = None, dtype: int = DETAG_F32) -> Context:
    ld = d if ld is None else ld
    h = C.c_void_p()
    st = lib().detag_create(C.byref(topology._as_struct()), n, d, ld, dtype, C.byref(h))
    if st != DETAG_OK:
        raise DetagError(st, lib().detag_last_error(None).decode())
    return Context(h.value, n, d, ld, dtype)


# Module-level aliases with the C names, for callers who prefer the flat API.
def detag_destroy(ctx: Context): ctx.close()
def detag_get_spectrum(ctx: Context): return ctx.spectrum()
def detag_get_csr(ctx: Context): return ctx.csr()
def detag_get_phase_length(ctx: Context, outer_ratio=0.0): return ctx.phase_length(outer_ratio)
def detag_get_gossip_polynomial(ctx: Context, K, eta=-1.0): return ctx.gossip_polynomial(K, eta)
def detag_set_path(ctx: Context, path: int): ctx.set_path(path)
def detag_has_fused(ctx: Context): return ctx.has_fused()
def detag_get_kernel(ctx: Context): return ctx.kernel()
def detag_reserve_gossip(ctx: Context, path, K=1, eta=-1.0): ctx.reserve_gossip(path, K, eta)
def detag_reserve_gradient(ctx: Context, m=0, F=0, C_classes=0, B=0): ctx.reserve_gradient(m, F, C_classes, B)
def detag_gossip_accel(ctx: Context, Z, K, eta=-1.0): ctx.gossip_accel(Z, K, eta)
def detag_track(ctx: Context, Y, G_new, G_old): ctx.track(Y, G_new, G_old)
def detag_step(ctx: Context, X, Y, G_new, G_old, alpha, K, eta=-1.0, variant=DETAG_VARIANT_ATC):
    ctx.step(X, Y, G_new, G_old, alpha, K, eta, variant)
def detag_dpsgd_step(ctx: Context, X, G, alpha): ctx.dpsgd_step(X, G, alpha)
def detag_gossip_round(ctx: Context, Z_cur, Z_prev, Z_out, eta=-1.0): ctx.gossip_round(Z_cur, Z_prev, Z_out, eta)
def detag_accumulate(ctx: Context, G_acc, g, scale=1.0): ctx.accumulate(G_acc, g, scale)
def detag_phase_end(ctx: Context, X, X_tilde, Y, G_k, G_km1, alpha): ctx.phase_end(X, X_tilde, Y, G_k, G_km1, alpha)
def detag_factors_create(ctx: Context, root=0): return Factors(ctx, root)
def detag_factors_destroy(f: Factors): f.close()
def detag_factors_count(f: Factors): return f.R
def detag_factors_get_csr(f: Factors, r): return f.dense(r)
def detag_factors_get_program(f: Factors): return f.program()
def detag_factor_apply(ctx: Context, f: Factors, r, Z_in, Z_out): f.apply(r, Z_in, Z_out)
def detag_average_consensus(ctx: Context, f: Factors, Z): f.average(Z)
def detag_defacto_update(ctx: Context, X, X_tilde, G, scale): ctx.defacto_update(X, X_tilde, G, scale)
def detag_mean(ctx: Context, X, out=None): return ctx.mean(X, out)
def detag_consensus_error(ctx: Context, X, out=None): return ctx.consensus_error(X, out)
def detag_consensus_error_static(ctx: Context, X, out): return ctx.consensus_error_static(X, out)
def detag_grad_quadratic_diag(ctx: Context, X, h, b, G, noise=None, sigma=0.0, seed=0, step=0):
    ctx.grad_quadratic_diag(X, h, b, G, noise, sigma, seed, step)
def detag_step_quadratic(ctx: Context, X, Y, G, h, b, alpha, K, sigma=0.0, seed=0, step=0, eta=-1.0,
                         variant=DETAG_VARIANT_ATC):
    ctx.step_quadratic(X, Y, G, h, b, alpha, K, sigma, seed, step, eta, variant)
def detag_grad_lstsq(ctx: Context, X, A, b, G): ctx.grad_lstsq(X, A, b, G)
def detag_grad_softmax_bf16(ctx: Context, X, feats, labels, batch, C_classes, G, loss=None):
    ctx.grad_softmax_bf16(X, feats, labels, batch, C_classes, G, loss)
def detag_version() -> str: return lib().detag_version().decode()
