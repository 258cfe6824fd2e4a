"""Build libdetag.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2006_08085_amd.build [--sanitize-host]

Objects go to _build/ at the repository root; the shared library lands next to
this file so that it travels with the source tree.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdetag.so")

SOURCES = ["topology.cpp", "consensus.cpp", "detag_api.hip", "k_stream.hip", "k_fused.hip", "k_fused_quad.hip", "k_fused_generic.hip", "k_fused_generic_quad.hip",
           "k_diag.hip", "k_grad.hip", "k_softmax.hip", "k_consensus.hip", "k_dense.hip"]

FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fno-gpu-rdc",
         # packed fp32 VALU forms are kept off for every kernel in this library
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # the register-resident kernels rely on full unrolling of their row loops (static register indices)
         "-mllvm", "-pragma-unroll-threshold=1000000",
         "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
         "-I", os.path.join(ROOT, "include")]


def _hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


# Host-side AddressSanitizer + UndefinedBehaviorSanitizer (the device code is compiled as usual): for running the
# host logic - graph and matrix ingestion, the eigen-solve, the consensus factors, the table builders, argument
# checks - under the sanitizers on a machine without a GPU.
SAN_FLAGS = ["-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
SAN_LIB = os.path.join(ROOT, "_build", "san", "libdetag_san.so")


def sanitizer_runtime() -> str:
    """The shared AddressSanitizer runtime of the compiler hipcc drives; a process that loads SAN_LIB into an
    uninstrumented executable (python) must have it in LD_PRELOAD."""
    import glob
    hits = sorted(glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so"))
    if not hits:
        raise RuntimeError("libclang_rt.asan-x86_64.so not found under /opt/rocm/lib/llvm")
    return hits[-1]


def build(verbose: bool = True, jobs: int = 8, sanitize_host: bool = False) -> str:
    """Builds libdetag.so next to this file; with sanitize_host the instrumented SAN_LIB under _build/san instead
    (load it with DETAG_LIB=<path> and LD_PRELOAD=sanitizer_runtime())."""
    hipcc = _hipcc()
    bdir = os.path.join(ROOT, "_build", "san") if sanitize_host else os.path.join(ROOT, "_build")
    os.makedirs(bdir, exist_ok=True)
    srcs = list(SOURCES)
    extra = SAN_FLAGS if sanitize_host else []
    link_extra = ["-fsanitize=address", "-fsanitize=undefined", "-shared-libsan", "-Wno-option-ignored"] if sanitize_host else []

    def compile_one(src: str) -> str:
        obj = os.path.join(bdir, src + ".o")
        cmd = [hipcc, *FLAGS, *extra, "-I", CSRC, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        out = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                        if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(compile_one, srcs))
    lib_out = SAN_LIB if sanitize_host else LIB
    tmp = lib_out + ".tmp"
    r = subprocess.run([hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-fno-gpu-rdc", *link_extra, "-o", tmp, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout + r.stderr)
    os.replace(tmp, lib_out)
    if verbose:
        print(f"built {lib_out}")
    return lib_out


if __name__ == "__main__":
    build(sanitize_host="--sanitize-host" in sys.argv[1:])
