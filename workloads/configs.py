"""The five synthetic workloads, as plain records.

Shapes follow the paper's experiments where it has them (8 workers on a ring
for the unshuffled-data experiment, 16 workers on a ring for the spectral-gap
experiment, Section "Experiments"); values are synthetic.
"""
from dataclasses import dataclass, field


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    n: int                    # workers
    d: int                    # parameters per worker
    topology: str             # "ring" | "torus" | "random_regular"
    torus_shape: tuple = ()   # (rows, cols) for "torus"
    degree: int = 2           # neighbours per worker (off-self)
    weights: str = "uniform"  # "uniform" (1/(deg+1)) | "metropolis"
    state_dtype: str = "f32"  # storage of X and Y: "f32" | "bf16"
    objective: str = "quadratic_diag"   # "lstsq" | "quadratic_diag" | "softmax"
    K: int = 1                # accelerated-gossip rounds per step
    T: int = 1                # steps
    lr: float = 0.5
    sigma: float = 0.0        # std of additive Gaussian gradient noise
    seed: int = 0
    extra: dict = field(default_factory=dict)


CONFIGS = {
    # config index -> record
    1: WorkloadConfig(
        name="ring8_lstsq", n=8, d=1024, topology="ring", degree=2,
        objective="lstsq", K=4, T=50, lr=0.05, seed=0,
        extra=dict(m=64, offset_shift=3.5)),
    2: WorkloadConfig(
        name="ring16_quadratic", n=16, d=272_474, topology="ring", degree=2,
        objective="quadratic_diag", K=6, T=200, lr=0.5, sigma=0.1, seed=0,
        extra=dict(b_mean="i/n", b_std=1.0, h_lo=1e-3, h_hi=1.0)),
    3: WorkloadConfig(
        name="ring32_softmax", n=32, d=30_730, topology="ring", degree=2,
        objective="softmax", K=8, T=100, lr=0.01, seed=0,
        extra=dict(F=3072, C=10, S=1562, B=128)),
    4: WorkloadConfig(
        name="torus8x8_resnet18", n=64, d=11_173_962, topology="torus",
        torus_shape=(8, 8), degree=4, objective="quadratic_diag",
        K=8, T=20, lr=0.5, sigma=0.1, seed=0,
        extra=dict(b_mean="0", b_std=1.0, h_lo=1e-3, h_hi=1.0)),
    5: WorkloadConfig(
        name="rr256_bf16", n=256, d=1_048_576, topology="random_regular",
        degree=4, weights="metropolis", state_dtype="bf16",
        objective="quadratic_diag", K=16, T=50, lr=0.5, seed=0,
        extra=dict(b_mean="0", b_std=2.0, h_lo=1e-3, h_hi=1.0)),
}
