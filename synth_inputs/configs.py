"""The five synthetic configurations of the benchmark contract.

They stand in for the paper's workloads (Fig. 1's random 2048x2048 matrix, the
AlexNet fully-connected layers of Table 2, an LSTM gate matrix), whose trained
weights are not available: shapes, pruning rates and bit-widths follow those
workloads, the values are seeded Gaussian draws.
"""
from dataclasses import dataclass, field
from typing import Tuple

SEED_BASE = 190510138 * 10


@dataclass(frozen=True)
class WorkloadConfig:
    cfg_id: int
    name: str
    m: int                  # rows of W (outputs)
    n: int                  # columns of W (inputs)
    sigma: float            # std of the Gaussian weight draw
    S: float                # pruning rate
    q: int                  # number of binary-coded bit-planes
    n_in: int               # encrypted bits per slice
    n_out: int = 64         # decoded bits per slice
    x_dtype: str = "bf16"   # "bf16" or "f32"
    batches: Tuple[int, ...] = field(default=(1,))

    @property
    def seed_W(self) -> int:
        return SEED_BASE + self.cfg_id

    @property
    def seed_M(self) -> int:
        return SEED_BASE + self.cfg_id + 100

    @property
    def seed_X(self) -> int:
        return SEED_BASE + self.cfg_id + 200


CONFIGS = {
    "tiny": WorkloadConfig(1, "tiny", 256, 256, 1.0, 0.90, 1, 16, x_dtype="f32", batches=(8,)),
    "fig1": WorkloadConfig(2, "fig1", 2048, 2048, 1.0, 0.91, 1, 16, batches=(64,)),
    "fc6": WorkloadConfig(3, "fc6", 4096, 9216, 0.01, 0.91, 2, 16, batches=(1, 64)),
    "lstm": WorkloadConfig(4, "lstm", 6000, 3000, 0.05, 0.80, 3, 24, batches=(1, 32)),
    "large_q1": WorkloadConfig(5, "large_q1", 16384, 4096, 1.0, 0.95, 1, 8, batches=(1, 8, 64, 256)),
    "large_q2": WorkloadConfig(5, "large_q2", 16384, 4096, 1.0, 0.95, 2, 8, batches=(1, 8, 64, 256)),
}


def get_config(name: str) -> WorkloadConfig:
    if name not in CONFIGS:
        raise KeyError(f"unknown workload {name!r}; choose from {sorted(CONFIGS)}")
    return CONFIGS[name]
