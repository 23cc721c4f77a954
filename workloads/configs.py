"""The five workload configurations (shapes, model lists, stopping rules).

Each mirrors a workload class of the paper's experiments section: cubic tensors with a mix
of 1..R_max-component models run for a fixed number of iterations (the speed-up and
efficiency experiments), and a fluorescence-shaped tensor fitted with many models under a
tolerance and an iteration cap (the real-application experiment; its datasets are not
available, so a synthetic tensor of the same shape class stands in).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

FLAG_NONNEG = 1
FLAG_LINESEARCH = 2


@dataclass(frozen=True)
class WorkloadConfig:
    cid: int
    name: str
    dims: Tuple[int, int, int]          # (I1, I2, I3); I1 is the fastest index in memory
    kind: str                           # "uniform" | "eem" | "collinear"
    true_rank: int
    noise: float                        # eta: noise std = eta * rms(T0)
    clip_at_zero: bool
    ranks: Tuple[int, ...]              # rank of every queued model, in enqueue order
    init_seeds: Tuple[int, ...]         # seed of every model's starting point
    tol: float                          # < 0: never converge by tolerance (fixed iterations)
    max_iters: int
    flags: int
    ls_alpha: float
    max_total_rank: int                 # R*
    max_slots: int                      # 0 = unlimited
    collinearity: float = 0.0

    @property
    def n_models(self) -> int:
        return len(self.ranks)

    @property
    def total_rank(self) -> int:
        return int(sum(self.ranks))

    @property
    def tensor_seed(self) -> int:
        return 1000 * self.cid + 1

    @property
    def noise_seed(self) -> int:
        return 1000 * self.cid + 2


def _twice(rmax: int) -> Tuple[int, ...]:
    return tuple(list(range(1, rmax + 1)) * 2)


def _seeds(cid: int, n: int) -> Tuple[int, ...]:
    return tuple(1000 * cid + 100 + m for m in range(n))


def _build() -> List[WorkloadConfig]:
    c1r = _twice(5)
    c2r = _twice(10)
    c3r = tuple(r for r in range(1, 21) for _ in range(3))
    c4r = _twice(20)
    c5r = tuple(r for r in range(1, 21) for _ in range(10))
    return [
        WorkloadConfig(1, "cfg1_32cube", (32, 32, 32), "uniform", 3, 0.01, False, c1r, _seeds(1, len(c1r)),
                       -1.0, 50, 0, 1.0, sum(c1r), 0),
        WorkloadConfig(2, "cfg2_200cube", (200, 200, 200), "uniform", 10, 0.05, False, c2r, _seeds(2, len(c2r)),
                       -1.0, 100, 0, 1.0, sum(c2r), 0),
        WorkloadConfig(3, "cfg3_eem_300x300x40", (300, 300, 40), "eem", 6, 0.02, True, c3r, _seeds(3, len(c3r)),
                       1e-7, 500, FLAG_NONNEG, 1.0, sum(c3r), 0),
        WorkloadConfig(4, "cfg4_1000cube", (1000, 1000, 1000), "uniform", 15, 0.01, False, c4r, _seeds(4, len(c4r)),
                       -1.0, 20, 0, 1.0, sum(c4r), 0),
        WorkloadConfig(5, "cfg5_skewed_4000x200x50", (4000, 200, 50), "collinear", 12, 0.03, False, c5r,
                       _seeds(5, len(c5r)), 1e-6, 1000, FLAG_LINESEARCH, 1.2, 640, 32, collinearity=0.8),
    ]


CONFIGS = {c.cid: c for c in _build()}


def get_config(cid: int) -> WorkloadConfig:
    return CONFIGS[int(cid)]
