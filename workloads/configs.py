"""The five synthetic workloads (shapes, class counts, label statistics, noise levels).

These stand in for the paper's video streams (Sec. 8.1: an action-recognition
frame stream and a long-tail image stream), reproducing the two properties its
memory relies on: long-tail class frequency and temporal locality (Sec. 3).
Only shapes and distribution parameters live here; no arithmetic of the method.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

BASE_SEED = 20211202


@dataclass(frozen=True)
class Workload:
    name: str
    index: int                      # position in the list of workloads; added to the base seed
    batch: int
    dtype: str                      # "f16" or "f32"
    exits: Tuple[Tuple[int, int, int], ...]   # (C, H, W) per exit point
    n_classes: int
    zipf_s: float
    run_mean: float                 # mean temporal run length in frames; 1.0 = no runs
    sigma: float                    # std of the per-element noise added to the broadcast centroid
    hot: int                        # initial fast-memory size
    off_memory: float = 0.0         # probability that a run shows something not in memory
    total_frames: int = 0           # 0 = one batch
    drift_every: int = 0            # frames between re-draws of the most probable classes
    drift_top: int = 0              # how many of the most probable ranks are re-drawn
    hot_min: int = 2
    hot_max: int = 0                # 0 = fixed fast memory (no adaptive size)
    window: int = 1024              # W of Eq. 5
    init_count: int = 100           # update count every centre starts with (Eq. 7's m)
    tau: float = 2.0                # benchmark threshold of Eq. 4
    tiers: int = 2

    @property
    def n_exits(self) -> int:
        return len(self.exits)

    @property
    def dims(self) -> List[int]:
        return [c for c, _, _ in self.exits]

    @property
    def esz(self) -> int:
        return 2 if self.dtype == "f16" else 4

    def frame_bytes(self) -> int:
        return sum(c * h * w for c, h, w in self.exits) * self.esz


TINY = Workload("tiny", 0, 64, "f32", ((64, 14, 14),), 10, 1.1, 1.0, 0.3, 4, tau=4.0)

RESNET18 = Workload("resnet18", 1, 256, "f16",
                    ((64, 56, 56), (128, 28, 28), (256, 14, 14), (512, 7, 7)),
                    100, 1.2, 8.0, 0.5, 16, tau=3.0)

RESNET50 = Workload("resnet50", 2, 1024, "f16",
                    ((256, 56, 56), (512, 28, 28), (1024, 14, 14), (2048, 7, 7)),
                    1000, 1.05, 16.0, 0.6, 100, off_memory=0.3, tau=5.0)

MOBILENETV2 = Workload("mobilenetv2", 3, 4096, "f16",
                       ((24, 56, 56), (32, 28, 28), (96, 14, 14), (320, 7, 7)),
                       1000, 1.1, 1.0, 0.5, 64, tau=1.0)

ADAPTIVE = Workload("adaptive", 4, 512, "f16",
                    ((256, 56, 56), (512, 28, 28), (512, 14, 14)),
                    1000, 1.1, 1.0, 0.5, 64, total_frames=100_000,
                    drift_every=10_000, drift_top=50, hot_min=32, hot_max=256,
                    window=1024, tau=4.0)

ALL = (TINY, RESNET18, RESNET50, MOBILENETV2, ADAPTIVE)
BY_NAME = {w.name: w for w in ALL}
