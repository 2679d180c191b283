"""Seeded synthetic frame streams: centroids, long-tail labels with temporal runs, feature maps.

Recipe (one place, used by the tests, the smoke check and the benchmark):
  * centroids: standard Gaussian in R^C per class and exit point, scaled to unit length,
    independent per exit point, float32;
  * labels: a class *rank* r is drawn with p(r) proportional to r^-s, mapped to a class id by
    a seeded permutation; a run length is drawn from Geometric(1/mean) on {1,2,...} and the
    class is emitted for that many frames; with probability `off_memory` a run shows
    something that is not in memory (label -1, a fresh random unit vector per exit point);
    for drifting streams the classes holding the `drift_top` most probable ranks are re-drawn
    every `drift_every` frames;
  * feature map of a frame at an exit point: its base vector broadcast over H x W plus
    i.i.d. N(0, sigma^2) noise per element, rounded once to the workload's dtype.

Nothing here belongs to the method under test: no pooling, similarity, metric or policy.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional

import numpy as np
import torch

from .configs import BASE_SEED, Workload


def _seed(w: Workload, *salt: int) -> int:
    s = BASE_SEED + 1000 * w.index
    for i, v in enumerate(salt):
        s += (i + 1) * 100_003 * int(v)
    return s


def torch_dtype(w: Workload) -> torch.dtype:
    return torch.float16 if w.dtype == "f16" else torch.float32


def centroids(w: Workload) -> List[torch.Tensor]:
    """Unit-length Gaussian class vectors, one [n_classes, C] float32 CPU tensor per exit point."""
    out = []
    for l, (c, _, _) in enumerate(w.exits):
        g = torch.Generator().manual_seed(_seed(w, 1, l))
        x = torch.randn(w.n_classes, c, generator=g, dtype=torch.float64)
        x = x / x.norm(dim=1, keepdim=True)
        out.append(x.to(torch.float32).contiguous())
    return out


@dataclass
class LabelStream:
    label: np.ndarray        # [N] int32, -1 for off-memory frames
    run: np.ndarray          # [N] int32 run index of each frame
    rank_of_run: np.ndarray  # [n_runs] int32 Zipf rank (0-based) drawn for the run
    initial_hot: np.ndarray  # class ids of the `hot` most probable ranks at frame 0


def labels(w: Workload, n_frames: Optional[int] = None) -> LabelStream:
    n_frames = int(n_frames or w.total_frames or w.batch)
    rng = np.random.Generator(np.random.Philox(_seed(w, 2)))
    n = w.n_classes
    p = np.arange(1, n + 1, dtype=np.float64) ** (-w.zipf_s)
    p /= p.sum()
    perm = rng.permutation(n).astype(np.int32)          # rank -> class id
    initial_hot = perm[: w.hot].copy()
    label = np.empty(n_frames, np.int32)
    run = np.empty(n_frames, np.int32)
    ranks = []
    t = 0
    next_drift = w.drift_every if w.drift_every else None
    while t < n_frames:
        if next_drift is not None and t >= next_drift:
            chosen = rng.choice(n, size=w.drift_top, replace=False)
            for r, c in enumerate(chosen):
                r_old = int(np.nonzero(perm == c)[0][0])
                perm[r], perm[r_old] = perm[r_old], perm[r]
            next_drift += w.drift_every
        r = int(rng.choice(n, p=p))
        length = int(rng.geometric(1.0 / w.run_mean)) if w.run_mean > 1.0 else 1
        off = w.off_memory > 0.0 and rng.random() < w.off_memory
        end = min(n_frames, t + length)
        if next_drift is not None:
            end = min(end, next_drift)
        label[t:end] = -1 if off else perm[r]
        run[t:end] = len(ranks)
        ranks.append(r)
        t = end
    return LabelStream(label, run, np.array(ranks, np.int32), initial_hot)


def bases(w: Workload, cents: List[torch.Tensor], ls: LabelStream, lo: int, hi: int,
          exit_index: int) -> torch.Tensor:
    """Base vector of frames lo..hi-1 at one exit point: [hi-lo, C] float32 CPU tensor."""
    lab = torch.from_numpy(ls.label[lo:hi].astype(np.int64))
    c = w.exits[exit_index][0]
    base = cents[exit_index][lab.clamp(min=0)].clone()
    off = lab < 0
    if bool(off.any()):
        runs = ls.run[lo:hi]
        for r in np.unique(runs[off.numpy()]):
            g = torch.Generator().manual_seed(_seed(w, 3, exit_index, int(r)))
            u = torch.randn(c, generator=g, dtype=torch.float64)
            u = (u / u.norm()).to(torch.float32)
            base[torch.from_numpy(runs == r)] = u
    return base


def feature_maps(w: Workload, exit_index: int, base: torch.Tensor, batch_index: int = 0,
                 device: str = "cpu", sigma: Optional[float] = None) -> torch.Tensor:
    """[B, C, H, W] tensor in the workload's dtype on `device`: base broadcast + Gaussian noise."""
    c, h, wd = w.exits[exit_index]
    b = base.shape[0]
    sigma = w.sigma if sigma is None else sigma
    dt = torch_dtype(w)
    out = torch.empty((b, c, h, wd), dtype=dt, device=device)
    g = torch.Generator(device=device).manual_seed(_seed(w, 4, exit_index, batch_index))
    base = base.to(device)
    per_frame = c * h * wd * 4
    step = max(1, min(b, (256 << 20) // per_frame))
    for s in range(0, b, step):
        e = min(b, s + step)
        x = torch.randn((e - s, c, h, wd), generator=g, dtype=torch.float32, device=device)
        x.mul_(sigma).add_(base[s:e, :, None, None])
        out[s:e] = x.to(dt)
    return out


def batch_feature_maps(w: Workload, cents: List[torch.Tensor], ls: LabelStream, batch_index: int,
                       device: str = "cpu") -> List[torch.Tensor]:
    """All exit points' feature maps of one batch of the stream."""
    lo = batch_index * w.batch
    hi = min(lo + w.batch, ls.label.shape[0])
    return [feature_maps(w, l, bases(w, cents, ls, lo, hi, l), batch_index, device)
            for l in range(w.n_exits)]
