"""Diagnostics on top of the library: exit ratio per exit point and a threshold sweep.

Mirrors the paper's parameter study (arXiv 2112.02644, Sec. 8.6 exit ratio per layer, Sec. 8.7
threshold against accuracy and latency) on synthetic streams.  Everything on the path still runs
in the library's kernels; this module only drives the calls and aggregates the per-frame results.

    python -m paper_2112_02644_amd.diagnostics --workload resnet18 --taus 0 0.5 1 2 4 8 16
"""
from __future__ import annotations

import argparse
import json
from typing import Dict, List, Optional, Sequence

import numpy as np


def run_batch(ctx, fmaps, batch: int):
    """One batch through every exit point (full-batch tensors addressed through the live list).
    Returns numpy arrays exit_layer, label, tier by original frame id."""
    import torch
    dev = fmaps[0].device
    ctx.begin_batch(batch)
    for l, F in enumerate(fmaps, start=1):
        ctx.stage(l, F, row_ids=ctx.live_ids())
    res = [torch.zeros(batch, dtype=torch.int32, device=dev) for _ in range(3)]
    ctx.batch_results(*res)
    torch.cuda.synchronize()
    return tuple(r.cpu().numpy() for r in res)


def summarise(exit_layer: np.ndarray, label: np.ndarray, truth: np.ndarray, n_exits: int,
              segment_cost: Optional[Sequence[float]] = None) -> Dict:
    """Exit ratio per exit point, share of the network's cost still executed, and agreement of the
    released labels with the stream's own labels.

    segment_cost[l] is the relative cost of the network segment in front of exit point l+1
    (l = 0..L-1) and segment_cost[L] that of the rest of the network after the last exit point;
    equal shares by default.  A frame released at exit point l pays segments 0..l-1."""
    B = exit_layer.shape[0]
    cost = np.asarray(segment_cost if segment_cost is not None else np.ones(n_exits + 1), np.float64)
    cost = cost / cost.sum()
    paid = np.cumsum(cost)                                  # paid[l-1] = cost up to exit point l
    per_frame = np.where(exit_layer > 0, paid[np.maximum(exit_layer, 1) - 1], 1.0)
    released = exit_layer > 0
    known = truth >= 0
    right = released & known & (label == truth)
    return {
        "exit_ratio": [float((exit_layer == l).mean()) for l in range(1, n_exits + 1)],
        "ran_to_end": float((~released).mean()),
        "cost_executed": float(per_frame.mean()),           # 1.0 = no frame left early
        "released_correct": float(right.sum() / max(1, (released & known).sum())),
        "released_off_memory": float((released & ~known).sum() / max(1, (~known).sum())) if (~known).any() else 0.0,
    }


def tau_sweep(workload, taus: Sequence[float], device: str = "cuda:0", tiers: Optional[int] = None,
              segment_cost: Optional[Sequence[float]] = None) -> List[Dict]:
    """Runs one synthetic batch of `workload` at every threshold of `taus`."""
    import torch
    from workloads import streams
    from .smtm import Smtm, SmtmConfig

    w = workload
    cents = streams.centroids(w)
    ls = streams.labels(w, w.batch)
    fmaps = streams.batch_feature_maps(w, cents, ls, 0, device)
    ctx = Smtm(SmtmConfig(n_classes=w.n_classes, dims=w.dims, max_batch=w.batch, hot_init=w.hot,
                          hot_min=min(2, w.hot), hot_max=w.hot, tiers=w.tiers if tiers is None else tiers,
                          tau=float(taus[0]), window=w.window, init_count=w.init_count))
    for l, c in enumerate(cents, start=1):
        ctx.memory_load(l, c.numpy())
    ctx.hot_set(ls.initial_hot)
    out = []
    truth = ls.label[: w.batch]
    for tau in taus:
        ctx.set_tau(float(tau))
        exit_layer, label, tier = run_batch(ctx, fmaps, w.batch)
        row = {"tau": float(tau)}
        row.update(summarise(exit_layer, label, truth, w.n_exits, segment_cost))
        row["tier1_share"] = float((tier == 1).sum() / max(1, (tier > 0).sum()))
        out.append(row)
    ctx.close()
    return out


def main() -> int:
    from workloads import configs
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--workload", default="resnet18", choices=sorted(configs.BY_NAME))
    ap.add_argument("--taus", type=float, nargs="+", default=[0, 0.25, 0.5, 1, 2, 4, 8, 16, 64])
    ap.add_argument("--tiers", type=int, default=None)
    ap.add_argument("--json", action="store_true")
    args = ap.parse_args()
    rows = tau_sweep(configs.BY_NAME[args.workload], args.taus, tiers=args.tiers)
    if args.json:
        print(json.dumps(rows))
        return 0
    L = len(rows[0]["exit_ratio"])
    print(f"{'tau':>8s} " + " ".join(f"{'exit ' + str(l + 1):>8s}" for l in range(L))
          + f" {'to end':>8s} {'cost':>8s} {'correct':>8s} {'off-mem':>8s} {'tier 1':>8s}")
    for r in rows:
        print(f"{r['tau']:8.2f} " + " ".join(f"{x:8.3f}" for x in r["exit_ratio"])
              + f" {r['ran_to_end']:8.3f} {r['cost_executed']:8.3f} {r['released_correct']:8.3f}"
                f" {r['released_off_memory']:8.3f} {r['tier1_share']:8.3f}")
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
