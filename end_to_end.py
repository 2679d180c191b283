"""End-to-end latency with real convolution blocks between the exit points.

A ResNet-50-shaped trunk (random weights, batch norm folded away, fp16, channels last) runs on the
GPU through PyTorch's convolutions; after each of its four stages the library encodes the stage's
output, looks it up, releases the frames whose accumulated confidence passes the threshold and
gathers the survivors' rows, so the next stage runs on the compacted batch only
(arXiv 2112.02644, Sec. 4 workflow; Sec. 8.2 and 8.7 measure the resulting latency).  Speed and
exit ratios only: with random weights and synthetic images the labels say nothing about accuracy
on real data.  The released labels are still compared with the stream's own labels.

Images: a class is a texture (a mean colour plus a few coloured gratings of its own frequencies and
orientations), a frame is its class texture at fresh phases plus per-pixel Gaussian noise;
off-memory frames show a texture of their own.  Centres come from the library's warm-up over a labelled pass of the same generator.

    python end_to_end.py --batch 1024 --taus 0.02 0.01 0.005

A demonstration next to the benchmark, not part of the library: the convolutions are PyTorch's.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import math
import sys
import time
from typing import Dict, List, Sequence

import numpy as np

ROOT = __import__("pathlib").Path(__file__).resolve().parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

STAGES = ((64, 256, 3, 1), (128, 512, 4, 2), (256, 1024, 6, 2), (512, 2048, 3, 2))   # mid, out, blocks, stride
SEED = 20211202


def _say(*a):
    print(*a, file=sys.stderr, flush=True)


def build_trunk(device, n_classes: int):
    """Stem, four stages of bottleneck blocks and the classifier head, as a list of modules."""
    import torch
    from torch import nn

    class Bottleneck(nn.Module):
        def __init__(self, cin, mid, cout, stride):
            super().__init__()
            self.a = nn.Conv2d(cin, mid, 1)
            self.b = nn.Conv2d(mid, mid, 3, stride=stride, padding=1)
            self.c = nn.Conv2d(mid, cout, 1)
            self.short = None if (cin == cout and stride == 1) else nn.Conv2d(cin, cout, 1, stride=stride)

        def forward(self, x):
            y = torch.relu_(self.a(x))
            y = torch.relu_(self.b(y))
            y = self.c(y)                           # its weights carry the damping factor, see below
            s = x if self.short is None else self.short(x)
            return torch.relu_(y.add_(s))

    torch.manual_seed(SEED)
    stem = nn.Sequential(nn.Conv2d(3, 64, 7, stride=2, padding=3), nn.ReLU(inplace=True),
                         nn.MaxPool2d(3, stride=2, padding=1))
    stages, cin = [], 64
    for mid, cout, blocks, stride in STAGES:
        layers = []
        for i in range(blocks):
            layers.append(Bottleneck(cin, mid, cout, stride if i == 0 else 1))
            cin = cout
        stages.append(nn.Sequential(*layers))
    head = nn.Sequential(nn.AdaptiveAvgPool2d(1), nn.Flatten(), nn.Linear(cin, n_classes))
    mods = [stem] + stages + [head]
    for m in mods:
        m.requires_grad_(False)
        for p in m.modules():
            if isinstance(p, nn.Conv2d):
                nn.init.kaiming_normal_(p.weight, nonlinearity="relu")
                nn.init.zeros_(p.bias)
        for p in m.modules():
            if isinstance(p, Bottleneck):              # damped branches keep fp16 activations in range
                p.c.weight.mul_(0.5)
                if p.short is not None:
                    p.short.weight.mul_(0.5)
        m.eval().to(device=device, dtype=torch.float16,
                                           memory_format=torch.channels_last)
    return mods


class Images:
    """Seeded synthetic frames on the device, [B, 3, 224, 224] fp16 channels last.

    A class is a texture: a mean colour plus `waves` coloured gratings of its own frequencies and
    orientations.  A frame of the class draws fresh phases and per-pixel noise, so frames of one
    class differ pixel by pixel and agree in the statistics that survive average pooling."""

    def __init__(self, n_classes: int, device, noise: float = 0.5, waves: int = 4):
        import torch
        self.torch, self.device, self.noise, self.waves = torch, device, noise, waves
        g = torch.Generator(device="cpu").manual_seed(SEED + 1)
        self.params = self._draw(n_classes, g).to(device)
        self.g = torch.Generator(device=device).manual_seed(SEED + 2)
        yy, xx = torch.meshgrid(torch.arange(224.0), torch.arange(224.0), indexing="ij")
        self.xx, self.yy = xx.to(device), yy.to(device)

    def _draw(self, count: int, g, device="cpu"):
        """[count, waves, 5] (fx, fy, colour) and, in row `waves`, the mean colour."""
        torch = self.torch
        k = self.waves
        period = 4.0 * (16.0 ** torch.rand(count, k, generator=g, device=device))      # 4 .. 64 pixels
        angle = math.pi * torch.rand(count, k, generator=g, device=device)
        f = 2.0 * math.pi / period
        colour = torch.randn(count, k, 3, generator=g, device=device)
        wave = torch.cat([(f * torch.cos(angle))[..., None], (f * torch.sin(angle))[..., None], colour], dim=2)
        mean = torch.cat([torch.zeros(count, 1, 2, device=device),
                          0.5 * torch.randn(count, 1, 3, generator=g, device=device)], dim=2)
        return torch.cat([wave, mean], dim=1)

    def batch(self, label: np.ndarray):
        torch = self.torch
        lab = torch.from_numpy(label.astype(np.int64)).to(self.device)
        par = self.params[lab.clamp(min=0)]
        off = lab < 0
        if bool(off.any()):
            par = par.clone()
            par[off] = self._draw(int(off.sum()), self.g, self.device)
        B, k = par.shape[0], self.waves
        phase = 2.0 * math.pi * torch.rand(B, k, generator=self.g, device=self.device)
        x = par[:, k, 2:5, None, None] + self.noise * torch.randn((B, 3, 224, 224), generator=self.g,
                                                                  device=self.device)
        for i in range(k):
            arg = (par[:, i, 0, None, None] * self.xx + par[:, i, 1, None, None] * self.yy
                   + phase[:, i, None, None])
            x = x + par[:, i, 2:5, None, None] * torch.cos(arg)[:, None]
        return x.to(torch.float16).contiguous(memory_format=torch.channels_last)


def nhwc(x):
    """[N, H, W, C] contiguous view of a channels-last [N, C, H, W] tensor."""
    import torch
    if not x.is_contiguous(memory_format=torch.channels_last):
        x = x.contiguous(memory_format=torch.channels_last)
    return x.permute(0, 2, 3, 1)


def warm_up(ctx, mods, images: Images, n_classes: int, batch: int, samples: int):
    """Centres as class means over `samples` labelled frames per class (Sec. 5 initialisation)."""
    import torch
    rng = np.random.Generator(np.random.Philox(SEED + 3))
    order = np.concatenate([rng.permutation(n_classes) for _ in range(samples)]).astype(np.int32)
    ctx.warmup_begin()
    for lo in range(0, order.shape[0], batch):
        lab = order[lo: lo + batch]
        x = mods[0](images.batch(lab))
        ctx.begin_batch(lab.shape[0])
        for l in range(1, 5):
            x = mods[l](x)
            ctx.encode_nhwc(l, nhwc(x))
        ctx.warmup_batch(torch.from_numpy(lab).to(x.device), lab.shape[0])
        torch.cuda.synchronize()
        _say(f"warm-up frames {lo + lab.shape[0]}/{order.shape[0]}")


def forward_plain(mods, img):
    x = img
    for m in mods:
        x = m(x)
    return x


def forward_cached(ctx, mods, img, bufs, bucket: int):
    """One batch with the memory in the loop.  Returns the survivors' count after each exit point.
    The host reads the live count after every exit point: PyTorch needs it to shape the next call."""
    B = img.shape[0]
    ctx.begin_batch(B)
    x = mods[0](img)
    live = []
    n_live = B
    for l in range(1, 5):
        x = mods[l](x)
        xv = nhwc(x)
        ctx.stage_nhwc(l, xv, fmap_out=bufs[l - 1])
        n_live, _ = ctx.read_counts()
        live.append(n_live)
        if n_live == 0:
            break
        n_pad = min(B, (n_live + bucket - 1) // bucket * bucket)   # few distinct shapes for the convolutions
        x = bufs[l - 1][:n_pad].permute(0, 3, 1, 2)
    if n_live:
        mods[5](x[:n_live])
    ctx.cache_update(None, None, B)
    return live + [0] * (4 - len(live))


def metric_profile(ctx, mods, img, label: np.ndarray, hot_ids: np.ndarray) -> List[Dict]:
    """Accumulated confidence (Eq. 4) of every frame at every exit point with nothing released,
    summarised per exit point: quantiles over the frames of fast-memory classes, and how often the
    best fast-memory class is the frame's own.  Shows which thresholds separate anything."""
    import torch
    B = img.shape[0]
    dev = img.device
    tv = torch.zeros(B, 2, 2, dtype=torch.float32, device=dev)
    ti = torch.zeros(B, 2, dtype=torch.int32, device=dev)
    ctx.set_tau(3.0e38)
    ctx.begin_batch(B)
    x = mods[0](img)
    in_hot = np.isin(label, hot_ids)
    out = []
    for l in range(1, 5):
        x = mods[l](x)
        ctx.encode_nhwc(l, nhwc(x))
        ctx.lookup_exit(l, top_val=tv, top_id=ti)
        torch.cuda.synchronize()
        v, i = tv.cpu().numpy(), ti.cpu().numpy()
        ac = (v[:, 0, 0] - v[:, 0, 1]) / np.maximum(v[:, 0, 1], 1e-30)
        q = lambda a: [float(t) for t in np.quantile(a, [0.1, 0.5, 0.9])] if a.size else []
        out.append({"exit": l, "ac_hot_q10_q50_q90": q(ac[in_hot]), "ac_other_q10_q50_q90": q(ac[~in_hot]),
                    "hot_top1_right": float((i[in_hot, 0] == label[in_hot]).mean()) if in_hot.any() else 0.0,
                    "global_top1_right": float((i[label >= 0, 1] == label[label >= 0]).mean())})
    return out


def timed(fn, reps: int) -> float:
    import torch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / reps * 1e3


def run(batch: int, taus: Sequence[float], n_classes: int, hot: int, reps: int, samples: int,
        bucket: int, device: str = "cuda:0") -> Dict:
    import torch
    from workloads import configs, streams
    from paper_2112_02644_amd import Smtm, SmtmConfig

    torch.backends.cudnn.benchmark = False
    w = dataclasses.replace(configs.RESNET50, n_classes=n_classes, hot=hot, batch=batch)
    dims = tuple(s[1] for s in STAGES)
    mods = build_trunk(device, n_classes)
    images = Images(n_classes, device)
    ctx = Smtm(SmtmConfig(n_classes=n_classes, dims=dims, max_batch=batch, hot_init=hot, hot_min=hot,
                          hot_max=hot, tiers=2, tau=float(taus[0]), window=w.window, init_count=1))
    _say("trunk built; warm-up")
    warm_up(ctx, mods, images, n_classes, batch, samples)

    ls = streams.labels(w, batch)
    label = ls.label.astype(np.int32)
    ctx.hot_set(ls.initial_hot)
    img = images.batch(label)
    shapes = [(56, 56, 256), (28, 28, 512), (14, 14, 1024), (7, 7, 2048)]
    bufs = [torch.zeros((batch,) + s, dtype=torch.float16, device=device) for s in shapes]

    forward_plain(mods, img)
    plain_ms = timed(lambda: forward_plain(mods, img), reps)
    _say(f"no memory: {plain_ms:.2f} ms per batch of {batch}")

    profile = metric_profile(ctx, mods, img, label, ls.initial_hot)
    for r in profile:
        _say(json.dumps(r))

    ft, ts, _, _ = ctx.tables_export()
    rows: List[Dict] = []
    res = [torch.zeros(batch, dtype=torch.int32, device=device) for _ in range(3)]
    for tau in taus:
        ctx.set_tau(float(tau))
        ctx.tables_import(ft, ts)                       # same tables and fast memory for every threshold
        ctx.hot_set(ls.initial_hot)
        for _ in range(2):                              # lets the convolutions see their shapes
            live = forward_cached(ctx, mods, img, bufs, bucket)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            live = forward_cached(ctx, mods, img, bufs, bucket)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / reps * 1e3
        ctx.batch_results(*res)                         # of the last timed batch
        torch.cuda.synchronize()
        exit_layer, lab, tier = (r.cpu().numpy() for r in res)
        released = exit_layer > 0
        known = label >= 0
        rows.append({
            "tau": float(tau), "ms": ms, "speedup": plain_ms / ms, "live_after_exit": live,
            "exit_ratio": [float((exit_layer == l).mean()) for l in range(1, 5)],
            "released_correct": float((released & known & (lab == label)).sum() / max(1, (released & known).sum())),
            "released_off_memory": float((released & ~known).sum() / max(1, (~known).sum())),
            "tier1_share": float((tier == 1).sum() / max(1, released.sum())),
        })
        _say(f"tau {tau:g}: {ms:.2f} ms, x{plain_ms / ms:.2f}, live after each exit point {live}")
    ctx.close()
    return {"batch": batch, "n_classes": n_classes, "hot": hot, "no_memory_ms": plain_ms, "confidence_profile": profile,
            "rows": rows,
            "data": "synthetic images, random weights"}


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--batch", type=int, default=1024)
    ap.add_argument("--classes", type=int, default=1000)
    ap.add_argument("--hot", type=int, default=100)
    ap.add_argument("--taus", type=float, nargs="+", default=[3.0e38, 0.02, 0.01, 0.005, 0.002])
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--samples", type=int, default=2, help="warm-up frames per class")
    ap.add_argument("--bucket", type=int, default=64, help="survivor counts are rounded up to this for the convolutions")
    args = ap.parse_args()
    out = run(args.batch, args.taus, args.classes, args.hot, args.reps, args.samples, args.bucket)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
