#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

A step is one batch of the ResNet-50-shaped workload through every part of the path:
begin_batch, then at each of the four exit points encode -> lookup -> exit/compact (lists of the
released frames with labels and tiers, the survivors' feature maps gathered for the next block),
then the memory update.  The steps walk along the workload's frame stream: step s processes batch s
of the stream (up to --distinct batches are generated, 3.08 GB of feature maps each, after which the
stream wraps around), so the memory update meets new frames at every step.  All inputs are resident in
HBM before the clock starts; nothing is read back inside the timed region.

Prints one JSON line.  `value` is frames/s over the timed steps.  `roofline` is for the dominant
kernel (the instance of the 16-byte streaming encode kernel that serves exit point 1), timed with
events on the launch stream inside the timed region.  `cpu_baseline` is the CPU oracle on a
bounded sample of the same batch.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak

# HBM bytes per launch of the dominant kernel from the FETCH_SIZE / WRITE_SIZE counter runs summarised in
# profiles/encode_kernels_hbm_traffic.txt (same command, same workload).  Reported only while the kernel's
# source is the one the counters were taken on; otherwise the field is null.
TRAFFIC = {"workload": "resnet50", "bytes_per_launch": 1645583082.8,
           "encode_sha256": "9fa795b93429140b7650dc784deb98f67b2fbf7c4079b6273e1593f2215e59b9"}


def measured_traffic(workload: str):
    import hashlib
    from pathlib import Path
    src = Path(__file__).resolve().parent / "paper_2112_02644_amd" / "csrc" / "encode.hip"
    try:
        sha = hashlib.sha256(src.read_bytes()).hexdigest()
    except OSError:
        return None
    if workload != TRAFFIC["workload"] or sha != TRAFFIC["encode_sha256"]:
        return None
    return TRAFFIC["bytes_per_launch"]


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="resnet50")
    ap.add_argument("--cpu-sample", type=int, default=1024, help="frames of the batch given to the CPU oracle")
    ap.add_argument("--cpu-reps", type=int, default=4, help="times the CPU oracle runs that sample")
    ap.add_argument("--distinct", type=int, default=24,
                    help="distinct batches of the stream kept in HBM (the steps wrap around after that many)")
    ap.add_argument("--skip-extras", action="store_true",
                    help="leave out the informational runs after the timed region (no_exit, two_contexts), "
                         "e.g. under a profiler, where their kernels would mix into the per-kernel figures")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU; --gpus must be 1 (frames are independent, so more GPUs "
              "would each take a share of the batch with the memory tables replicated)", file=sys.stderr)
        return 2

    import torch
    from paper_2112_02644_amd import Smtm, SmtmConfig
    from workloads import configs, streams

    w = configs.BY_NAME[args.workload]
    dev = "cuda:0"
    torch.cuda.set_device(0)
    B, L, n = w.batch, w.n_exits, w.n_classes
    from oracle import smtm_oracle as O                     # only the cpu_baseline leg below uses it
    assert not os.environ.get("SMTM_ORACLE_LIB"), "the CPU baseline is the oracle built from oracle/smtm_oracle.c"
    cents = streams.centroids(w)
    total = args.steps + args.warmup
    n_distinct = max(1, min(total, args.distinct))
    ls = streams.labels(w, B * n_distinct)
    stream_fmaps = [streams.batch_feature_maps(w, cents, ls, b, dev) for b in range(n_distinct)]
    fmaps = stream_fmaps[0]
    gathers = [torch.empty_like(f) for f in fmaps]
    hot_max = w.hot_max or w.hot
    cfg = SmtmConfig(n_classes=n, dims=w.dims, max_batch=B, hot_init=w.hot,
                     hot_min=w.hot_min if w.hot_max else w.hot, hot_max=hot_max, tiers=w.tiers, tau=w.tau,
                     window=w.window, init_count=w.init_count)
    ctx = Smtm(cfg)
    for l, c in enumerate(cents, start=1):
        ctx.memory_load(l, c.numpy())
    ctx.hot_set(ls.initial_hot)

    i32 = dict(dtype=torch.int32, device=dev)
    # what a caller gets back per exit point: ids, labels and tiers of the frames released there
    exit_ids = [torch.zeros(B, **i32) for _ in range(L)]
    exit_labels = [torch.zeros(B, **i32) for _ in range(L)]
    exit_tier = [torch.zeros(B, **i32) for _ in range(L)]
    live_log = torch.zeros((total, L), **i32)              # survivors after each exit point, per step
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(L)]
          for _ in range(total)]
    esz = w.esz
    live_ptr0 = live_log.data_ptr()
    # dominant kernel: the encode kernel instance that serves the largest feature map; the library names the
    # instance each encode launched, and every exit point served by that same instance is timed with it
    big = max(range(L), key=lambda l: w.exits[l][0] * w.exits[l][1] * w.exits[l][2])
    ctx.begin_batch(B)
    for l in range(1, L + 1):
        ctx.encode(l, fmaps[l - 1], row_ids=ctx.live_ids())
    torch.cuda.synchronize()
    enc_names = [ctx.encode_kernel(l) for l in range(1, L + 1)]
    dom = [l for l in range(L) if enc_names[l] == enc_names[big]]

    def step(s: int):
        ctx.begin_batch(B)
        for l in range(1, L + 1):
            F = stream_fmaps[s % n_distinct][l - 1]
            ids = ctx.live_ids()
            if (l - 1) in dom:                              # events only around the dominant kernel's launches
                a, b = ev[s][l - 1]
                a.record()
                ctx.encode(l, F, row_ids=ids)
                b.record()
            else:
                ctx.encode(l, F, row_ids=ids)
            ctx.lookup_exit(l, exit_ids=exit_ids[l - 1], exit_labels=exit_labels[l - 1], exit_tier=exit_tier[l - 1],
                            n_live_dev=live_ptr0 + 4 * (s * L + l - 1), fmap_in=F, row_ids=ids,
                            fmap_out=gathers[l - 1], row_bytes=F[0].numel() * esz)
        ctx.cache_update(None, None, B)                     # memory update with the batch's own exits

    for s in range(args.warmup):
        step(s)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.warmup, total):
        step(s)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    fps = B * args.steps / elapsed

    # ---- what the timed steps did
    live = live_log.cpu().numpy()[args.warmup:]            # [steps, L] survivors after exit l
    entering = np.concatenate([np.full((args.steps, 1), B), live[:, :-1]], axis=1)   # live frames entering exit l
    exits = entering - live
    enc_ms = np.array([[ev[s][l][0].elapsed_time(ev[s][l][1]) if l in dom else np.nan for l in range(L)]
                       for s in range(args.warmup, total)])
    per_exit_bytes = np.array([c * h * wd * esz + c * 4 for c, h, wd in w.exits], dtype=np.float64)
    enc_bytes = entering * per_exit_bytes[None, :]
    dom_bytes = enc_bytes[:, dom].sum() / (args.steps * len(dom))
    dom_ms = enc_ms[:, dom].sum() / (args.steps * len(dom))
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9
    gat_bytes = live * (per_exit_bytes[None, :] - np.array([c * 4 for c, _, _ in w.exits])[None, :]) * 2.0
    path_bytes = (enc_bytes.sum(axis=1) + gat_bytes.sum(axis=1)).mean()   # algorithmic bytes per step: encode stream + gather (read + write)
    stage_gbs = path_bytes / (ms_per_step * 1e-3) / 1e9

    # ---- after the timed region: the exit-point-1 stage alone (encode + lookup + exit/compact on the full
    # batch, no gather), bracketed by events, as a fraction of the HBM roofline
    reps = 10
    sev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for r in range(reps):
        ctx.begin_batch(B)
        sev[r][0].record()
        ctx.encode(1, fmaps[0], row_ids=ctx.live_ids())
        ctx.lookup_exit(1)
        sev[r][1].record()
        # keep the L2 / memory-side cache from holding the start of the tensor for the next repetition
        if L > 1:
            ctx.encode(2, fmaps[1], row_ids=ctx.live_ids())
    torch.cuda.synchronize()
    stage1_ms = float(np.median([a.elapsed_time(b) for a, b in sev]))
    stage1_bytes = B * per_exit_bytes[0]

    noexit_clean, noexit_ms, noexit_bytes = False, 1.0, 0.0
    if not args.skip_extras:
        # ---- the clean bandwidth case: an unreachable threshold, so every frame is live at every exit point
        # (encode + lookup + exit/compact at all exit points; nothing to gather, nothing released)
        ctx.set_tau(3.0e38)
        # timed like the headline: one pair of events around all repetitions (an event record between two
        # batches costs microseconds of its own), batches taken from along the stream
        nreps = 2 * reps
        nev = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
        left = torch.zeros(nreps + 2, **i32)             # frames still live at the end of each batch
        for r in range(-2, nreps):
            if r == 0:
                nev[0].record()
            F = stream_fmaps[r % n_distinct]
            ctx.begin_batch(B)
            for l in range(1, L + 1):
                ctx.encode(l, F[l - 1], row_ids=ctx.live_ids())
                ctx.lookup_exit(l, n_live_dev=left[r + 2:r + 3] if l == L else None)
        nev[1].record()
        torch.cuda.synchronize()
        n_live_end = int(left.min().item())
        # a frame whose second-best class is not positively correlated leaves at any threshold (the exit rule has
        # max(SA_SH, 0) on its right-hand side); the figure is reported only when no frame did
        noexit_clean = n_live_end == B
        ctx.set_tau(w.tau)
        noexit_ms = nev[0].elapsed_time(nev[1]) / nreps
        noexit_bytes = B * per_exit_bytes.sum()

    two_fps = None
    if not args.skip_extras:
        # ---- two independent streams of frames (two contexts with their own memory, inputs and outputs) driven
        # from two HIP streams: the small dependent kernels of one overlap the streaming kernels of the other.
        # Informational; `value` above is the single-context figure.
        def make_lane():
            c2 = Smtm(cfg)
            for l, c in enumerate(cents, start=1):
                c2.memory_load(l, c.numpy())
            c2.hot_set(ls.initial_hot)
            st = torch.cuda.Stream()
            c2.stream = st.cuda_stream
            return dict(ctx=c2, st=st, gathers=[torch.empty_like(f) for f in fmaps],
                        lists=[[torch.zeros(B, **i32) for _ in range(3)] for _ in range(L)])

        def lane_step(lane, s):
            c2 = lane["ctx"]
            c2.begin_batch(B)
            for l in range(1, L + 1):
                F = stream_fmaps[s % n_distinct][l - 1]     # each lane walks the stream too, half a lap apart
                ids = c2.live_ids()
                c2.encode(l, F, row_ids=ids)
                e = lane["lists"][l - 1]
                c2.lookup_exit(l, exit_ids=e[0], exit_labels=e[1], exit_tier=e[2], fmap_in=F, row_ids=ids,
                               fmap_out=lane["gathers"][l - 1], row_bytes=F[0].numel() * esz)
            c2.cache_update(None, None, B)

        lanes = [make_lane(), make_lane()]
        torch.cuda.synchronize()
        for k in range(args.warmup + args.steps):
            if k == args.warmup:
                torch.cuda.synchronize()
                t2 = time.perf_counter()
            for i, lane in enumerate(lanes):
                lane_step(lane, k + i * (n_distinct // 2))
        torch.cuda.synchronize()
        two_fps = 2 * B * args.steps / (time.perf_counter() - t2)
        for lane in lanes:
            lane["ctx"].close()
        del lanes

    # ---- one frame at a time (the paper's own cadence): a batch of one through every exit point and the
    # memory update, recorded once in a HIP graph and replayed.  Informational: latency, not throughput.
    one_frame_us = None
    if not args.skip_extras:
        try:
            c1 = Smtm(SmtmConfig(n_classes=n, dims=w.dims, max_batch=1, hot_init=w.hot,
                                 hot_min=w.hot_min if w.hot_max else w.hot, hot_max=hot_max, tiers=w.tiers,
                                 tau=w.tau, window=w.window, init_count=w.init_count))
            for l, c in enumerate(cents, start=1):
                c1.memory_load(l, c.numpy())
            c1.hot_set(ls.initial_hot)
            one = [f[:1].clone() for f in fmaps]

            def one_step():
                c1.begin_batch(1)
                for l in range(1, L + 1):
                    c1.encode(l, one[l - 1], row_ids=c1.live_ids())
                    c1.lookup_exit(l)
                c1.cache_update(None, None, 1)

            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                one_step()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                one_step()
            for _ in range(5):
                graph.replay()
            torch.cuda.synchronize()
            t3 = time.perf_counter()
            n_rep = 200
            for _ in range(n_rep):
                graph.replay()
            torch.cuda.synchronize()
            one_frame_us = (time.perf_counter() - t3) / n_rep * 1e6
            del graph
            c1.close()
        except Exception as e:                               # reported, never fatal for the main figure
            print(f"bench.py: single-frame graph run skipped: {e}", file=sys.stderr)

    ns = min(args.cpu_sample, B)
    host = [f[:ns].cpu().numpy() for f in fmaps]
    cores = O.get_max_threads()

    def oracle_seconds(frames: int, times: int) -> float:
        total_s = 0.0
        for _ in range(times):                           # the same frames each time, from a fresh memory
            mem = O.Memory([c.numpy() for c in cents], ls.initial_hot, tau=w.tau, tiers=w.tiers, window=w.window,
                           hot_min=cfg.hot_min, hot_max=hot_max, init_count=w.init_count)
            t1 = time.perf_counter()
            mem.begin_batch(frames)
            for l in range(1, L + 1):
                mem.stage(l, host[l - 1][:frames], row_ids=mem.live.copy())
            mem.cache_update(mem.label, mem.exit_layer)
            total_s += time.perf_counter() - t1
        return total_s

    cpu_s = oracle_seconds(ns, args.cpu_reps)
    n1 = min(ns, 128)                                    # one thread: a smaller sample of the same frames
    O.set_threads(1)
    cpu1_s = oracle_seconds(n1, 1)
    O.set_threads(cores)
    try:
        cpu_model = next(ln.split(":", 1)[1].strip() for ln in open("/proc/cpuinfo") if ln.startswith("model name"))
    except (OSError, StopIteration):
        cpu_model = "unknown"

    out = {
        "metric": "frames/sec through encode+lookup+exit (ResNet-50 exits)" if w.name == "resnet50"
                  else f"frames/sec through encode+lookup+exit ({w.name} exits)",
        "value": fps, "unit": "frames/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16" if w.dtype == "f16" else "f32", "accumulate": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}-shaped: batch {B}, {L} exit points "
                               + ",".join(f"[{c},{h},{wd}]" for c, h, wd in w.exits)
                               + f", {n} classes, hot {w.hot}, tau {w.tau}, tiers {w.tiers}, survivors gathered, "
                                 f"memory update every batch, {n_distinct} distinct batches of the stream",
                   "exits_per_exit_point": exits.mean(axis=0).round(1).tolist(),
                   "ran_to_end": float(live[:, -1].mean())},
        "roofline": {"bound": "hbm", "kernel": enc_names[big], "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(w.name),
                     "bytes_per_launch": dom_bytes, "avg_launch_ms": dom_ms},
        "cpu_baseline": {"value": ns * args.cpu_reps / cpu_s, "unit": "frames/s", "cores": cores, "kind": "oracle",
                         "sample": f"first {ns} frames of the same batch, all {L} exit points and the memory "
                                   f"update, {args.cpu_reps} times over: {cpu_s:.2f} s on {cores} threads",
                         "one_thread": {"value": n1 / cpu1_s, "sample": f"first {n1} frames, once: {cpu1_s:.2f} s"},
                         "cpu": cpu_model, "host_cpus": os.cpu_count(),
                         "gpu_over_oracle": fps / (ns * args.cpu_reps / cpu_s)},
        "encode_ms_per_exit_point": [None if np.isnan(x) else round(float(x), 4) for x in enc_ms.mean(axis=0)],
        "encode_gbs_per_exit_point": [None if np.isnan(t) else round(float(b / (t * 1e-3) / 1e9), 1)
                                      for b, t in zip(enc_bytes.mean(axis=0), enc_ms.mean(axis=0))],
        "path_hbm_frac": stage_gbs / HBM_PEAK_GBS,
        "exit1_stage": {"what": "encode + lookup + exit/compact of exit point 1 on the full batch, no gather",
                        "ms": stage1_ms, "GB/s": stage1_bytes / (stage1_ms * 1e-3) / 1e9,
                        "hbm_frac": stage1_bytes / (stage1_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "no_exit": {"what": "unreachable threshold: every frame live at every exit point; encode + lookup + "
                            "exit/compact at all exit points, nothing to gather; batches along the stream, "
                            "one pair of events around all of them",
                    "ms": noexit_ms, "frames/s": B / (noexit_ms * 1e-3),
                    "GB/s": noexit_bytes / (noexit_ms * 1e-3) / 1e9,
                    "hbm_frac": noexit_bytes / (noexit_ms * 1e-3) / 1e9 / HBM_PEAK_GBS} if noexit_clean else None,
        "two_contexts": {"what": "two independent frame streams (two contexts with their own memory, walking the same "
                                 "stream of batches half a lap apart) on two HIP streams; aggregate", "frames/s": two_fps} if two_fps else None,
        "one_frame": {"what": "batch of one through every exit point and the memory update, replayed from a HIP "
                              "graph; microseconds per frame", "us": one_frame_us} if one_frame_us else None,
        # survivors after each exit point for every step run (warm-up included), so that per-dispatch
        # byte counts of a profile of this command can be reconstructed
        "survivors_log": live_log.cpu().numpy().tolist(),
        "encode_kernels": enc_names,
    }
    print(json.dumps(out))
    ctx.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
