"""Parity harness: runs a workload through the HIP library (via its C ABI) and through the CPU
oracle on the same bits, exit point by exit point with teacher forcing, and checks

  * semantic vectors, similarities and accumulated similarities within the stated tolerance,
  * exit decisions and labels identical except for frames whose metric lies within the
    tolerance band of the threshold (counted and returned),
  * index work (exit lists, live lists, counts, gathered rows) bit-exact,
  * the library's own decisions equal to the exit rule applied to its own top-2 values.

Tolerances (see the derivation in the design notes): a similarity computed from fp32 feature
maps is within 1e-5, from fp16 feature maps within 2e-3, of the oracle's, relative to
max(|s|, a) where a = sum_c |v_c||c_c| / (|v||c|) is the rounding-error scale of the dot product.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch

from oracle import smtm_oracle as O
from paper_2112_02644_amd import Smtm, SmtmConfig, SCORE_AUTO, SCORE_FP32, SCORE_MFMA
from workloads import streams
from workloads.configs import Workload

SV_RTOL = 1e-5


def sim_rtol(w: Workload, score_path: int = SCORE_AUTO) -> float:
    if score_path == SCORE_FP32:
        return 1e-5
    if score_path == SCORE_MFMA:
        return 2e-3
    return 2e-3 if w.dtype == "f16" else 1e-5


def rule_fp32(h, sh, tau):
    """The exit rule in fp32 arithmetic, as the library evaluates it."""
    h = np.float32(h); sh = np.float32(sh); tau = np.float32(tau)
    if not (h > 0) or sh == -np.inf:
        return False
    runner = sh if sh > 0 else np.float32(0)
    return bool(np.float32(h - sh) > np.float32(tau * runner))


def dot_scale(SV: np.ndarray, SC: np.ndarray) -> np.ndarray:
    """a[i, j] = sum_c |v_c||c_c| / (|v||c|): the rounding-error scale of the cosine of row i of SV
    with row j of SC (the similarity tolerance is rtol * max(|s|, a), and |s| <= a <= 1)."""
    nv = np.linalg.norm(SV, axis=1)
    nc = np.linalg.norm(SC, axis=1)
    with np.errstate(divide="ignore", invalid="ignore"):
        a = (np.abs(SV) @ np.abs(SC).T) / (nv[:, None] * nc[None, :])
    a[~np.isfinite(a)] = 0.0
    return a


def in_band(h, sh, tau, l, delta, scale=None):
    """Frames whose metric is within the tolerance of the threshold may differ in decision.

    Every similarity may be off by delta * a, so an accumulated similarity of exit point l may be
    off by delta * scale, scale = sum over the exit points so far of 2^(l'-1) * a (at most 2^l - 1,
    the default).  The exit rule compares SA_H with (1 + tau) * max(SA_SH, 0): its two sides may
    move by delta * scale * (2 + tau) against each other, and the sign of SA_H is uncertain while
    |SA_H| <= delta * scale.  `scale` is the largest one over the tier's classes, because rounding
    may also change which class is second."""
    if not np.isfinite(h) or not np.isfinite(sh):
        return False
    if scale is None:
        scale = 2.0 ** l - 1.0
    g = h - (1.0 + tau) * max(sh, 0.0)
    if abs(g) <= delta * scale * (2.0 + tau):
        return True
    return abs(h) <= delta * scale


def in_narrow_band(h, sh, tau, l, delta):
    """The narrower band relative to the frame's own accumulated similarities:
    |SA_H - (1+tau) max(SA_SH,0)| <= delta (|SA_H| + (1+tau)|SA_SH|), or |SA_H| <= delta (2^l - 1).
    Flips outside it (but inside in_band) are reported separately: they are frames that resemble
    nothing in memory, whose similarities are small while their rounding error is not."""
    if not np.isfinite(h) or not np.isfinite(sh):
        return False
    g = h - (1.0 + tau) * max(sh, 0.0)
    return abs(g) <= delta * (abs(h) + (1.0 + tau) * abs(sh)) or abs(h) <= delta * (2.0 ** l - 1.0)


@dataclass
class ParityReport:
    frames: int = 0
    stage_rows: int = 0
    in_band_flips: int = 0
    flips_outside_narrow_band: int = 0
    label_only_diffs: int = 0
    in_band_frames: int = 0
    near_tie_id_diffs: int = 0
    max_sv_err: float = 0.0
    max_sim_err: float = 0.0         # in units of the tolerance scale
    max_sa_err: float = 0.0
    exit_hist: List[int] = field(default_factory=list)
    tier_hist: List[int] = field(default_factory=lambda: [0, 0, 0])
    hot_sizes: List[int] = field(default_factory=list)


def make_ctx(w: Workload, cents, hot_ids, *, tau=None, tiers=None, score_path=SCORE_AUTO,
             max_batch=None, forgetting=0) -> Smtm:
    cfg = SmtmConfig(n_classes=w.n_classes, dims=w.dims, max_batch=max_batch or w.batch,
                     hot_init=len(hot_ids), hot_min=w.hot_min if w.hot_max else min(2, len(hot_ids)),
                     hot_max=w.hot_max or len(hot_ids), tiers=w.tiers if tiers is None else tiers,
                     tau=w.tau if tau is None else tau, window=w.window, init_count=w.init_count,
                     score_path=score_path, forgetting=forgetting)
    ctx = Smtm(cfg)
    for l, c in enumerate(cents, start=1):
        ctx.memory_load(l, c.numpy())
    ctx.hot_set(np.asarray(hot_ids, np.int32))
    torch.cuda.synchronize()
    return ctx


def make_oracle(w: Workload, cents, hot_ids, *, tau=None, tiers=None, forgetting=0) -> O.Memory:
    return O.Memory([c.numpy() for c in cents], hot_ids, tau=w.tau if tau is None else tau,
                    tiers=w.tiers if tiers is None else tiers, window=w.window,
                    hot_min=w.hot_min if w.hot_max else min(2, len(hot_ids)),
                    hot_max=w.hot_max or len(hot_ids), init_count=w.init_count, forgetting=forgetting)


_pinned = {}


def to_host(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> numpy through a pinned staging buffer kept per shape (several times faster than a
    pageable copy for the GB-sized feature maps).  The array is a view of the buffer: use it before the next
    call with the same shape."""
    key = (tuple(t.shape), t.dtype)
    buf = _pinned.get(key)
    if buf is None:
        if len(_pinned) > 24:
            _pinned.clear()
        buf = _pinned[key] = torch.empty(t.shape, dtype=t.dtype, pin_memory=True)
    buf.copy_(t)
    return buf.numpy()


def _mean_abs(F: torch.Tensor, rows: np.ndarray) -> np.ndarray:
    """mean |F| per (row, channel): the scale of the rounding error of the pooled sum."""
    out = []
    idx = torch.from_numpy(rows.astype(np.int64)).to(F.device)
    step = max(1, (64 << 20) // max(1, F[0].numel()))
    for s in range(0, len(rows), step):
        out.append(F[idx[s:s + step]].float().abs().mean(dim=(2, 3)).cpu())
    return torch.cat(out).numpy().astype(np.float64) if out else np.zeros((0, F.shape[1]))


def check_batch(ctx: Smtm, mem: O.Memory, w: Workload, fmaps: List[torch.Tensor], *, tau: float,
                rtol: float, mode: str = "row_ids", fused: bool = False, check_sims: bool = True,
                report: Optional[ParityReport] = None) -> ParityReport:
    """One batch through both sides.  mode: "row_ids" (full-batch tensors addressed through the
    context's live list) or "dense" (each exit point gets a tensor holding only the live frames,
    and the survivors' maps are gathered for the next block).  fused: False = the three calls,
    "lookup_exit" = smtm_encode + smtm_lookup_exit, True = smtm_stage."""
    rep = report or ParityReport()
    dev = fmaps[0].device
    B = fmaps[0].shape[0]
    n = w.n_classes
    L = len(fmaps)
    ctx.set_tau(tau)
    mem.tau = float(tau)
    ctx.begin_batch(B)
    mem.begin_batch(B)
    live = np.arange(B, dtype=np.int32)
    if not rep.exit_hist:
        rep.exit_hist = [0] * (L + 1)
    acc_scale = np.zeros((B, n), np.float64)            # per frame and class: sum of 2^(l-1) * a so far

    i32 = dict(dtype=torch.int32, device=dev)
    exit_ids = torch.full((B,), -7, **i32); exit_labels = torch.full((B,), -7, **i32)
    exit_tier = torch.full((B,), -7, **i32); live_out = torch.full((B,), -7, **i32)
    n_exit_dev = torch.zeros(1, **i32); n_live_dev = torch.zeros(1, **i32)

    for l in range(1, L + 1):
        F_full = fmaps[l - 1]
        C, H, W = F_full.shape[1:]
        n_live = len(live)
        for t in (exit_ids, exit_labels, exit_tier, live_out):   # entries past the counts must stay untouched
            t.fill_(-7)
        if mode == "dense":
            F_in = F_full[torch.from_numpy(live.astype(np.int64)).to(dev)].contiguous() if n_live else F_full[:1].clone()
            row_ids = None
            rows_host = np.arange(n_live)
        else:
            F_in = F_full
            row_ids = ctx.live_ids()
            rows_host = live
        sv_out = torch.full((B, C), float("nan"), dtype=torch.float32, device=dev)
        top_val = torch.full((B, 2, 2), float("nan"), dtype=torch.float32, device=dev)
        top_id = torch.full((B, 2), -7, **i32)
        sims = torch.full((B, n), float("nan"), dtype=torch.float32, device=dev) if check_sims else None
        # survivors' feature maps are gathered in both modes (through the row list in "row_ids" mode)
        gather = torch.full((max(n_live, 1),) + tuple(F_full.shape[1:]), 0, dtype=F_full.dtype, device=dev)
        row_bytes = C * H * W * F_full.element_size()
        if fused == "lookup_exit":
            # encode, then lookup + exit/compact in one call (no similarities out)
            ctx.encode(l, F_in, row_ids=row_ids, sv_out=sv_out)
            ctx.lookup_exit(l, top_val=top_val, top_id=top_id, exit_ids=exit_ids, exit_labels=exit_labels,
                            exit_tier=exit_tier, n_exit_dev=n_exit_dev, live_ids=live_out,
                            n_live_dev=n_live_dev, fmap_in=F_in if gather is not None else None,
                            row_ids=row_ids, fmap_out=gather, row_bytes=row_bytes)
        elif fused:
            ctx.stage(l, F_in, row_ids=row_ids, exit_ids=exit_ids, exit_labels=exit_labels,
                      exit_tier=exit_tier, n_exit_dev=n_exit_dev, live_ids=live_out,
                      n_live_dev=n_live_dev, fmap_out=gather)
        else:
            ctx.encode(l, F_in, row_ids=row_ids, sv_out=sv_out)
            ctx.lookup(l, top_val=top_val, top_id=top_id, sims_out=sims)
            ctx.exit_compact(l, exit_ids=exit_ids, exit_labels=exit_labels, exit_tier=exit_tier,
                             n_exit_dev=n_exit_dev, live_ids=live_out, n_live_dev=n_live_dev,
                             fmap_in=F_in if gather is not None else None, row_ids=row_ids,
                             fmap_out=gather, row_bytes=row_bytes)
        torch.cuda.synchronize()
        n_live_next, n_exit = ctx.read_counts()
        assert n_live_next + n_exit == n_live
        assert int(n_exit_dev.item()) == n_exit and int(n_live_dev.item()) == n_live_next

        # ---- oracle on the same bits, from the library's live set (teacher forcing)
        F_host = to_host(F_in)
        full = fused in (False, "lookup_exit")           # semantic vectors and top-2 values were captured
        with_sims = check_sims and fused is False
        ref = mem.stage(l, F_host, row_ids=rows_host.astype(np.int32) if mode != "dense" else None,
                        live=live, want_sims=with_sims)

        g_exit = exit_ids[:n_exit].cpu().numpy(); g_lab = exit_labels[:n_exit].cpu().numpy()
        g_tier = exit_tier[:n_exit].cpu().numpy(); g_live = live_out[:n_live_next].cpu().numpy()
        dec_gpu = np.zeros(n_live, np.int32)
        lab_gpu = np.full(n_live, -1, np.int32)
        pos = np.searchsorted(live, g_exit)
        assert np.array_equal(live[pos], g_exit), "exit list holds frames that were not live"
        dec_gpu[pos] = g_tier
        lab_gpu[pos] = g_lab
        # index work: bit-exact
        assert np.all(np.diff(g_exit) > 0) and np.all(np.diff(g_live) > 0)
        assert np.array_equal(g_exit, live[dec_gpu != 0]) and np.array_equal(g_live, live[dec_gpu == 0])
        assert np.all((g_tier == 1) | (g_tier == 2))
        for t in (exit_ids, exit_labels, exit_tier):
            assert bool(t[n_exit:].eq(-7).all()), f"exit {l}: an exit list was written past n_exit"
        assert bool(live_out[n_live_next:].eq(-7).all()), f"exit {l}: the live list was written past n_live"

        if full:
            # ---- semantic vectors
            sv_g = sv_out[:n_live].cpu().numpy().astype(np.float64)
            assert np.isnan(sv_out[n_live:].cpu().numpy()).all(), "rows past the live count were written"
            fin_sv = np.isfinite(ref["SV"])
            assert np.array_equal(np.isfinite(sv_g), fin_sv), f"exit {l}: non-finite semantic vectors differ"
            scale = np.maximum(np.abs(ref["SV"]), _mean_abs(F_in, rows_host))
            with np.errstate(invalid="ignore"):
                err = np.where(fin_sv, np.abs(sv_g - ref["SV"]) / np.maximum(scale, 1e-300), 0.0)
            rep.max_sv_err = max(rep.max_sv_err, float(err.max(initial=0.0)))
            assert err.max(initial=0.0) <= SV_RTOL, f"exit {l}: semantic vector error {err.max():.3e}"
            # ---- similarities
            if with_sims:
                s_g = sims[:n_live].cpu().numpy().astype(np.float64)
                tol = rtol * np.maximum(np.abs(ref["sims"]), ref["sims_scale"])
                e = np.abs(s_g - ref["sims"]) / np.maximum(tol, 1e-300)
                rep.max_sim_err = max(rep.max_sim_err, float(e.max(initial=0.0)))
                assert e.max(initial=0.0) <= 1.0, f"exit {l}: similarity error {e.max():.3f} x tolerance"
            # ---- top-2 values and ids
            tv = top_val[:n_live].cpu().numpy().astype(np.float64)
            ti = top_id[:n_live].cpu().numpy()
            sa_tol = rtol * (2.0 ** l - 1.0)
            rv = ref["top_val"]
            fin = np.isfinite(rv)
            assert np.array_equal(np.isfinite(tv), fin)
            if fin.any():
                d = np.abs(tv[fin] - rv[fin])
                rep.max_sa_err = max(rep.max_sa_err, float(d.max()) / sa_tol)
                assert d.max() <= sa_tol, f"exit {l}: accumulated similarity error {d.max():.3e}"
            id_diff = ti != ref["top_id"]
            for i, t in zip(*np.nonzero(id_diff)):
                assert abs(rv[i, t, 0] - rv[i, t, 1]) <= 2 * sa_tol, f"exit {l}: best class differs away from a tie"
                rep.near_tie_id_diffs += 1
            # ---- the library's decision = exit rule on its own values
            tvf = top_val[:n_live].cpu().numpy()
            for i in range(n_live):
                want = 0
                if rule_fp32(tvf[i, 0, 0], tvf[i, 0, 1], tau):
                    want = 1
                elif mem.tiers == 2 and rule_fp32(tvf[i, 1, 0], tvf[i, 1, 1], tau):
                    want = 2
                assert dec_gpu[i] == want, f"exit {l} slot {i}: decision {dec_gpu[i]} but own values say {want}"
                if want:
                    assert lab_gpu[i] == ti[i, want - 1]

        # ---- decisions and labels against the oracle, with the tolerance band
        rv = ref["top_val"]
        acc_scale[live] += 2.0 ** (l - 1) * dot_scale(ref["SV"], mem.SC[l - 1])
        scale1 = acc_scale[live][:, mem.hot_ids].max(axis=1) if n_live else np.zeros(0)
        scale2 = acc_scale[live].max(axis=1) if n_live else np.zeros(0)
        for i in np.flatnonzero((dec_gpu != ref["decision"]) | (lab_gpu != ref["label"])):
            band = in_band(rv[i, 0, 0], rv[i, 0, 1], tau, l, rtol, scale1[i]) or \
                (mem.tiers == 2 and in_band(rv[i, 1, 0], rv[i, 1, 1], tau, l, rtol, scale2[i]))
            if dec_gpu[i] == ref["decision"][i]:
                # same decision, another label: only where the two best classes of that tier are as good as tied
                t = int(dec_gpu[i]) - 1
                assert abs(rv[i, t, 0] - rv[i, t, 1]) <= 2 * rtol * (2.0 ** l - 1.0), \
                    f"exit {l} frame {live[i]}: label {lab_gpu[i]} vs oracle {ref['label'][i]} away from a tie, top={rv[i]}"
                rep.label_only_diffs += 1
                continue
            assert band, (f"exit {l} frame {live[i]}: decision/label {dec_gpu[i]}/{lab_gpu[i]} vs oracle "
                          f"{ref['decision'][i]}/{ref['label'][i]} outside the tolerance band, top={rv[i]}")
            rep.in_band_flips += 1
            if not (in_narrow_band(rv[i, 0, 0], rv[i, 0, 1], tau, l, rtol) or
                    (mem.tiers == 2 and in_narrow_band(rv[i, 1, 0], rv[i, 1, 1], tau, l, rtol))):
                rep.flips_outside_narrow_band += 1
        for i in range(n_live):
            if in_band(rv[i, 0, 0], rv[i, 0, 1], tau, l, rtol, scale1[i]) or \
                    (mem.tiers == 2 and in_band(rv[i, 1, 0], rv[i, 1, 1], tau, l, rtol, scale2[i])):
                rep.in_band_frames += 1

        # ---- gathered survivors: byte-identical rows
        if gather is not None and n_live_next:
            keep = np.flatnonzero(dec_gpu == 0)
            want_rows = F_in[torch.from_numpy(np.asarray(rows_host)[keep].astype(np.int64)).to(dev)]
            assert torch.equal(gather[:n_live_next].view(torch.int16 if F_full.element_size() == 2 else torch.int32),
                               want_rows.view(torch.int16 if F_full.element_size() == 2 else torch.int32))

        rep.stage_rows += n_live
        rep.exit_hist[l] += n_exit
        rep.tier_hist[1] += int((g_tier == 1).sum()); rep.tier_hist[2] += int((g_tier == 2).sum())
        # teacher forcing: both sides continue from the library's live set and results
        mem.exit_layer[live] = np.where(dec_gpu != 0, l, 0)
        mem.label[live] = lab_gpu
        mem.tier[live] = dec_gpu
        live = g_live.astype(np.int32)
        mem.live = live.copy()

    rep.exit_hist[0] += len(live)
    rep.frames += B
    # per-frame results
    res = [torch.full((B,), -7, **i32) for _ in range(3)]
    ctx.batch_results(*res)
    torch.cuda.synchronize()
    assert np.array_equal(res[0].cpu().numpy(), mem.exit_layer)
    assert np.array_equal(res[1].cpu().numpy(), mem.label)
    assert np.array_equal(res[2].cpu().numpy(), mem.tier)
    return rep


def check_cache_update(ctx: Smtm, mem: O.Memory, label: np.ndarray, stop_layer: np.ndarray,
                       centre_rtol: float = 1e-5, own: bool = False):
    """Memory update on both sides from the same labels; tables / order / size bit-exact,
    centres within centre_rtol of the oracle's (relative to the centre's largest component).
    own: the library takes labels and stop layers from its own per-frame results of the batch (the
    arrays given here are then what the oracle's side of the batch says those results are)."""
    dev = "cuda"
    B = len(label)
    if own:
        ctx.cache_update(None, None, B)
    else:
        lab_d = torch.from_numpy(label.astype(np.int32)).to(dev)
        stop_d = torch.from_numpy(stop_layer.astype(np.int32)).to(dev)
        ctx.cache_update(lab_d, stop_d, B)
    torch.cuda.synchronize()
    upd = mem.cache_update(label, stop_layer)
    ft, ts, hot, k = ctx.tables_export()
    assert np.array_equal(ft, mem.FT) and np.array_equal(ts, mem.TS)
    assert k == len(mem.hot_ids) and np.array_equal(hot, mem.hot_ids)
    worst = 0.0
    for l in range(1, mem.L + 1):
        cg, mg = ctx.memory_export(l)
        assert np.array_equal(mg, mem.m[l - 1])
        ref = mem.SC[l - 1]
        scale = np.abs(ref).max(axis=1, keepdims=True)
        e = (np.abs(cg.astype(np.float64) - ref) / np.maximum(scale, 1e-300)).max()
        worst = max(worst, float(e))
        assert e <= centre_rtol, f"exit {l}: centre error {e:.3e}"
    return upd, worst
