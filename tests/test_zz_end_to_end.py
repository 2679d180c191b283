"""The memory in the loop of a real convolutional trunk (Sec. 4 workflow): a small run of the
end-to-end script (plumbing: channels-last encode, gather into the next stage's input, live counts
driving the batch shapes), and one batch whose every stage is also given to the CPU oracle."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_trunk_with_memory_in_the_loop():
    import end_to_end

    out = end_to_end.run(batch=96, taus=[3.0e38, 0.02, 0.002], n_classes=40, hot=8, reps=1, samples=2,
                         bucket=32)
    rows = out["rows"]
    assert [r["tau"] for r in rows] == [pytest.approx(3.0e38), 0.02, 0.002]
    # nothing passes an unreachable threshold; a lower threshold never releases fewer frames at exit point 1
    assert rows[0]["live_after_exit"] == [96, 96, 96, 96]
    assert sum(rows[0]["exit_ratio"]) == 0.0
    assert rows[1]["exit_ratio"][0] <= rows[2]["exit_ratio"][0]
    assert sum(rows[2]["exit_ratio"]) > 0.5
    for r in rows:
        live = r["live_after_exit"]
        assert all(a >= b for a, b in zip(live, live[1:]))
        released = sum(r["exit_ratio"])
        assert abs(released - (1.0 - live[-1] / 96)) < 1e-6
    # the warm-up centres identify the class of every in-memory frame at every exit point
    for p in out["confidence_profile"]:
        assert p["global_top1_right"] == 1.0
    assert np.isfinite(out["no_memory_ms"]) and out["no_memory_ms"] > 0


def test_every_stage_of_the_trunk_against_the_oracle():
    # The trunk's own stage outputs (PyTorch convolutions on the compacted batch) go to the library as
    # channels-last tensors and, as the same bits in NCHW order, to the oracle: semantic vectors, top-2 values,
    # released ids, labels and tiers, survivors and gathered rows at every exit point, with the tolerance band
    # of the fp16 scoring path.  The oracle's centres are its own class means over the warm-up frames.
    import dataclasses

    import torch

    import end_to_end as E
    import parity as P
    from oracle import smtm_oracle as O
    from paper_2112_02644_amd import Smtm, SmtmConfig
    from workloads import configs, streams

    dev = "cuda:0"
    B, n, hot, L = 96, 40, 8, 4
    rtol = 2e-3
    dims = tuple(s[1] for s in E.STAGES)
    mods = E.build_trunk(dev, n)
    images = E.Images(n, dev)
    ctx = Smtm(SmtmConfig(n_classes=n, dims=dims, max_batch=B, hot_init=hot, hot_min=hot, hot_max=hot, tiers=2,
                          tau=0.01, window=1024, init_count=1))
    i32 = dict(dtype=torch.int32, device=dev)

    # ---- warm-up on both sides from the same stage outputs
    rng = np.random.Generator(np.random.Philox(E.SEED + 3))
    order = np.concatenate([rng.permutation(n) for _ in range(2)]).astype(np.int32)
    sv_all = [[] for _ in range(L)]
    ctx.warmup_begin()
    for lo in range(0, order.shape[0], B):
        lab = order[lo: lo + B]
        x = mods[0](images.batch(lab))
        ctx.begin_batch(lab.shape[0])
        for l in range(1, L + 1):
            x = mods[l](x)
            ctx.encode_nhwc(l, E.nhwc(x))
            sv_all[l - 1].append(O.encode(P.to_host(x.contiguous())))        # the same values in NCHW order
        ctx.warmup_batch(torch.from_numpy(lab).to(dev), lab.shape[0])
    torch.cuda.synchronize()
    cents = []
    for l in range(L):
        SC, m = O.warmup_centres(np.concatenate(sv_all[l]), order, n)
        cents.append(SC)
        cg, mg = ctx.memory_export(l + 1)
        assert np.array_equal(mg, m)
        assert (np.abs(cg - SC) / np.abs(SC).max(axis=1, keepdims=True)).max() <= 1e-5

    # ---- one batch through the trunk with the memory in the loop
    w = dataclasses.replace(configs.RESNET50, n_classes=n, hot=hot, batch=B)
    ls = streams.labels(w, B)
    ctx.hot_set(ls.initial_hot)
    img = images.batch(ls.label.astype(np.int32))
    shapes = [(56, 56, 256), (28, 28, 512), (14, 14, 1024), (7, 7, 2048)]
    bufs = [torch.zeros((B,) + s, dtype=torch.float16, device=dev) for s in shapes]
    flips = released = 0
    for tau in (0.0032, 0.0015):                          # between the confidences of fast-memory frames and of the others
        ctx.set_tau(tau)
        mem = O.Memory(cents, ls.initial_hot, tau=tau, tiers=2, window=1024, hot_min=hot, hot_max=hot, init_count=1)
        for l in range(L):
            mem.m[l][:] = 2                                   # two warm-up samples per class
        ctx.begin_batch(B); mem.begin_batch(B)
        live = np.arange(B, dtype=np.int32)
        x = mods[0](img)
        for l in range(1, L + 1):
            x = mods[l](x)
            n_in = len(live)
            xv = E.nhwc(x)
            lists = [torch.full((B,), -7, **i32) for _ in range(4)] + [torch.zeros(1, **i32), torch.zeros(1, **i32)]
            sv = torch.full((B, dims[l - 1]), float("nan"), device=dev)
            tv = torch.full((B, 2, 2), float("nan"), device=dev); ti = torch.full((B, 2), -7, **i32)
            ctx.encode_nhwc(l, xv, sv_out=sv)
            ctx.lookup_exit(l, top_val=tv, top_id=ti, exit_ids=lists[0], exit_labels=lists[1], exit_tier=lists[2],
                            live_ids=lists[3], n_exit_dev=lists[4], n_live_dev=lists[5], fmap_in=xv,
                            fmap_out=bufs[l - 1], row_bytes=xv[0].numel() * 2)
            n_live, n_exit = ctx.read_counts()
            assert n_live + n_exit == n_in == int(lists[4].item()) + int(lists[5].item())
            ref = mem.stage(l, P.to_host(x[:n_in].contiguous()), live=live)
            # semantic vectors and accumulated similarities
            got = sv[:n_in].cpu().numpy().astype(np.float64)
            scale = np.maximum(np.abs(ref["SV"]), x[:n_in].float().abs().mean(dim=(2, 3)).cpu().numpy())
            assert (np.abs(got - ref["SV"]) / np.maximum(scale, 1e-300)).max() <= P.SV_RTOL
            assert np.abs(tv[:n_in].cpu().numpy() - ref["top_val"]).max() <= rtol * (2.0 ** l - 1.0)
            # released frames, labels, tiers, survivors: identical outside the tolerance band
            g_exit = lists[0][:n_exit].cpu().numpy(); g_lab = lists[1][:n_exit].cpu().numpy()
            g_tier = lists[2][:n_exit].cpu().numpy(); g_live = lists[3][:n_live].cpu().numpy()
            assert bool(lists[0][n_exit:].eq(-7).all()) and bool(lists[3][n_live:].eq(-7).all())
            dec = np.zeros(n_in, np.int32); lab = np.full(n_in, -1, np.int32)
            pos = np.searchsorted(live, g_exit)
            assert np.array_equal(live[pos], g_exit)
            dec[pos] = g_tier; lab[pos] = g_lab
            assert np.array_equal(g_live, live[dec == 0])
            rv = ref["top_val"]
            for i in np.flatnonzero((dec != ref["decision"]) | (lab != ref["label"])):
                if dec[i] == ref["decision"][i]:
                    t = int(dec[i]) - 1
                    assert abs(rv[i, t, 0] - rv[i, t, 1]) <= 2 * rtol * (2.0 ** l - 1.0)
                    continue
                assert P.in_band(rv[i, 0, 0], rv[i, 0, 1], tau, l, rtol) or P.in_band(rv[i, 1, 0], rv[i, 1, 1], tau, l, rtol), \
                    f"tau {tau} exit {l} frame {live[i]}: {dec[i]}/{lab[i]} vs oracle {ref['decision'][i]}/{ref['label'][i]}"
                flips += 1
            released += n_exit
            # the rows handed to the next stage are the survivors' rows of this stage's output
            keep = torch.from_numpy(np.flatnonzero(dec == 0).astype(np.int64)).to(dev)
            assert torch.equal(bufs[l - 1][:n_live].view(torch.int16), xv[keep].contiguous().view(torch.int16))
            # teacher forcing, then the next stage runs on the compacted batch
            mem.exit_layer[live] = np.where(dec != 0, l, 0); mem.label[live] = lab; mem.tier[live] = dec
            live = g_live.astype(np.int32); mem.live = live.copy()
            if n_live == 0:
                break
            x = bufs[l - 1][:n_live].permute(0, 3, 1, 2)
        print(f"tau {tau}: released {released}, threshold flips so far {flips}", flush=True)
    assert released > 0
    ctx.close()
