"""smtm_cache_update_static (the memory update for callers that cannot allocate: its scratch is a
device array inside the library) against smtm_cache_update, through the C ABI, on two calls in a
row, the second with a smaller batch.  Tables, order and size are integer work (bit-exact); the
centres come out of the same kernels in the same order, so they are bit-exact too."""
import dataclasses

import numpy as np
import pytest
import torch

from paper_2112_02644_amd import Smtm, SmtmConfig, SmtmError
from workloads import configs, streams

import parity as P

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _state(ctx, L):
    torch.cuda.synchronize()
    ft, ts, hot, k = ctx.tables_export()
    cm = [ctx.memory_export(l) for l in range(1, L + 1)]
    return ft, ts, hot, k, cm


def test_cache_update_static_equals_cache_update_on_two_calls_in_a_row():
    print("cache_update_static vs cache_update", flush=True)
    w = dataclasses.replace(configs.ADAPTIVE, batch=384, exits=((32, 14, 14), (48, 7, 7)), n_classes=300, hot=12,
                            hot_min=4, hot_max=200, window=128, total_frames=384 + 200, drift_every=0)
    cents = streams.centroids(w)
    ls = streams.labels(w)
    ref = P.make_ctx(w, cents, ls.initial_hot)           # existing entry point
    new = P.make_ctx(w, cents, ls.initial_hot)           # the one that allocates nothing
    for b, Bi in enumerate((384, 200)):                  # the second call is smaller
        fm = streams.batch_feature_maps(w, cents, ls, b, DEV)
        assert fm[0].shape[0] == Bi
        truth = ls.label[b * 384: b * 384 + Bi]
        outs = []
        for ctx in (ref, new):
            ctx.begin_batch(Bi)
            for l in range(1, w.n_exits + 1):
                ctx.stage(l, fm[l - 1], row_ids=ctx.live_ids())
            res = [torch.zeros(Bi, dtype=torch.int32, device=DEV) for _ in range(3)]
            ctx.batch_results(*res)
            torch.cuda.synchronize()
            layer = res[0].cpu().numpy()
            label = np.where(layer > 0, res[1].cpu().numpy(), truth).astype(np.int32)
            lab_d = torch.from_numpy(label).to(DEV)
            if ctx is ref:
                ctx.cache_update(lab_d, res[0], Bi)
            else:
                ctx.cache_update_static(lab_d, res[0], Bi)
            outs.append(_state(ctx, w.n_exits))
        a, c = outs
        assert a[0].sum() > 0
        assert np.array_equal(a[0], c[0]) and np.array_equal(a[1], c[1]), f"call {b}: FT / TS differ"
        assert a[3] == c[3] and np.array_equal(a[2], c[2]), f"call {b}: fast-memory set or size differs"
        for (ca, ma), (cc, mc) in zip(a[4], c[4]):
            assert np.array_equal(ma, mc), f"call {b}: update counts differ"
            assert np.array_equal(ca.view(np.int32), cc.view(np.int32)), f"call {b}: centres differ"
    # the batch's own results (NULL lists) go through the same path
    for ctx in (ref, new):
        ctx.begin_batch(64)
        for l in range(1, w.n_exits + 1):
            ctx.stage(l, fm[l - 1][:64].contiguous())
    ref.cache_update(None, None, 64)
    new.cache_update_static(None, None, 64)
    a, c = _state(ref, w.n_exits), _state(new, w.n_exits)
    assert np.array_equal(a[0], c[0]) and np.array_equal(a[1], c[1]) and np.array_equal(a[2], c[2]) and a[3] == c[3]
    ref.close(); new.close()


def test_cache_update_static_rejects_more_classes_than_its_scratch_holds():
    ctx = Smtm(SmtmConfig(n_classes=4097, dims=[8], max_batch=4, hot_init=2))
    ctx.begin_batch(4)
    with pytest.raises(SmtmError) as e:
        ctx.cache_update_static(None, None, 4)
    assert e.value.code == 4 and "4096" in str(e.value)
    ctx.cache_update(None, None, 4)                      # the allocating entry point still takes it
    torch.cuda.synchronize()
    ctx.close()
    ok = Smtm(SmtmConfig(n_classes=4096, dims=[8], max_batch=4, hot_init=2))
    ok.begin_batch(4)
    ok.cache_update_static(None, None, 4)
    torch.cuda.synchronize()
    ok.close()
