"""The memory in the loop of a real convolutional trunk (Sec. 4 workflow): a small run of the
end-to-end script.  Checks the plumbing (channels-last encode, gather into the next stage's input,
live counts driving the batch shapes), not speed."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_trunk_with_memory_in_the_loop():
    from paper_2112_02644_amd import end_to_end

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
