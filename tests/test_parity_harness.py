"""CPU checks of the tolerance helpers the GPU parity tests rely on (tests/parity.py)."""
import numpy as np

from tests import parity as P


def test_dot_scale_is_the_absolute_value_cosine_and_bounds_the_cosine():
    rng = np.random.default_rng(11)
    SV = rng.standard_normal((5, 17)); SC = rng.standard_normal((7, 17))
    a = P.dot_scale(SV, SC)
    for i in range(5):
        for j in range(7):
            want = sum(abs(SV[i, c]) * abs(SC[j, c]) for c in range(17)) / (np.linalg.norm(SV[i]) * np.linalg.norm(SC[j]))
            assert abs(a[i, j] - want) < 1e-12
            cos = float(SV[i] @ SC[j]) / (np.linalg.norm(SV[i]) * np.linalg.norm(SC[j]))
            assert abs(cos) <= a[i, j] + 1e-12 <= 1.0 + 1e-12
    SV[2] = 0.0                                           # a zero vector has no scale: its similarities are 0 by definition
    assert np.all(P.dot_scale(SV, SC)[2] == 0.0)


def test_in_band_is_the_propagated_similarity_tolerance():
    tau, l, d = 4.0, 2, 2e-3
    # on the threshold: SA_H = (1 + tau) * SA_SH
    assert P.in_band(0.5, 0.1, tau, l, d, scale=1.0)
    # the two sides may move by d * scale * (2 + tau) against each other, not more
    edge = d * 1.0 * (2.0 + tau)
    assert P.in_band(0.5 + 0.99 * edge, 0.1, tau, l, d, scale=1.0)
    assert not P.in_band(0.5 + 1.01 * edge, 0.1, tau, l, d, scale=1.0)
    assert not P.in_band(0.5 - 1.01 * edge, 0.1, tau, l, d, scale=1.0)
    # a smaller accumulated scale narrows the band, the default is the bound 2^l - 1
    assert not P.in_band(0.5 + 0.99 * edge, 0.1, tau, l, d, scale=0.5)
    assert P.in_band(0.5 + 2.9 * edge, 0.1, tau, l, d)
    # a runner-up that is not positive counts as 0 on the right-hand side; the sign of SA_H is uncertain near 0
    assert P.in_band(0.5 * edge, -0.3, tau, l, d, scale=1.0)
    assert P.in_band(-0.9 * d, -0.3, tau, l, d, scale=1.0)
    assert not P.in_band(-3.0 * edge, -0.3, tau, l, d, scale=1.0)
    assert not P.in_band(float("inf"), 0.1, tau, l, d)


def test_rule_fp32_is_the_exit_rule_in_single_precision():
    assert P.rule_fp32(3.0, 1.0, 1.9) and not P.rule_fp32(3.0, 1.0, 2.0)      # AC = 2: strict >
    assert P.rule_fp32(0.2, -0.1, 100.0)                                     # runner-up not positive
    assert not P.rule_fp32(0.0, -0.1, 0.0) and not P.rule_fp32(-0.1, -0.2, 0.0)


def test_narrow_band_is_relative_to_the_frames_own_values():
    tau, l, d = 4.0, 2, 2e-3
    h, sh = 0.5, 0.1                                        # on the threshold
    assert P.in_narrow_band(h, sh, tau, l, d)
    edge = d * (abs(h) + (1 + tau) * abs(sh))
    assert P.in_narrow_band(h + 0.9 * edge, sh, tau, l, d) and not P.in_narrow_band(h + 1.2 * edge, sh, tau, l, d)
    # small accumulated similarities: the narrow band shrinks with them, the propagated one does not
    assert not P.in_narrow_band(0.012, 0.001, tau, l, d) and P.in_band(0.012, 0.001, tau, l, d, scale=2.0)
    assert P.in_narrow_band(0.9 * d * 3.0, -0.2, tau, l, d)  # sign of SA_H uncertain
    assert not P.in_narrow_band(float("nan"), 0.1, tau, l, d)
