"""Pins for the CPU oracle: closed forms, library routines, invariants, brute force.

Each test fixes the oracle against something other than itself, chosen so that a dropped
term, a wrong sign or index, or a transposed operand fails at least one of them.
Equation and section numbers refer to arXiv 2112.02644.
"""
import itertools
import math
from fractions import Fraction
from pathlib import Path

import numpy as np
import pytest

from oracle import smtm_oracle as O

GOLDEN = Path(__file__).resolve().parent / "golden"
rng = np.random.default_rng(7)


# ------------------------------------------------------------------ binary16 decoding

def test_half_to_double_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([O.half_to_double(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


# ------------------------------------------------------------------ encode (Sec. 4.1, GAP)

@pytest.mark.parametrize("dtype", [np.float16, np.float32])
def test_encode_constant_map_is_exact(dtype):
    F = np.empty((3, 5, 7, 7), dtype)
    vals = np.array([0.5, -1.25, 3.0, 0.0, 1024.0], dtype)
    F[:] = vals[None, :, None, None]
    SV = O.encode(F)
    assert np.array_equal(SV, np.broadcast_to(vals.astype(np.float64), (3, 5)))


@pytest.mark.parametrize("dtype,shape", [(np.float16, (4, 6, 7, 7)), (np.float16, (3, 5, 14, 14)),
                                          (np.float32, (2, 9, 28, 28)), (np.float16, (2, 3, 56, 56)),
                                          (np.float32, (5, 2, 3, 5))])
def test_encode_equals_numpy_mean(dtype, shape):
    F = rng.standard_normal(shape).astype(dtype)
    want = F.astype(np.float64).mean(axis=(2, 3))
    assert np.allclose(O.encode(F), want, rtol=1e-13, atol=1e-15)


def test_encode_is_mean_not_sum_and_divides_by_hw():
    F = np.ones((1, 1, 4, 5), np.float32) * 2.0
    F[0, 0, 0, 0] = 22.0            # sum = 2*19 + 22 = 60, mean = 3
    assert O.encode(F)[0, 0] == 3.0


def test_encode_permutation_of_positions_invariant():
    F = rng.standard_normal((2, 4, 6, 6)).astype(np.float32)
    perm = rng.permutation(36)
    G = F.reshape(2, 4, 36)[:, :, perm].reshape(2, 4, 6, 6).copy()
    assert np.allclose(O.encode(F), O.encode(G), rtol=1e-14, atol=1e-16)


def test_encode_channels_and_frames_not_mixed():
    # one hot element: only (frame 1, channel 2) may be non-zero
    F = np.zeros((3, 4, 5, 5), np.float16)
    F[1, 2, 3, 4] = 25.0
    SV = O.encode(F)
    want = np.zeros((3, 4)); want[1, 2] = 1.0
    assert np.array_equal(SV, want)


def test_encode_linear():
    F = rng.standard_normal((2, 3, 7, 7)).astype(np.float32)
    G = rng.standard_normal((2, 3, 7, 7)).astype(np.float32)
    H = (2.0 * F.astype(np.float64) - 0.5 * G.astype(np.float64)).astype(np.float32)
    # exact inputs: use values that stay exact in float32
    F = np.round(F * 64) / 64; G = np.round(G * 64) / 64
    H = (2.0 * F - 0.5 * G).astype(np.float32)
    assert np.allclose(O.encode(H), 2.0 * O.encode(F) - 0.5 * O.encode(G), rtol=1e-13, atol=1e-15)


def test_encode_row_ids_select_rows():
    F = rng.standard_normal((6, 3, 4, 4)).astype(np.float16)
    ids = np.array([4, 0, 5], np.int32)
    assert np.array_equal(O.encode(F, row_ids=ids), O.encode(F)[ids])
    assert O.encode(F, n_live=0).shape == (0, 3)


# ------------------------------------------------------------------ cosine (Eq. 1)

def test_cosine_self_is_one_and_opposite_minus_one():
    for C in (1, 3, 64, 2048):
        v = rng.standard_normal(C)
        assert abs(O.cosine(v, v) - 1.0) <= 4e-16
        assert abs(O.cosine(v, -v) + 1.0) <= 4e-16


def test_cosine_orthogonal_and_known_angle():
    e = np.eye(4)
    assert O.cosine(e[0], e[1]) == 0.0
    assert abs(O.cosine(np.array([1.0, 0.0]), np.array([1.0, 1.0])) - math.sqrt(0.5)) < 1e-15
    assert abs(O.cosine(np.array([3.0, 4.0]), np.array([4.0, 3.0])) - 24.0 / 25.0) < 1e-15


def test_cosine_scale_invariant_and_bounded():
    for _ in range(20):
        v = rng.standard_normal(37); c = rng.standard_normal(37)
        s = O.cosine(v, c)
        assert -1.0 <= s <= 1.0
        assert abs(O.cosine(3.5 * v, c) - s) < 1e-15
        assert abs(O.cosine(v, 0.01 * c) - s) < 1e-15
        assert abs(O.cosine(-2.0 * v, c) + s) < 1e-15
        assert O.cosine(v, c) == O.cosine(c, v)


def test_cosine_equals_normalised_numpy_matmul():
    V = rng.standard_normal((5, 48)); Cn = rng.standard_normal((7, 48))
    want = (V / np.linalg.norm(V, axis=1, keepdims=True)) @ (Cn / np.linalg.norm(Cn, axis=1, keepdims=True)).T
    got = np.array([[O.cosine(v, c) for c in Cn] for v in V])
    assert np.allclose(got, want, rtol=0, atol=1e-15)


def test_cosine_zero_or_nonfinite_vector_gives_zero():
    z = np.zeros(5); v = np.arange(5.0)
    assert O.cosine(z, v) == 0.0 and O.cosine(v, z) == 0.0
    w = v.copy(); w[2] = np.inf
    assert O.cosine(w, v) == 0.0
    w[2] = np.nan
    assert O.cosine(w, v) == 0.0


# ------------------------------------------------------------------ tolerance scale of Eq. 1

def test_abs_scale_is_the_sum_of_absolute_products_over_the_norms():
    # brute force with Python floats, one term at a time
    for C in (1, 2, 7, 33):
        for _ in range(6):
            v = rng.standard_normal(C); c = rng.standard_normal(C)
            num = 0.0
            for k in range(C):
                num += abs(float(v[k])) * abs(float(c[k]))
            want = num / (math.sqrt(sum(float(x) ** 2 for x in v)) * math.sqrt(sum(float(x) ** 2 for x in c)))
            assert abs(O.cosine_abs_scale(v, c) - want) <= 1e-15


def test_abs_scale_hand_values():
    # (3,-4).(4,3) = 0 but |3*4| + |-4*3| = 24 over norms 5*5
    assert abs(O.cosine_abs_scale(np.array([3.0, -4.0]), np.array([4.0, 3.0])) - 24.0 / 25.0) < 1e-15
    assert O.cosine(np.array([3.0, -4.0]), np.array([4.0, 3.0])) == 0.0
    # (1,0) against (1,1): 1 / sqrt(2); an orthogonal basis pair has no overlapping terms at all
    assert abs(O.cosine_abs_scale(np.array([1.0, 0.0]), np.array([1.0, 1.0])) - math.sqrt(0.5)) < 1e-15
    assert O.cosine_abs_scale(np.array([1.0, 0.0]), np.array([0.0, 1.0])) == 0.0


def test_abs_scale_bounds_the_cosine_and_is_at_most_one():
    for _ in range(50):
        C = int(rng.integers(1, 40))
        v = rng.standard_normal(C); c = rng.standard_normal(C)
        a = O.cosine_abs_scale(v, c)
        assert abs(O.cosine(v, c)) <= a + 1e-15 and a <= 1.0 + 1e-15      # triangle inequality, Cauchy-Schwarz
        # invariant to the signs and to positive scaling of either argument, symmetric
        assert abs(O.cosine_abs_scale(-v, 3.0 * c) - a) < 1e-15
        assert abs(O.cosine_abs_scale(np.abs(v), c) - a) < 1e-15
        assert O.cosine_abs_scale(c, v) == a


def test_abs_scale_is_one_for_parallel_vectors_and_the_cosine_for_non_negative_ones():
    v = np.abs(rng.standard_normal(19)) + 0.1
    assert abs(O.cosine_abs_scale(v, 2.5 * v) - 1.0) <= 4e-16
    assert abs(O.cosine_abs_scale(v, -v) - 1.0) <= 4e-16                  # the cosine is -1 there, the scale +1
    c = np.abs(rng.standard_normal(19))
    assert abs(O.cosine_abs_scale(v, c) - O.cosine(v, c)) <= 1e-15


def test_abs_scale_of_a_zero_or_nonfinite_vector_is_zero():
    z = np.zeros(5); v = np.arange(1.0, 6.0)
    assert O.cosine_abs_scale(z, v) == 0.0 and O.cosine_abs_scale(v, z) == 0.0
    w = v.copy(); w[2] = np.inf
    assert O.cosine_abs_scale(w, v) == 0.0


def test_lookup_reports_the_abs_scale_of_every_similarity():
    # the scale array that the GPU parity tests divide by comes out of orc_lookup
    SV = rng.standard_normal((4, 9)); SC = rng.standard_normal((6, 9))
    SA = np.zeros((4, 6))
    out = O.lookup(SV, SC, 1, np.arange(4, dtype=np.int32), SA, np.array([0, 1], np.int32), 2, 1.0, want_sims=True)
    want = (np.abs(SV) @ np.abs(SC).T) / (np.linalg.norm(SV, axis=1)[:, None] * np.linalg.norm(SC, axis=1)[None, :])
    assert np.allclose(out["sims_scale"], want, rtol=0, atol=1e-15)


def test_lookup_cached_vector_scores_one_against_itself():
    # a frame whose semantic vector IS centre j scores cosine 1 with j.
    n, C = 12, 64
    SC = rng.standard_normal((n, C))
    SA = np.zeros((n, n))
    out = O.lookup(SC.copy(), SC, 1, np.arange(n, dtype=np.int32), SA, np.arange(n, dtype=np.int32), 2, 0.5,
                   want_sims=True)
    assert np.allclose(np.diag(out["sims"]), 1.0, rtol=0, atol=4e-16)
    assert np.array_equal(out["top_id"][:, 1], np.arange(n))


# ------------------------------------------------------------------ SA (Eq. 3) and weights

def test_weights_are_powers_of_two_and_identity_of_sec5():
    assert [O.weight(l) for l in range(1, 9)] == [1, 2, 4, 8, 16, 32, 64, 128]
    for l in range(1, 9):
        assert sum(O.weight(l0) for l0 in range(1, l)) == O.weight(l) - 1


def _run_layers(sims_per_layer, hot_ids, tiers, tau):
    """Drive orc_lookup with prescribed similarities: class j's centre is basis vector e_j and
    the frame's semantic vector is built so its cosine with e_j is the wanted value."""
    n = len(sims_per_layer[0])
    SA = np.zeros((1, n))
    out = None
    for l, s in enumerate(sims_per_layer, start=1):
        s = np.asarray(s, float)
        rest = 1.0 - float(np.sum(s * s))
        assert rest >= -1e-12
        v = np.concatenate([s, [math.sqrt(max(rest, 0.0))]])       # unit vector in R^(n+1)
        SC = np.eye(n, n + 1)
        out = O.lookup(v[None, :], SC, l, np.zeros(1, np.int32), SA, np.asarray(hot_ids, np.int32), tiers, tau,
                       want_sims=True)
        assert np.allclose(out["sims"][0], s, atol=1e-15)
    return SA[0].copy(), out


def test_sa_all_ones_gives_two_pow_l_minus_one():
    # similarities of exactly 1 for one class across l exit points: SA = 2^l - 1
    for L in range(1, 7):
        SA, _ = _run_layers([[1.0, 0.0]] * L, [0, 1], 2, 0.0)
        assert SA[0] == 2 ** L - 1 and SA[1] == 0.0


def test_sa_newest_layer_outweighs_all_earlier_by_one():
    for L in range(2, 7):
        sims = [[-1.0, 0.0]] * (L - 1) + [[1.0, 0.0]]
        SA, _ = _run_layers(sims, [0, 1], 2, 0.0)
        assert SA[0] == 1.0


def test_sa_bound_and_second_formula_concatenated_vectors():
    # SA_j^l = < [2^0 v1^; 2^1 v2^; ...], [c1_j^; c2_j^; ...] >  with unit-normalised pieces.
    n, dims = 9, [8, 16, 5]
    cents = [rng.standard_normal((n, c)) for c in dims]
    svs = [rng.standard_normal((1, c)) for c in dims]
    SA = np.zeros((1, n))
    for l, (sv, sc) in enumerate(zip(svs, cents), start=1):
        O.lookup(sv, sc, l, np.zeros(1, np.int32), SA, np.arange(n, dtype=np.int32), 2, 1.0)
        assert np.all(np.abs(SA) <= 2 ** l - 1 + 1e-12)
    vcat = np.concatenate([2.0 ** l * sv[0] / np.linalg.norm(sv[0]) for l, sv in enumerate(svs)])
    ccat = np.concatenate([sc / np.linalg.norm(sc, axis=1, keepdims=True) for sc in cents], axis=1)
    assert np.allclose(SA[0], ccat @ vcat, rtol=0, atol=1e-14)


def test_sa_rows_follow_original_frame_ids():
    n, C = 5, 6
    SC = rng.standard_normal((n, C)); SV = rng.standard_normal((2, C))
    SA = np.zeros((4, n))
    out = O.lookup(SV, SC, 2, np.array([3, 1], np.int32), SA, np.arange(n, dtype=np.int32), 2, 1.0, want_sims=True)
    assert np.all(SA[0] == 0) and np.all(SA[2] == 0)
    assert np.allclose(SA[3], 2.0 * out["sims"][0]) and np.allclose(SA[1], 2.0 * out["sims"][1])


# ------------------------------------------------------------------ top-2, AC (Eq. 4), predicate

def test_golden_hand_cases_eq3_eq4():
    rows = [ln for ln in (GOLDEN / "eq3_eq4_hand_cases.txt").read_text().splitlines()
            if ln.strip() and not ln.startswith("#")]
    assert len(rows) >= 6
    for ln in rows:
        sims_s, sa_s, ac_s, tau_s, ex_s, lab_s = [x.strip() for x in ln.split(";")]
        layers = [[float(x) for x in g.split(",")] for g in sims_s.split("|")]
        want_sa = np.array([float(x) for x in sa_s.split(",")])
        # the equations are linear in s: feed them through Eq. 3 by hand, then orc_top2/predicate
        SA = np.zeros(3)
        for l, s in enumerate(layers, start=1):
            SA += O.weight(l) * np.array(s)
        assert np.allclose(SA, want_sa, atol=1e-15)
        h, idx, sh = O.top2(SA)
        assert idx == int(lab_s)
        assert abs(O.accumulated_confidence(h, sh) - float(ac_s)) < 1e-12
        assert O.exit_predicate(h, sh, float(tau_s)) == bool(int(ex_s))


def test_golden_cases_through_lookup_when_similarities_are_cosines():
    # rows of the fixture whose numbers are valid cosines also go through orc_lookup end to end
    sims = [[0.5, 0.25, 0.0], [0.25, 0.5, 0.125]]
    SA, out = _run_layers(sims, [0, 1, 2], 1, 0.2)
    assert np.allclose(SA, [1.0, 1.25, 0.25], atol=1e-15)
    assert out["decision"][0] == 1 and out["label"][0] == 1
    SA, out = _run_layers(sims, [0, 1, 2], 1, 0.25)       # AC = 0.25 exactly (up to rounding): not above
    assert abs((SA[1] - SA[0]) / SA[0] - 0.25) < 1e-15


def test_top2_matches_full_sort_brute_force():
    for trial in range(200):
        n = int(rng.integers(2, 12))
        SA = rng.integers(-3, 4, size=n).astype(float)     # many ties on purpose
        k = int(rng.integers(2, n + 1))
        ids = rng.permutation(n)[:k].astype(np.int32)
        order = sorted(ids.tolist(), key=lambda j: (-SA[j], j))
        h, idx, sh = O.top2(SA, ids)
        assert idx == order[0] and h == SA[order[0]] and sh == SA[order[1]]
        # independent of the order the set is stored in
        assert O.top2(SA, ids[::-1].copy()) == (h, idx, sh)


def test_top2_degenerate_sets():
    h, idx, sh = O.top2(np.array([0.3, 0.1]), np.array([1], np.int32))
    assert (h, idx) == (0.1, 1) and sh == -np.inf
    assert not O.exit_predicate(h, sh, 0.0)                 # fewer than two entries never exit
    h, idx, sh = O.top2(np.array([0.3]), np.zeros(0, np.int32))
    assert idx == -1 and not O.exit_predicate(h, sh, 0.0)


def test_predicate_equals_eq4_division_when_runner_up_positive():
    for _ in range(2000):
        sh = float(rng.uniform(1e-3, 5.0)); h = sh + float(rng.uniform(0.0, 10.0))
        tau = float(rng.choice([0.0, 0.25, 1.0, 4.0, 16.0]))
        ac = (h - sh) / sh
        if abs(ac - tau) < 1e-9:
            continue
        assert O.exit_predicate(h, sh, tau) == (ac > tau)


def test_predicate_sign_cases_and_strictness():
    assert O.exit_predicate(0.99, -0.01, 16.0)        # runner-up not positively correlated: exits
    assert O.exit_predicate(0.99, 0.0, 16.0)
    assert not O.exit_predicate(0.0, -0.5, 0.0)       # nothing matches: never exits
    assert not O.exit_predicate(-0.1, -0.5, 0.0)
    assert not O.exit_predicate(1.0, 1.0, 0.0)        # exact tie: AC = 0, not > 0
    assert not O.exit_predicate(3.0, 1.0, 2.0)        # AC == tau: strict '>' does not exit
    assert O.exit_predicate(3.0, 1.0, 1.999)
    assert O.accumulated_confidence(3.0, 1.0) == 2.0
    assert O.accumulated_confidence(0.5, -0.1) == np.inf
    assert O.accumulated_confidence(-0.5, -0.6) == -np.inf


def test_duplicate_best_centre_never_exits_and_label_is_smaller_id():
    n, C = 6, 16
    SC = rng.standard_normal((n, C))
    SC[4] = SC[1]                                     # classes 1 and 4 identical
    v = SC[1] + 0.01 * rng.standard_normal(C)
    SA = np.zeros((1, n))
    out = O.lookup(v[None], SC, 1, np.zeros(1, np.int32), SA, np.arange(n, dtype=np.int32), 2, 0.0)
    assert out["decision"][0] == 0
    assert out["top_id"][0, 0] == 1 and out["top_val"][0, 0, 0] == out["top_val"][0, 0, 1]


def test_class_permutation_equivariance():
    n, C, B = 8, 12, 30
    SC = rng.standard_normal((n, C)); SV = rng.standard_normal((B, C))
    perm = rng.permutation(n)
    hot = np.array([0, 2, 5, 6], np.int32)
    SA1 = np.zeros((B, n)); SA2 = np.zeros((B, n))
    a = O.lookup(SV, SC, 1, np.arange(B, dtype=np.int32), SA1, hot, 2, 0.5)
    SCp = np.empty_like(SC); SCp[perm] = SC              # class j becomes class perm[j]
    b = O.lookup(SV, SCp, 1, np.arange(B, dtype=np.int32), SA2, perm[hot].astype(np.int32), 2, 0.5)
    assert np.array_equal(a["decision"], b["decision"])
    lab = a["label"].copy(); lab[lab >= 0] = perm[lab[lab >= 0]]
    assert np.array_equal(lab, b["label"])


def test_exit_set_shrinks_as_tau_grows_at_first_exit():
    n, C, B = 10, 16, 200
    SC = rng.standard_normal((n, C)); SV = SC[rng.integers(0, n, B)] + 0.8 * rng.standard_normal((B, C))
    prev = None
    for tau in (0.0, 0.25, 1.0, 4.0, 16.0):
        SA = np.zeros((B, n))
        d = O.lookup(SV, SC, 1, np.arange(B, dtype=np.int32), SA, np.arange(4, dtype=np.int32), 2, tau)["decision"] != 0
        if prev is not None:
            assert np.all(prev | ~d)                   # d subset of prev
        prev = d
    assert prev.sum() < B


def test_tiers_one_is_tier_two_restricted_and_full_hot_never_reaches_tier_two():
    n, C, B = 10, 16, 300
    SC = rng.standard_normal((n, C)); SV = SC[rng.integers(0, n, B)] + 0.5 * rng.standard_normal((B, C))
    hot = np.array([1, 3, 4, 8], np.int32)
    ids = np.arange(B, dtype=np.int32)
    SA1 = np.zeros((B, n)); SA2 = np.zeros((B, n))
    a = O.lookup(SV, SC, 1, ids, SA1, hot, 1, 1.0)
    b = O.lookup(SV, SC, 1, ids, SA2, hot, 2, 1.0)
    assert np.array_equal(a["decision"] == 1, b["decision"] == 1)
    assert np.array_equal(a["label"][a["decision"] == 1], b["label"][b["decision"] == 1])
    assert set(np.unique(a["decision"])) <= {0, 1}
    assert (b["decision"] == 2).any()
    SA3 = np.zeros((B, n))
    c = O.lookup(SV, SC, 1, ids, SA3, np.arange(n, dtype=np.int32), 2, 1.0)
    assert not (c["decision"] == 2).any()
    # hot-tier labels are hot classes; tier-2 labels come from the whole memory
    assert set(b["label"][b["decision"] == 1]) <= set(hot.tolist())


def test_lookup_brute_force_python_on_tiny_inputs():
    n, C, B, L = 5, 4, 12, 3
    cents = [rng.standard_normal((n, C)) for _ in range(L)]
    hot = [3, 0, 4]
    tau = 0.7
    SA = np.zeros((B, n))
    live = list(range(B))
    for l in range(1, L + 1):
        SV = rng.standard_normal((len(live), C))
        snapshot = SA.copy()
        out = O.lookup(SV, cents[l - 1], l, np.array(live, np.int32), SA, np.array(hot, np.int32), 2, tau)
        nxt = []
        for i, b in enumerate(live):
            sa = []
            for j in range(n):
                dot = sum(SV[i][c] * cents[l - 1][j][c] for c in range(C))
                nv = math.sqrt(sum(x * x for x in SV[i])); nc = math.sqrt(sum(x * x for x in cents[l - 1][j]))
                sa.append(snapshot[b][j] + 2 ** (l - 1) * dot / (nv * nc))
            assert np.allclose(SA[b], sa, atol=1e-14)

            def decide(ids):
                o = sorted(ids, key=lambda j: (-sa[j], j))
                H, S = sa[o[0]], sa[o[1]]
                if H <= 0:
                    return False, o[0]
                if S <= 0:
                    return True, o[0]
                return (H - S) / S > tau, o[0]
            e1, l1 = decide(hot)
            e2, l2 = decide(range(n))
            want = (1, l1) if e1 else ((2, l2) if e2 else (0, -1))
            assert (out["decision"][i], out["label"][i]) == want
            if want[0] == 0:
                nxt.append(b)
        live = nxt


# ------------------------------------------------------------------ compaction

def test_compact_is_stable_partition_and_matches_flatnonzero():
    for n_live in (0, 1, 7, 64, 300):
        decision = rng.integers(0, 3, n_live).astype(np.int32)
        frame_ids = np.sort(rng.choice(1000, n_live, replace=False)).astype(np.int32)
        label = np.where(decision != 0, rng.integers(0, 9, n_live), -1).astype(np.int32)
        out = O.compact(decision, label, frame_ids)
        ex = np.flatnonzero(decision != 0); lv = np.flatnonzero(decision == 0)
        assert np.array_equal(out["exit_ids"], frame_ids[ex])
        assert np.array_equal(out["live_ids"], frame_ids[lv])
        assert np.array_equal(out["live_slots"], lv)
        assert np.array_equal(out["exit_labels"], label[ex])
        assert np.array_equal(out["exit_tier"], decision[ex])
        assert len(out["exit_ids"]) + len(out["live_ids"]) == n_live
    allx = O.compact(np.ones(5, np.int32), np.zeros(5, np.int32), np.arange(5, dtype=np.int32))
    assert len(allx["live_ids"]) == 0 and len(allx["exit_ids"]) == 5
    none = O.compact(np.zeros(5, np.int32), np.full(5, -1, np.int32), np.arange(5, dtype=np.int32))
    assert len(none["live_ids"]) == 5 and len(none["exit_ids"]) == 0


# ------------------------------------------------------------------ FT / TS (Sec. 6.1)

def test_tables_sequential_equals_closed_form_per_batch():
    n = 11
    FT = rng.integers(0, 50, n).astype(np.uint32); TS = rng.integers(0, 3000, n).astype(np.uint32)
    for B in (1, 5, 64, 257):
        label = rng.integers(-1, n, B).astype(np.int32)
        FT0, TS0 = FT.copy(), TS.copy()
        O.tables_update(FT, TS, label)
        for i in range(n):
            pos = np.flatnonzero(label == i)
            assert FT[i] == FT0[i] + len(pos)
            assert TS[i] == (B - 1 - pos[-1] if len(pos) else TS0[i] + B)


def test_tables_hand_example():
    FT = np.zeros(3, np.uint32); TS = np.zeros(3, np.uint32)
    O.tables_update(FT, TS, np.array([0, 0, 2, -1, 0], np.int32))
    assert FT.tolist() == [3, 0, 1]
    assert TS.tolist() == [0, 5, 2]


# ------------------------------------------------------------------ Score (Eq. 5), policy, P(A) (Eq. 6)

def test_score_integer_form_is_eq5_times_four_pow_15():
    W = 100
    for FT in (0, 1, 3, 1000, 2 ** 32 - 1):
        for TS in (0, 1, 99, 100, 101, 199, 200, 1499, 1500):
            assert O.score_int(FT, TS, W) == Fraction(FT) * Fraction(1, 4) ** (TS // W) * 4 ** 15
            assert O.score_real(FT, TS, W) == FT * 0.25 ** (TS // W)


def test_score_quarters_exactly_when_ts_crosses_a_multiple_of_w():
    W = 37
    for q in range(0, 14):
        assert O.score_int(64, q * W + W - 1, W) == 4 * O.score_int(64, (q + 1) * W, W)
        assert O.score_int(64, q * W, W) == O.score_int(64, q * W + W - 1, W)
    assert O.score_int(64, 15 * W, W) == O.score_int(64, 400 * W, W) == 64      # exponent clamped at 15


def _policy_brute(FT, TS, W, num, den, kmin, kmax):
    n = len(FT)
    sc = [Fraction(int(FT[i])) * Fraction(1, 4) ** min(int(TS[i]) // W, 15) for i in range(n)]
    order = sorted(range(n), key=lambda i: (-sc[i], i))
    tot = sum(sc)
    if tot == 0:
        return order, -1, -1
    part = Fraction(0); k = None
    for t, i in enumerate(order):
        part += sc[i]
        if part / tot >= Fraction(num, den):
            k = t + 1
            break
    return order, min(max(k, kmin), kmax), k


def test_select_hot_matches_brute_force_with_exact_fractions():
    for trial in range(300):
        n = int(rng.integers(2, 9))
        FT = rng.integers(0, 6, n).astype(np.uint32); TS = rng.integers(0, 50, n).astype(np.uint32)
        W = int(rng.integers(1, 20))
        kmin = int(rng.integers(1, n + 1)); kmax = int(rng.integers(kmin, n + 1))
        order, k, ku = O.select_hot(FT, TS, W, 19, 20, kmin, kmax)
        bo, bk, bku = _policy_brute(FT, TS, W, 19, 20, kmin, kmax)
        assert order.tolist() == bo and k == bk and ku == bku


def test_p_of_a_monotone_reaches_one_and_threshold_is_first_crossing():
    n = 40
    FT = rng.integers(0, 100, n).astype(np.uint32); TS = rng.integers(0, 5000, n).astype(np.uint32)
    order, k, ku = O.select_hot(FT, TS, 1024, 19, 20, 1, n)
    p = [O.p_of_a(FT, TS, 1024, order, kk) for kk in range(n + 1)]
    assert p[0] == 0.0 and abs(p[n] - 1.0) < 1e-15
    assert all(p[i] <= p[i + 1] + 1e-18 for i in range(n))
    assert p[ku] >= 0.95 - 1e-12 and p[ku - 1] < 0.95 + 1e-12 and k == ku


def test_select_hot_special_cases():
    n = 100
    TS = np.zeros(n, np.uint32)
    FT = np.zeros(n, np.uint32); FT[17] = 1000
    order, k, ku = O.select_hot(FT, TS, 10, 19, 20, 8, 64)
    assert ku == 1 and k == 8 and order[0] == 17          # one dominant class -> clamped to k_min
    assert order[1:9].tolist() == [0, 1, 2, 3, 4, 5, 6, 7]  # zero scores fall back to id order
    FT[:] = 5
    order, k, ku = O.select_hot(FT, TS, 10, 19, 20, 8, 64)
    assert ku == 95 and k == 64                           # uniform scores -> ceil(0.95 n) -> k_max
    assert order.tolist() == list(range(n))
    FT[:] = 0
    assert O.select_hot(FT, TS, 10, 19, 20, 8, 64)[1] == -1   # no history: keep the previous set
    # recency beats frequency once a window has passed: 10 seen now vs 39 seen W frames ago
    FT = np.array([39, 10], np.uint32); TS = np.array([10, 0], np.uint32)
    assert O.select_hot(FT, TS, 10, 19, 20, 1, 2)[0].tolist() == [1, 0]
    FT = np.array([41, 10], np.uint32)
    assert O.select_hot(FT, TS, 10, 19, 20, 1, 2)[0].tolist() == [0, 1]
    # exactly at the confidence level counts as reached (>=): scores 19 and 1 -> k = 1
    FT = np.array([19, 1], np.uint32); TS = np.zeros(2, np.uint32)
    assert O.select_hot(FT, TS, 10, 19, 20, 1, 2)[2] == 1


def test_select_hot_huge_counts_do_not_overflow():
    n = 8
    FT = np.full(n, 2 ** 32 - 1, np.uint32); TS = np.zeros(n, np.uint32)
    order, k, ku = O.select_hot(FT, TS, 10, 19, 20, 1, n)
    assert ku == 8 and order.tolist() == list(range(n))     # 7/8 < 0.95 <= 8/8


# ------------------------------------------------------------------ centres (Eq. 7)

def test_centres_running_mean_closed_form_and_layer_range():
    n, dims, B = 6, [4, 3, 5], 40
    SC = [rng.standard_normal((n, c)) for c in dims]
    SC0 = [s.copy() for s in SC]
    m = [np.full(n, 7, np.uint32) for _ in dims]
    SV = [rng.standard_normal((B, c)) for c in dims]
    label = rng.integers(-1, n, B).astype(np.int32)
    stop = rng.integers(0, 4, B).astype(np.int32)
    O.centres_update(SC, m, SV, label, stop)
    for l0 in range(3):
        for j in range(n):
            sel = (label == j) & (stop >= l0 + 1)          # inclusive range 1..stop_layer
            cnt = int(sel.sum())
            want = (7 * SC0[l0][j] + SV[l0][sel].sum(axis=0)) / (7 + cnt)
            assert np.allclose(SC[l0][j], want, rtol=1e-13, atol=1e-15)
            assert m[l0][j] == 7 + cnt


def test_centres_single_step_is_eq7_and_m0_zero_identical_updates():
    SC = [np.array([[1.0, 2.0], [5.0, 5.0]])]; m = [np.array([3, 9], np.uint32)]
    SV = [np.array([[5.0, -2.0]])]
    O.centres_update(SC, m, SV, np.array([0], np.int32), np.array([1], np.int32))
    assert np.array_equal(SC[0], [[2.0, 1.0], [5.0, 5.0]]) and m[0].tolist() == [4, 9]
    SC = [np.array([[9.0, 9.0]])]; m = [np.zeros(1, np.uint32)]
    sv = np.array([[0.25, -3.0]])
    SV = [np.repeat(sv, 5, axis=0)]
    O.centres_update(SC, m, SV, np.zeros(5, np.int32), np.ones(5, np.int32))
    assert np.allclose(SC[0][0], sv[0], rtol=1e-15) and m[0][0] == 5
    assert abs(O.cosine(SC[0][0], SC[0][0]) - 1.0) < 1e-15


def test_centres_ignore_unlabelled_and_not_stopped_frames():
    SC = [np.array([[1.0, 1.0]])]; m = [np.array([2], np.uint32)]
    SV = [np.array([[100.0, 100.0], [50.0, 50.0]])]
    O.centres_update(SC, m, SV, np.array([-1, 0], np.int32), np.array([1, 0], np.int32))
    assert np.array_equal(SC[0], [[1.0, 1.0]]) and m[0][0] == 2


# ------------------------------------------------------------------ Eq. 2

def test_sep_eq2():
    assert O.sep(0.9, 0.3) == pytest.approx(2.0)


# ------------------------------------------------------------------ Memory driver (host logic around the C calls)

def test_memory_stage_on_generated_tiny_workload_recovers_classes():
    from workloads import configs, streams
    w = configs.TINY
    cents = streams.centroids(w); ls = streams.labels(w)
    F = streams.batch_feature_maps(w, cents, ls, 0)[0].numpy()
    mem = O.Memory([c.numpy() for c in cents], ls.initial_hot, tau=1.0, tiers=2)
    mem.begin_batch(w.batch)
    out = mem.stage(1, F, want_sims=True)
    # generator property: SV ~ centroid + N(0, sigma^2/HW) per channel
    resid = out["SV"] - cents[0].numpy()[ls.label]
    assert abs(resid.std() - w.sigma / 14.0) < 0.15 * w.sigma / 14.0
    # every frame's best class over the whole memory is its true class at this noise level
    assert np.array_equal(out["top_id"][:, 1], ls.label)
    # at a low threshold hot-class frames leave on tier 1 with the right label
    hot = np.isin(ls.label, ls.initial_hot)
    assert np.all(out["decision"][hot] == 1) and np.array_equal(out["label"][hot], ls.label[hot])
    assert len(out["exit_ids"]) + len(out["live_ids"]) == w.batch
    assert np.array_equal(mem.exit_layer != 0, out["decision"] != 0)
    # at the workload's own threshold all three outcomes occur and tier-1 labels are hot classes
    mem = O.Memory([c.numpy() for c in cents], ls.initial_hot, tau=w.tau, tiers=2)
    mem.begin_batch(w.batch)
    out = mem.stage(1, F)
    assert set(np.unique(out["decision"])) == {0, 1, 2}
    assert set(out["label"][out["decision"] == 1]) <= set(ls.initial_hot.tolist())
    assert np.array_equal(out["label"][out["decision"] == 2], ls.label[out["decision"] == 2])


# ------------------------------------------------------------------ forgetting applied in place (Sec. 6.1 text)

def _inplace_brute(FT, TS, W, label):
    FT = [int(x) for x in FT]; TS = [int(x) for x in TS]
    for j in label:
        for i in range(len(FT)):
            if i == j:
                continue
            TS[i] += 1
            if TS[i] % W == 0:
                FT[i] = FT[i] // 4
        if j >= 0:
            TS[j] = 0
            FT[j] += 1
    return FT, TS


def test_inplace_forgetting_matches_python_brute_force():
    for trial in range(100):
        n = int(rng.integers(2, 7)); W = int(rng.integers(1, 9)); B = int(rng.integers(1, 40))
        FT = rng.integers(0, 300, n).astype(np.uint32); TS = rng.integers(0, 30, n).astype(np.uint32)
        label = rng.integers(-1, n, B).astype(np.int32)
        want = _inplace_brute(FT, TS, W, label.tolist())
        O.tables_update_inplace(FT, TS, W, label)
        assert FT.tolist() == want[0] and TS.tolist() == want[1]


def test_inplace_forgetting_hand_example_and_relation_to_eq5():
    # class 0 seen 64 times, then 10 frames of class 1 with W = 4: TS_0 = 10, two decays -> 64/16 = 4
    FT = np.array([64, 0], np.uint32); TS = np.zeros(2, np.uint32)
    O.tables_update_inplace(FT, TS, 4, np.ones(10, np.int32))
    assert FT.tolist() == [4, 10] and TS.tolist() == [10, 0]
    # while a class stays away, the in-place value is the floor of Eq. 5's score ...
    assert FT[0] == math.floor(O.score_real(64, 10, 4))
    # ... but when it comes back the decayed history stays forgotten (Eq. 5 would give 65 again)
    O.tables_update_inplace(FT, TS, 4, np.zeros(1, np.int32))
    assert FT[0] == 5 and TS[0] == 0
    FT2 = np.array([64, 0], np.uint32); TS2 = np.zeros(2, np.uint32)
    O.tables_update(FT2, TS2, np.array([1] * 10 + [0], np.int32))
    assert O.score_int(int(FT2[0]), int(TS2[0]), 4) == 65 * 4 ** 15


def test_frame_by_frame_cadence_equals_one_batch_for_both_forgetting_modes():
    n, W = 9, 5
    label = rng.integers(-1, n, 137).astype(np.int32)
    for inplace in (False, True):
        FT = rng.integers(0, 50, n).astype(np.uint32); TS = rng.integers(0, 20, n).astype(np.uint32)
        FTa, TSa, FTb, TSb = FT.copy(), TS.copy(), FT.copy(), TS.copy()
        if inplace:
            O.tables_update_inplace(FTa, TSa, W, label)
            for x in label:
                O.tables_update_inplace(FTb, TSb, W, np.array([x], np.int32))
        else:
            O.tables_update(FTa, TSa, label)
            for x in label:
                O.tables_update(FTb, TSb, np.array([x], np.int32))
        assert np.array_equal(FTa, FTb) and np.array_equal(TSa, TSb)
        a = O.select_hot(FTa, TSa, W, 19, 20, 2, n, inplace=inplace)
        b = O.select_hot(FTb, TSb, W, 19, 20, 2, n, inplace=inplace)
        assert a[0].tolist() == b[0].tolist() and a[1:] == b[1:]


def test_select_hot_inplace_scores_are_the_frequencies():
    FT = np.array([3, 9, 9, 0, 1], np.uint32); TS = np.array([0, 500, 0, 0, 7], np.uint32)
    order, k, ku = O.select_hot(FT, TS, 10, 19, 20, 1, 5, inplace=True)
    assert order.tolist() == [1, 2, 0, 4, 3]            # TS plays no part any more; ties by id
    assert ku == 3                                       # (9+9+3)/22 = 0.9545 >= 0.95, (9+9)/22 is not


# ------------------------------------------------------------------ warm-up (Sec. 5, Sec. 6.3)

def test_warmup_centres_are_class_means():
    n, C, N = 7, 5, 60
    SV = rng.standard_normal((N, C)); label = rng.integers(-1, n, N).astype(np.int32)
    label[label == 3] = 2                                  # class 3 has no samples
    SC, m = O.warmup_centres(SV, label, n)
    for j in range(n):
        sel = label == j
        assert m[j] == sel.sum()
        want = SV[sel].mean(axis=0) if sel.any() else np.zeros(C)
        assert np.allclose(SC[j], want, rtol=1e-14, atol=1e-16)
    assert np.all(SC[3] == 0) and m[3] == 0


def test_warmup_equals_eq7_started_from_count_zero():
    # the running mean of Eq. 7 with m = 0 at the start reaches the same centres
    n, C, N = 4, 3, 25
    SV = rng.standard_normal((N, C)); label = rng.integers(0, n, N).astype(np.int32)
    SC, m = O.warmup_centres(SV, label, n)
    SC2 = [np.full((n, C), 123.0)]; m2 = [np.zeros(n, np.uint32)]
    O.centres_update(SC2, m2, [SV], label, np.ones(N, np.int32))
    seen = m > 0
    assert np.allclose(SC2[0][seen], SC[seen], rtol=1e-13) and np.array_equal(m2[0], m)


def test_separability_eq2_hand_values_and_sign_cases():
    assert O.separability(np.array([0.9, 0.3, 0.1])) == pytest.approx(2.0)            # (0.9 - 0.3) / 0.3
    assert O.separability(np.array([0.9, 0.3, 0.6]), np.array([0, 1], np.int32)) == pytest.approx(2.0)
    assert O.separability(np.array([0.9, 0.3, 0.6])) == pytest.approx(0.5)            # runner-up is 0.6
    assert O.separability(np.array([0.5, -0.2])) == np.inf
    assert O.separability(np.array([-0.5, -0.2])) == -np.inf
    assert O.separability(np.array([0.5]), np.array([0], np.int32)) == -np.inf
    assert O.separability(np.array([0.4, 0.4])) == 0.0
