"""ctypes/numpy front end of the C oracle in smtm_oracle.c.

TEST INFRASTRUCTURE, NOT THE PRODUCT: only the tests, the smoke check and the
benchmark's CPU-baseline leg may use this module.  It imports nothing from the
GPU package and the GPU package imports nothing from here.

The arithmetic of the method lives in smtm_oracle.c; this file only marshals
numpy arrays and keeps the memory state (centres, update counts, frequency and
time-stamp tables, fast-memory set) that Sec. 6 of arXiv 2112.02644 describes.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "smtm_oracle.c"
_LIB = _HERE / "libsmtm_oracle.so"
_lib = None

F16, F32 = 0, 1


def build(force: bool = True) -> Path:
    """Compile smtm_oracle.c with gcc (-O2, no fast-math, OpenMP over frames)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", str(_LIB), str(_SRC), "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        # SMTM_ORACLE_LIB: a test may point this module at a deliberately broken build of the oracle
        # to show that the pins notice (tests/test_oracle_mutations.py)
        override = os.environ.get("SMTM_ORACLE_LIB")
        if override:
            L = C.CDLL(override)
        else:
            build(force=False)
            L = C.CDLL(str(_LIB))
        dp, ip, vp = C.POINTER(C.c_double), C.POINTER(C.c_int32), C.c_void_p
        up = C.POINTER(C.c_uint32)
        L.orc_half_to_double.restype = C.c_double
        L.orc_half_to_double.argtypes = [C.c_uint16]
        L.orc_encode.restype = None
        L.orc_encode.argtypes = [vp, C.c_int, C.c_int, C.c_int, vp, C.c_int64, vp]
        L.orc_cosine.restype = C.c_double
        L.orc_cosine.argtypes = [vp, vp, C.c_int]
        L.orc_cosine_abs_scale.restype = C.c_double
        L.orc_cosine_abs_scale.argtypes = [vp, vp, C.c_int]
        L.orc_weight.restype = C.c_double
        L.orc_weight.argtypes = [C.c_int]
        L.orc_top2.restype = None
        L.orc_top2.argtypes = [vp, vp, C.c_int, dp, ip, dp]
        L.orc_exit_predicate.restype = C.c_int
        L.orc_exit_predicate.argtypes = [C.c_double, C.c_double, C.c_double]
        L.orc_accumulated_confidence.restype = C.c_double
        L.orc_accumulated_confidence.argtypes = [C.c_double, C.c_double]
        L.orc_lookup.restype = None
        L.orc_lookup.argtypes = [vp, vp, C.c_int, C.c_int, C.c_int, vp, C.c_int64, vp,
                                 vp, C.c_int, C.c_int, C.c_double, vp, vp, vp, vp, vp, vp]
        L.orc_compact.restype = None
        L.orc_compact.argtypes = [vp, vp, vp, C.c_int64, vp, vp, vp, ip, vp, vp, ip]
        L.orc_tables_update.restype = None
        L.orc_tables_update.argtypes = [vp, vp, C.c_int, vp, C.c_int64]
        L.orc_tables_update_inplace.restype = None
        L.orc_tables_update_inplace.argtypes = [vp, vp, C.c_int, C.c_uint32, vp, C.c_int64]
        L.orc_select_hot_mode.restype = C.c_int32
        L.orc_select_hot_mode.argtypes = [vp, vp, C.c_int, C.c_uint32, C.c_int, C.c_uint32, C.c_uint32,
                                          C.c_int32, C.c_int32, vp, ip]
        L.orc_score_int.restype = C.c_uint64
        L.orc_score_int.argtypes = [C.c_uint32, C.c_uint32, C.c_uint32]
        L.orc_score_real.restype = C.c_double
        L.orc_score_real.argtypes = [C.c_uint32, C.c_uint32, C.c_uint32]
        L.orc_select_hot.restype = C.c_int32
        L.orc_select_hot.argtypes = [vp, vp, C.c_int, C.c_uint32, C.c_uint32, C.c_uint32,
                                     C.c_int32, C.c_int32, vp, ip]
        L.orc_p_of_a.restype = C.c_double
        L.orc_p_of_a.argtypes = [vp, vp, C.c_int, C.c_uint32, vp, C.c_int]
        L.orc_centres_update.restype = None
        L.orc_centres_update.argtypes = [vp, vp, vp, C.c_int, C.c_int, vp, vp, vp, C.c_int64]
        L.orc_warmup_centres.restype = None
        L.orc_warmup_centres.argtypes = [vp, vp, C.c_int64, C.c_int, C.c_int, vp, vp]
        L.orc_separability.restype = C.c_double
        L.orc_separability.argtypes = [vp, vp, C.c_int]
        L.orc_sep.restype = C.c_double
        L.orc_sep.argtypes = [C.c_double, C.c_double]
        _lib = L
    return _lib


def set_threads(n: int) -> None:
    """Number of OpenMP threads the frame loops use (libgomp's omp_set_num_threads)."""
    gomp = C.CDLL("libgomp.so.1")
    gomp.omp_set_num_threads(int(n))


def get_max_threads() -> int:
    gomp = C.CDLL("libgomp.so.1")
    gomp.omp_get_max_threads.restype = C.c_int
    return int(gomp.omp_get_max_threads())


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _c(a, dt):
    a = np.ascontiguousarray(a, dtype=dt)
    return a


# --------------------------------------------------------------------------- thin wrappers

def half_to_double(bits: int) -> float:
    return float(lib().orc_half_to_double(int(bits) & 0xFFFF))


def encode(F: np.ndarray, row_ids=None, n_live=None) -> np.ndarray:
    """Sec. 4.1 GAP.  F is [rows, C, H, W] float16 or float32.  Returns [n_live, C] float64."""
    assert F.ndim == 4 and F.flags.c_contiguous
    if F.dtype == np.float16:
        dt = F16
    elif F.dtype == np.float32:
        dt = F32
    else:
        raise TypeError("feature maps are float16 or float32")
    rows, Cc, H, W = F.shape
    if row_ids is not None:
        row_ids = _c(row_ids, np.int32)
        if n_live is None:
            n_live = row_ids.shape[0]
        assert row_ids[:n_live].min(initial=0) >= 0 and row_ids[:n_live].max(initial=0) < rows
    elif n_live is None:
        n_live = rows
    assert n_live <= (rows if row_ids is None else row_ids.shape[0])
    SV = np.empty((n_live, Cc), dtype=np.float64)
    lib().orc_encode(_p(F), dt, Cc, H * W, _p(row_ids), n_live, _p(SV))
    return SV


def cosine(v, c) -> float:
    v = _c(v, np.float64); c = _c(c, np.float64)
    assert v.shape == c.shape and v.ndim == 1
    return float(lib().orc_cosine(_p(v), _p(c), v.shape[0]))


def cosine_abs_scale(v, c) -> float:
    """Rounding-error scale of the cosine: sum |v_k||c_k| / (|v||c|) (the tests' tolerance unit)."""
    v = _c(v, np.float64); c = _c(c, np.float64)
    assert v.shape == c.shape and v.ndim == 1
    return float(lib().orc_cosine_abs_scale(_p(v), _p(c), v.shape[0]))


def weight(l: int) -> float:
    return float(lib().orc_weight(l))


def top2(SA, ids=None):
    SA = _c(SA, np.float64)
    if ids is not None:
        ids = _c(ids, np.int32)
        cnt = ids.shape[0]
    else:
        cnt = SA.shape[0]
    h, sh, i = C.c_double(), C.c_double(), C.c_int32()
    lib().orc_top2(_p(SA), _p(ids), cnt, C.byref(h), C.byref(i), C.byref(sh))
    return h.value, i.value, sh.value


def exit_predicate(SA_H, SA_SH, tau) -> bool:
    return bool(lib().orc_exit_predicate(float(SA_H), float(SA_SH), float(tau)))


def accumulated_confidence(SA_H, SA_SH) -> float:
    return float(lib().orc_accumulated_confidence(float(SA_H), float(SA_SH)))


def lookup(SV, SC, l, frame_ids, SA, hot_ids, tiers, tau, want_sims=False):
    """One exit point for the live frames (orc_lookup).  SA is updated in place.

    Returns dict(decision, label, top_val [n_live,2,2], top_id [n_live,2], sims, sims_scale).
    """
    SV = _c(SV, np.float64); SC = _c(SC, np.float64)
    n_live, Cc = SV.shape
    n = SC.shape[0]
    assert SC.shape[1] == Cc
    frame_ids = _c(frame_ids, np.int32)
    hot_ids = _c(hot_ids, np.int32)
    assert SA.dtype == np.float64 and SA.flags.c_contiguous and SA.shape[1] == n
    assert frame_ids.shape[0] == n_live
    if n_live:
        assert 0 <= frame_ids.min() and frame_ids.max() < SA.shape[0]
    decision = np.zeros(n_live, np.int32)
    label = np.full(n_live, -1, np.int32)
    top_val = np.full((n_live, 2, 2), -np.inf, np.float64)
    top_id = np.full((n_live, 2), -1, np.int32)
    sims = np.empty((n_live, n), np.float64) if want_sims else None
    scale = np.empty((n_live, n), np.float64) if want_sims else None
    lib().orc_lookup(_p(SV), _p(SC), n, Cc, int(l), _p(frame_ids), n_live, _p(SA),
                     _p(hot_ids), hot_ids.shape[0], int(tiers), float(tau),
                     _p(decision), _p(label), _p(top_val), _p(top_id), _p(sims), _p(scale))
    return dict(decision=decision, label=label, top_val=top_val, top_id=top_id,
                sims=sims, sims_scale=scale)


def compact(decision, label, frame_ids):
    decision = _c(decision, np.int32); label = _c(label, np.int32); frame_ids = _c(frame_ids, np.int32)
    n = decision.shape[0]
    ex_i = np.empty(n, np.int32); ex_l = np.empty(n, np.int32); ex_t = np.empty(n, np.int32)
    lv = np.empty(n, np.int32); ls = np.empty(n, np.int32)
    ne, nl = C.c_int32(), C.c_int32()
    lib().orc_compact(_p(decision), _p(label), _p(frame_ids), n, _p(ex_i), _p(ex_l), _p(ex_t),
                      C.byref(ne), _p(lv), _p(ls), C.byref(nl))
    return dict(exit_ids=ex_i[:ne.value].copy(), exit_labels=ex_l[:ne.value].copy(),
                exit_tier=ex_t[:ne.value].copy(), live_ids=lv[:nl.value].copy(),
                live_slots=ls[:nl.value].copy())


def score_int(FT, TS, W) -> int:
    return int(lib().orc_score_int(int(FT), int(TS), int(W)))


def score_real(FT, TS, W) -> float:
    return float(lib().orc_score_real(int(FT), int(TS), int(W)))


def tables_update(FT, TS, label):
    assert FT.dtype == np.uint32 and TS.dtype == np.uint32
    label = _c(label, np.int32)
    lib().orc_tables_update(_p(FT), _p(TS), FT.shape[0], _p(label), label.shape[0])


def tables_update_inplace(FT, TS, W, label):
    """Sec. 6.1 with the forgetting applied to the frequency table itself."""
    assert FT.dtype == np.uint32 and TS.dtype == np.uint32
    label = _c(label, np.int32)
    lib().orc_tables_update_inplace(_p(FT), _p(TS), FT.shape[0], int(W), _p(label), label.shape[0])


def select_hot(FT, TS, W, cl_num, cl_den, k_min, k_max, inplace=False):
    """Returns (order [n], k or -1, k before clamping)."""
    assert FT.dtype == np.uint32 and TS.dtype == np.uint32
    n = FT.shape[0]
    order = np.empty(n, np.int32)
    ku = C.c_int32()
    k = lib().orc_select_hot_mode(_p(FT), _p(TS), n, int(W), int(bool(inplace)), int(cl_num), int(cl_den),
                                  int(k_min), int(k_max), _p(order), C.byref(ku))
    return order, int(k), int(ku.value)


def p_of_a(FT, TS, W, order, k) -> float:
    order = _c(order, np.int32)
    return float(lib().orc_p_of_a(_p(FT), _p(TS), FT.shape[0], int(W), _p(order), int(k)))


def centres_update(SC_list, m_list, SV_list, label, stop_layer):
    """Eq. 7 in place.  SC_list[l0]: [n,C] float64; m_list[l0]: [n] uint32; SV_list[l0]: [batch,C] float64."""
    L = len(SC_list)
    n = SC_list[0].shape[0]
    label = _c(label, np.int32); stop_layer = _c(stop_layer, np.int32)
    batch = label.shape[0]
    dims = np.array([sc.shape[1] for sc in SC_list], np.int32)
    for sc, m, sv in zip(SC_list, m_list, SV_list):
        assert sc.dtype == np.float64 and sc.flags.c_contiguous
        assert m.dtype == np.uint32 and sv.dtype == np.float64 and sv.flags.c_contiguous
        assert sv.shape == (batch, sc.shape[1])
    PP = C.c_void_p * L
    sc_p = PP(*[sc.ctypes.data for sc in SC_list])
    m_p = PP(*[m.ctypes.data for m in m_list])
    sv_p = PP(*[sv.ctypes.data for sv in SV_list])
    lib().orc_centres_update(sc_p, m_p, _p(dims), L, n, sv_p, _p(label), _p(stop_layer), batch)


def warmup_centres(SV, label, n):
    """Class means of the training frames' semantic vectors: returns (SC [n,C] float64, m [n] uint32)."""
    SV = _c(SV, np.float64); label = _c(label, np.int32)
    N, Cc = SV.shape
    assert label.shape[0] == N
    SC = np.empty((n, Cc), np.float64); m = np.empty(n, np.uint32)
    lib().orc_warmup_centres(_p(SV), _p(label), N, int(n), Cc, _p(SC), _p(m))
    return SC, m


def separability(s, ids=None) -> float:
    """Eq. 2 for one frame's similarities over a set of classes (None = all)."""
    s = _c(s, np.float64)
    if ids is not None:
        ids = _c(ids, np.int32)
    return float(lib().orc_separability(_p(s), _p(ids), s.shape[0] if ids is None else ids.shape[0]))


def sep(s_H, s_SH) -> float:
    return float(lib().orc_sep(float(s_H), float(s_SH)))


# --------------------------------------------------------------------------- memory state

class Memory:
    """Global memory + fast memory of Sec. 6: centres per exit point, their update counts,
    the frequency and time-stamp tables, and the fast-memory set Psi (policy order)."""

    def __init__(self, centres, hot_ids, *, tau, tiers=2, window=1024, cl=(19, 20),
                 hot_min=2, hot_max=None, init_count=100, forgetting=0):
        self.forgetting = int(forgetting)        # 0: at scoring time (Eq. 5); 1: in place (Sec. 6.1 text)
        self.SC = [np.ascontiguousarray(c, dtype=np.float64).copy() for c in centres]
        self.L = len(self.SC)
        self.n = self.SC[0].shape[0]
        self.dims = [c.shape[1] for c in self.SC]
        self.m = [np.full(self.n, init_count, np.uint32) for _ in self.SC]
        self.FT = np.zeros(self.n, np.uint32)
        self.TS = np.zeros(self.n, np.uint32)
        self.hot_ids = np.array(hot_ids, np.int32).copy()
        self.tau = float(tau)
        self.tiers = int(tiers)
        self.window = int(window)
        self.cl = (int(cl[0]), int(cl[1]))
        self.hot_min = int(hot_min)
        self.hot_max = int(hot_max if hot_max is not None else self.n)

    # one batch ------------------------------------------------------------
    def begin_batch(self, batch):
        self.batch = int(batch)
        self.SA = np.zeros((self.batch, self.n), np.float64)
        self.live = np.arange(self.batch, dtype=np.int32)
        self.SV = [np.zeros((self.batch, c), np.float64) for c in self.dims]
        self.exit_layer = np.zeros(self.batch, np.int32)
        self.label = np.full(self.batch, -1, np.int32)
        self.tier = np.zeros(self.batch, np.int32)

    def stage(self, l, F, row_ids=None, live=None, want_sims=False):
        """Exit point l (1-based) on feature maps F.  `live` overrides the oracle's own live
        list (teacher forcing).  Returns the lookup dict plus the compaction lists."""
        if live is not None:
            self.live = np.array(live, np.int32).copy()
        n_live = self.live.shape[0]
        SV = encode(F, row_ids=row_ids, n_live=n_live)
        self.SV[l - 1][self.live] = SV
        out = lookup(SV, self.SC[l - 1], l, self.live, self.SA, self.hot_ids, self.tiers,
                     self.tau, want_sims=want_sims)
        out["SV"] = SV
        out["frame_ids"] = self.live.copy()
        out.update(compact(out["decision"], out["label"], self.live))
        ex = out["exit_ids"]
        self.exit_layer[ex] = l
        self.label[ex] = out["exit_labels"]
        self.tier[ex] = out["exit_tier"]
        self.live = out["live_ids"].copy()
        return out

    # between batches -----------------------------------------------------
    def cache_update(self, label, stop_layer):
        """Sec. 6: tables, centres (Eq. 7), score (Eq. 5), fast-memory set and size (Eq. 6)."""
        label = np.asarray(label, np.int32); stop_layer = np.asarray(stop_layer, np.int32)
        if self.forgetting:
            tables_update_inplace(self.FT, self.TS, self.window, label)
        else:
            tables_update(self.FT, self.TS, label)
        centres_update(self.SC, self.m, self.SV, label, stop_layer)
        order, k, ku = select_hot(self.FT, self.TS, self.window, self.cl[0], self.cl[1],
                                  self.hot_min, self.hot_max, inplace=bool(self.forgetting))
        if k >= 0:
            self.hot_ids = order[:k].copy()
        return dict(order=order, k=k, k_unclamped=ku)
