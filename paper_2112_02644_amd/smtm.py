"""ctypes binding of libsmtm.so.  Argument marshalling only: every step of the path runs in
the library's HIP kernels.  There is no fallback: if the library is missing or a call fails,
an exception is raised."""
from __future__ import annotations

import ctypes as C
from dataclasses import dataclass, field
from pathlib import Path
from typing import List, Optional, Sequence

_PKG = Path(__file__).resolve().parent
_LIB_PATH = _PKG / "libsmtm.so"
_lib = None

F16, F32 = 0, 1
SCORE_AUTO, SCORE_FP32, SCORE_MFMA = 0, 1, 2
MAX_EXITS = 8

_ERR_NAMES = {1: "INVALID_ARG", 2: "SHAPE", 3: "STATE", 4: "UNSUPPORTED", 5: "NOMEM", 6: "HIP"}


class SmtmError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"SMTM_ERR_{_ERR_NAMES.get(code, code)}: {text}")
        self.code = code


class _Config(C.Structure):
    _fields_ = [("n_classes", C.c_int32), ("n_exits", C.c_int32), ("dims", C.c_int32 * MAX_EXITS),
                ("max_batch", C.c_int32), ("hot_init", C.c_int32), ("hot_min", C.c_int32),
                ("hot_max", C.c_int32), ("tiers", C.c_int32), ("tau", C.c_float),
                ("window", C.c_int32), ("cl_num", C.c_int32), ("cl_den", C.c_int32),
                ("init_count", C.c_int32), ("score_path", C.c_int32), ("forgetting", C.c_int32)]


@dataclass
class SmtmConfig:
    n_classes: int
    dims: Sequence[int]
    max_batch: int
    hot_init: int
    hot_min: int = 2
    hot_max: Optional[int] = None
    tiers: int = 2
    tau: float = 1.0
    window: int = 1024
    cl_num: int = 19
    cl_den: int = 20
    init_count: int = 100
    score_path: int = SCORE_AUTO
    forgetting: int = 0              # 0: at scoring time (Eq. 5), 1: in place (Sec. 6.1 text)

    def to_c(self) -> _Config:
        c = _Config()
        c.n_classes = self.n_classes
        c.n_exits = len(self.dims)
        for i, d in enumerate(list(self.dims)[:MAX_EXITS]):
            c.dims[i] = int(d)
        c.max_batch = self.max_batch
        c.hot_init = self.hot_init
        c.hot_min = self.hot_min
        c.hot_max = self.hot_init if self.hot_max is None else self.hot_max
        c.tiers = self.tiers
        c.tau = self.tau
        c.window = self.window
        c.cl_num = self.cl_num
        c.cl_den = self.cl_den
        c.init_count = self.init_count
        c.score_path = self.score_path
        c.forgetting = self.forgetting
        return c


def load_library():
    """Loads libsmtm.so built in-tree (python -m paper_2112_02644_amd.build, or
    __graft_entry__.build()).  A library that is missing, or that was built from other sources than
    the ones in the tree (their hash is compiled into it), is built first."""
    global _lib
    if _lib is not None:
        return _lib
    from . import build as _b
    if _b.needs_build():
        _b.build(verbose=False)
        if _b.needs_build():
            raise RuntimeError("libsmtm.so does not match the sources after a rebuild")
    L = C.CDLL(str(_LIB_PATH))
    vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    sig = {
        "smtm_create": [C.POINTER(vp), C.POINTER(_Config)],
        "smtm_destroy": [vp],
        "smtm_version": [],
        "smtm_memory_load": [vp, i32, vp, vp],
        "smtm_hot_set": [vp, vp, i32, vp],
        "smtm_warmup_begin": [vp, vp],
        "smtm_warmup_batch": [vp, vp, i32, vp],
        "smtm_memory_export": [vp, i32, vp, vp, vp],
        "smtm_tables_export": [vp, vp, vp, vp, vp, vp],
        "smtm_tables_import": [vp, vp, vp, vp],
        "smtm_set_tau": [vp, f32],
        "smtm_begin_batch": [vp, i32, vp],
        "smtm_encode": [vp, i32, vp, i32, i32, i32, vp, vp, vp],
        "smtm_encode_nhwc": [vp, i32, vp, i32, i32, i32, vp, vp, vp],
        "smtm_lookup": [vp, i32, vp, vp, vp, vp],
        "smtm_separability": [vp, i32, vp, vp, vp],
        "smtm_exit_compact": [vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, vp],
        "smtm_lookup_exit": [vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, vp],
        "smtm_stage": [vp, i32, vp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp],
        "smtm_stage_nhwc": [vp, i32, vp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp],
        "smtm_batch_results": [vp, vp, vp, vp, vp],
        "smtm_read_counts": [vp, vp, vp, vp],
        "smtm_read_stats": [vp, vp, vp],
        "smtm_cache_update": [vp, vp, vp, i32, vp],
        "smtm_cache_update_static": [vp, vp, vp, i32, vp],
        "smtm_memory_import": [vp, i32, vp, vp, vp],
    }
    for name, args in sig.items():
        fn = getattr(L, name)
        fn.argtypes = args
        fn.restype = i32
    L.smtm_last_error.argtypes = [vp]
    L.smtm_last_error.restype = C.c_char_p
    L.smtm_live_ids.argtypes = [vp]
    L.smtm_live_ids.restype = vp
    L.smtm_build_id.argtypes = []
    L.smtm_build_id.restype = C.c_char_p
    L.smtm_encode_kernel.argtypes = [vp, i32]
    L.smtm_encode_kernel.restype = C.c_char_p
    _lib = L
    return L


def _ptr(x) -> Optional[int]:
    """Device/host address of a torch tensor, numpy array, raw int, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        assert x.is_contiguous(), "tensors passed to the library must be contiguous"
        return x.data_ptr()
    if hasattr(x, "ctypes"):
        assert x.flags.c_contiguous
        return x.ctypes.data
    raise TypeError(type(x))


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float16:
        return F16
    if t.dtype == torch.float32:
        return F32
    raise TypeError("feature maps are float16 or float32")


class Smtm:
    """One context of the library (same names as the C entry points, minus the smtm_ prefix)."""

    def __init__(self, cfg: SmtmConfig, stream: Optional[int] = None):
        self.lib = load_library()
        self.cfg = cfg
        self._c = cfg.to_c()
        self._h = C.c_void_p()
        rc = self.lib.smtm_create(C.byref(self._h), C.byref(self._c))
        if rc != 0:
            raise SmtmError(rc, self.lib.smtm_last_error(None).decode())
        self.stream = stream
        self._keep = {}

    # -- plumbing
    def _st(self, stream=None):
        s = self.stream if stream is None else stream
        if s is None:
            import torch
            s = torch.cuda.current_stream().cuda_stream
        return C.c_void_p(s)

    def _ck(self, rc: int):
        if rc != 0:
            raise SmtmError(rc, self.lib.smtm_last_error(self._h).decode())

    def close(self):
        if self._h:
            self.lib.smtm_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- memory
    def memory_load(self, exit: int, centres_host, stream=None):
        self._ck(self.lib.smtm_memory_load(self._h, exit, _ptr(centres_host), self._st(stream)))

    def warmup_begin(self, stream=None):
        self._ck(self.lib.smtm_warmup_begin(self._h, self._st(stream)))

    def warmup_batch(self, label, batch: int, stream=None):
        self._ck(self.lib.smtm_warmup_batch(self._h, _ptr(label), batch, self._st(stream)))

    def memory_import(self, exit: int, centres_host, counts_host, stream=None):
        import numpy as np
        centres = np.ascontiguousarray(centres_host, dtype=np.float32)
        counts = np.ascontiguousarray(counts_host, dtype=np.uint32)
        assert centres.shape == (self.cfg.n_classes, self.cfg.dims[exit - 1]) and counts.shape == (self.cfg.n_classes,)
        self._ck(self.lib.smtm_memory_import(self._h, exit, _ptr(centres), _ptr(counts), self._st(stream)))
        self._keep[exit] = (centres, counts)             # the copies are stream-ordered: keep the host arrays alive

    def hot_set(self, class_ids_host, stream=None):
        import numpy as np
        ids = np.ascontiguousarray(class_ids_host, dtype=np.int32)
        self._ck(self.lib.smtm_hot_set(self._h, _ptr(ids), int(ids.shape[0]), self._st(stream)))

    def memory_export(self, exit: int, stream=None):
        import numpy as np
        n, c = self.cfg.n_classes, self.cfg.dims[exit - 1]
        centres = np.empty((n, c), np.float32)
        counts = np.empty(n, np.uint32)
        self._ck(self.lib.smtm_memory_export(self._h, exit, _ptr(centres), _ptr(counts), self._st(stream)))
        return centres, counts

    def tables_export(self, stream=None):
        import numpy as np
        n = self.cfg.n_classes
        ft = np.empty(n, np.uint32); ts = np.empty(n, np.uint32)
        hot = np.empty(self._c.hot_max, np.int32)
        k = C.c_int32()
        self._ck(self.lib.smtm_tables_export(self._h, _ptr(ft), _ptr(ts), _ptr(hot), C.addressof(k), self._st(stream)))
        return ft, ts, hot[: k.value].copy(), int(k.value)

    def tables_import(self, ft_host=None, ts_host=None, stream=None):
        self._ck(self.lib.smtm_tables_import(self._h, _ptr(ft_host), _ptr(ts_host), self._st(stream)))

    def set_tau(self, tau: float):
        self._ck(self.lib.smtm_set_tau(self._h, float(tau)))

    # -- one batch
    def begin_batch(self, batch: int, stream=None):
        self._ck(self.lib.smtm_begin_batch(self._h, batch, self._st(stream)))

    def encode(self, exit: int, fmap, row_ids=None, sv_out=None, stream=None, dtype=None, H=None, W=None):
        if dtype is None:
            dtype = _dtype_code(fmap)
            H, W = fmap.shape[2], fmap.shape[3]
        self._ck(self.lib.smtm_encode(self._h, exit, _ptr(fmap), dtype, H, W, _ptr(row_ids), _ptr(sv_out),
                                      self._st(stream)))

    def encode_nhwc(self, exit: int, fmap, row_ids=None, sv_out=None, stream=None, dtype=None, H=None, W=None):
        """fmap is [rows, H, W, C] (channels last)."""
        if dtype is None:
            dtype = _dtype_code(fmap)
            H, W = fmap.shape[1], fmap.shape[2]
        self._ck(self.lib.smtm_encode_nhwc(self._h, exit, _ptr(fmap), dtype, H, W, _ptr(row_ids), _ptr(sv_out),
                                           self._st(stream)))

    def lookup(self, exit: int, top_val=None, top_id=None, sims_out=None, stream=None):
        self._ck(self.lib.smtm_lookup(self._h, exit, _ptr(top_val), _ptr(top_id), _ptr(sims_out), self._st(stream)))

    def separability(self, exit: int, sims, sep_out, stream=None):
        self._ck(self.lib.smtm_separability(self._h, exit, _ptr(sims), _ptr(sep_out), self._st(stream)))

    def exit_compact(self, exit: int, exit_ids=None, exit_labels=None, exit_tier=None, n_exit_dev=None,
                     live_ids=None, n_live_dev=None, fmap_in=None, row_ids=None, fmap_out=None,
                     row_bytes: int = 0, stream=None):
        self._ck(self.lib.smtm_exit_compact(self._h, exit, _ptr(exit_ids), _ptr(exit_labels), _ptr(exit_tier),
                                            _ptr(n_exit_dev), _ptr(live_ids), _ptr(n_live_dev), _ptr(fmap_in),
                                            _ptr(row_ids), _ptr(fmap_out), int(row_bytes), self._st(stream)))

    def lookup_exit(self, exit: int, top_val=None, top_id=None, exit_ids=None, exit_labels=None,
                    exit_tier=None, n_exit_dev=None, live_ids=None, n_live_dev=None, fmap_in=None,
                    row_ids=None, fmap_out=None, row_bytes: int = 0, stream=None):
        self._ck(self.lib.smtm_lookup_exit(self._h, exit, _ptr(top_val), _ptr(top_id), _ptr(exit_ids),
                                           _ptr(exit_labels), _ptr(exit_tier), _ptr(n_exit_dev), _ptr(live_ids),
                                           _ptr(n_live_dev), _ptr(fmap_in), _ptr(row_ids), _ptr(fmap_out),
                                           int(row_bytes), self._st(stream)))

    def stage(self, exit: int, fmap, row_ids=None, exit_ids=None, exit_labels=None, exit_tier=None,
              n_exit_dev=None, live_ids=None, n_live_dev=None, fmap_out=None, stream=None,
              dtype=None, H=None, W=None):
        if dtype is None:
            dtype = _dtype_code(fmap)
            H, W = fmap.shape[2], fmap.shape[3]
        self._ck(self.lib.smtm_stage(self._h, exit, _ptr(fmap), dtype, H, W, _ptr(row_ids), _ptr(exit_ids),
                                     _ptr(exit_labels), _ptr(exit_tier), _ptr(n_exit_dev), _ptr(live_ids),
                                     _ptr(n_live_dev), _ptr(fmap_out), self._st(stream)))

    def stage_nhwc(self, exit: int, fmap, row_ids=None, exit_ids=None, exit_labels=None, exit_tier=None,
                   n_exit_dev=None, live_ids=None, n_live_dev=None, fmap_out=None, stream=None,
                   dtype=None, H=None, W=None):
        """fmap is [rows, H, W, C] (channels last)."""
        if dtype is None:
            dtype = _dtype_code(fmap)
            H, W = fmap.shape[1], fmap.shape[2]
        self._ck(self.lib.smtm_stage_nhwc(self._h, exit, _ptr(fmap), dtype, H, W, _ptr(row_ids), _ptr(exit_ids),
                                          _ptr(exit_labels), _ptr(exit_tier), _ptr(n_exit_dev), _ptr(live_ids),
                                          _ptr(n_live_dev), _ptr(fmap_out), self._st(stream)))

    def encode_kernel(self, exit: int) -> str:
        """Name of the kernel instance that the last encode of this exit point launched."""
        return (self.lib.smtm_encode_kernel(self._h, exit) or b"").decode()

    def live_ids(self) -> int:
        """Device address of the context's current live list (int32)."""
        return int(self.lib.smtm_live_ids(self._h) or 0)

    def batch_results(self, exit_layer=None, label=None, tier=None, stream=None):
        self._ck(self.lib.smtm_batch_results(self._h, _ptr(exit_layer), _ptr(label), _ptr(tier), self._st(stream)))

    def read_counts(self, stream=None):
        a, b = C.c_int32(), C.c_int32()
        self._ck(self.lib.smtm_read_counts(self._h, C.addressof(a), C.addressof(b), self._st(stream)))
        return int(a.value), int(b.value)

    def read_stats(self, stream=None):
        import numpy as np
        out = np.zeros((len(self.cfg.dims), 4), np.int32)
        self._ck(self.lib.smtm_read_stats(self._h, _ptr(out), self._st(stream)))
        return out

    # -- between batches
    def cache_update(self, label, stop_layer, batch: int, stream=None):
        self._ck(self.lib.smtm_cache_update(self._h, _ptr(label), _ptr(stop_layer), batch, self._st(stream)))

    def cache_update_static(self, label, stop_layer, batch: int, stream=None):
        self._ck(self.lib.smtm_cache_update_static(self._h, _ptr(label), _ptr(stop_layer), batch, self._st(stream)))
