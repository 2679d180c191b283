"""CPU-side checks of the C-ABI library: it loads without a GPU, exports every symbol the
header declares, and rejects bad arguments before any GPU call.  No compute is launched."""
import ctypes as C
import re
from pathlib import Path

import pytest

from paper_2112_02644_amd import smtm

ROOT = Path(__file__).resolve().parent.parent
HEADER = (ROOT / "include" / "smtm.h").read_text()


def declared_functions():
    body = re.sub(r"/\*.*?\*/", "", HEADER, flags=re.S)
    names = re.findall(r"\b(smtm_[a-z_0-9]+)\s*\(", body)
    return sorted(set(names))


def test_header_declares_the_four_core_calls():
    names = declared_functions()
    for must in ("smtm_encode", "smtm_lookup", "smtm_exit_compact", "smtm_cache_update"):
        assert must in names
    assert len(names) >= 15


def test_library_loads_and_exports_every_declared_symbol():
    lib = smtm.load_library()
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} is declared in smtm.h but not exported"
    assert lib.smtm_version() >= 100


def test_binding_covers_every_declared_symbol():
    methods = {m for m in dir(smtm.Smtm)}
    skip = {"smtm_create", "smtm_destroy", "smtm_last_error", "smtm_version", "smtm_build_id"}
    for name in declared_functions():
        if name in skip:
            continue
        assert name[len("smtm_"):] in methods, f"no binding method for {name}"


def test_config_struct_matches_header_layout():
    # 4 + 4 + 8*4 + 4*5 + 4 (float) + 4*6 = 88 bytes, all 4-byte fields in header order
    assert C.sizeof(smtm._Config) == 88
    fields = [f[0] for f in smtm._Config._fields_]
    header_fields = re.findall(r"^\s+(?:int32_t|float)\s+([a-z_, ]+?)(?:\[SMTM_MAX_EXITS\])?;", HEADER, flags=re.M)
    flat = [x.strip() for grp in header_fields for x in grp.split(",")]
    assert flat == fields


BAD = [
    (dict(n_classes=1), 1), (dict(n_classes=20000), 1), (dict(dims=[]), 1), (dict(dims=[4] * 9), 1),
    (dict(dims=[0]), 2), (dict(max_batch=0), 1), (dict(max_batch=70000), 1),
    (dict(hot_init=1, hot_min=1), 1), (dict(hot_min=5, hot_init=4), 1), (dict(hot_max=3, hot_init=4), 1),
    (dict(hot_max=11), 1), (dict(tiers=3), 1), (dict(tau=-1.0), 1), (dict(tau=float("nan")), 1),
    (dict(window=0), 1), (dict(cl_num=0), 1), (dict(cl_num=21, cl_den=20), 1), (dict(init_count=-1), 1),
    (dict(score_path=7), 1), (dict(forgetting=2), 1),
]


@pytest.mark.parametrize("override,code", BAD)
def test_bad_config_is_rejected_before_any_gpu_call(override, code):
    base = dict(n_classes=10, dims=[8, 16], max_batch=4, hot_init=4, hot_min=2, hot_max=8)
    base.update(override)
    cfg = smtm.SmtmConfig(**base)
    if len(cfg.dims) > 8:
        c = cfg.to_c(); c.n_exits = 9
        lib = smtm.load_library()
        h = C.c_void_p()
        assert lib.smtm_create(C.byref(h), C.byref(c)) == code and not h
        return
    with pytest.raises(smtm.SmtmError) as e:
        smtm.Smtm(cfg)
    assert e.value.code == code
    assert smtm.load_library().smtm_last_error(None)


def test_null_arguments():
    lib = smtm.load_library()
    assert lib.smtm_create(None, None) == 1
    h = C.c_void_p()
    assert lib.smtm_create(C.byref(h), None) == 1
    assert lib.smtm_destroy(None) == 0
    assert lib.smtm_begin_batch(None, 4, None) == 1
    assert lib.smtm_encode(None, 1, None, 0, 1, 1, None, None, None) == 1
    assert lib.smtm_lookup(None, 1, None, None, None, None) == 1
    assert lib.smtm_cache_update(None, None, None, 1, None) == 1
    assert lib.smtm_live_ids(None) is None
