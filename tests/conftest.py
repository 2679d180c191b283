import os
import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    # SMTM_ORACLE_LIB swaps the checker for a deliberately broken build (tests/test_oracle_mutations.py runs the
    # pins against it in a child process).  A GPU parity test must never be judged by such a build.
    if os.environ.get("SMTM_ORACLE_LIB") and any("gpu" in item.keywords for item in items):
        raise pytest.UsageError("SMTM_ORACLE_LIB is set: GPU parity tests only run against the oracle built from "
                                "oracle/smtm_oracle.c")
    # GPU tests are skipped (not failed) where no GPU is visible and -m gpu was not asked for.
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)
