"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer, on the CPU: the oracle (every function, edge
cases included) and the library's host side (configuration checks, NULL handles, clean-up of a failed creation).
Both are small C drivers built against sanitizer builds of the code under test; any report ends the driver
with a non-zero status."""
import os
import subprocess
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
TESTS = ROOT / "tests"
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def _run(exe, cwd):
    r = subprocess.run([str(exe)], cwd=str(cwd), env=ENV, capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, f"{exe.name} failed ({r.returncode}):\n{r.stdout}\n{r.stderr[-4000:]}"
    assert "all checks hold" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = tmp_path / "oracle_san"
    subprocess.run(["gcc", "-std=c11", "-fopenmp", *SAN, "-o", str(exe), str(ROOT / "oracle" / "smtm_oracle.c"),
                    str(TESTS / "oracle_sanitize_driver.c"), "-lm"], check=True)
    _run(exe, tmp_path)


def test_library_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    from paper_2112_02644_amd import build as B
    clang = Path("/opt/rocm/llvm/bin/clang")
    if not clang.exists():
        pytest.skip("ROCm's clang (for the driver's sanitizer runtime) is not at /opt/rocm/llvm/bin/clang")
    lib = tmp_path / "libsmtm_san.so"
    flags = [f for f in B.FLAGS if f != "-O3"]
    host_san = []
    for f in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all"):
        host_san += ["-Xarch_host", f]                 # the sanitizers go to the host pass only
    subprocess.run([B.hipcc(), *flags, "-O1", "-g", *host_san, "-o", str(lib)] + [str(B.CSRC / s) for s in B.SOURCES],
                   check=True, capture_output=True)
    exe = tmp_path / "abi_san"
    subprocess.run([str(clang), *SAN, "-o", str(exe), str(TESTS / "abi_sanitize_driver.c"), str(lib),
                    f"-Wl,-rpath,{tmp_path}"], check=True)
    _run(exe, tmp_path)
