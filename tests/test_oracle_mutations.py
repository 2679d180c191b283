"""The pins must notice a broken oracle: each planted mistake (a dropped term, a wrong sign, index or
bound) is compiled into a scratch copy of the C oracle on the CPU, and the pin tests are run against
it in a child process.  Every mutant has to fail at least one pin; the untouched source has to pass."""
import os
import subprocess
import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
SRC = (ROOT / "oracle" / "smtm_oracle.c").read_text()

MUTANTS = [
    ("mean -> sum", "acc / (double)HW", "acc"),
    ("norm of v taken from the wrong operand", "dot += v[k] * c[k];\n        vv += v[k] * v[k];",
     "dot += v[k] * c[k];\n        vv += v[k] * c[k];"),
    ("weight 2^l instead of 2^(l-1)", "return ldexp(1.0, l - 1);", "return ldexp(1.0, l);"),
    ("SA overwritten instead of accumulated", "sa[j] += s * w;", "sa[j] = s * w;"),
    ("tie broken towards the larger id", "x > best || (x == best && j < best_id)",
     "x > best || (x == best && j > best_id)"),
    ("threshold not strict", "return (SA_H - SA_SH) > tau * runner;", "return (SA_H - SA_SH) >= tau * runner;"),
    ("frames with nothing matching may exit", "if (!(SA_H > 0.0)) return 0;\n    if (SA_SH == -INFINITY)",
     "if (SA_SH == -INFINITY)"),
    ("tier 2 overrides tier 1", "if (d == 0 && orc_exit_predicate(h2, sh2, tau)) { d = 2; lab = id2; }",
     "if (orc_exit_predicate(h2, sh2, tau)) { d = 2; lab = id2; }"),
    ("fast memory ignored", "orc_top2(sa, hot_ids, k, &h1, &id1, &sh1);", "orc_top2(sa, NULL, k, &h1, &id1, &sh1);"),
    ("decay by 2 instead of 4", "return (uint64_t)FT << (2 * (ORC_QMAX - q));",
     "return (uint64_t)FT << (1 * (ORC_QMAX - q));"),
    ("ceil instead of floor in the exponent", "uint32_t q = TS / W;\n    if (q > ORC_QMAX)",
     "uint32_t q = (TS + W - 1) / W;\n    if (q > ORC_QMAX)"),
    ("confidence level must be exceeded", "if (part * cl_den >= total * cl_num) { k = i + 1; break; }",
     "if (part * cl_den > total * cl_num) { k = i + 1; break; }"),
    ("running mean divides by m + 2", "sc[c] = (sc[c] * mm + sv[c]) / (mm + 1.0);",
     "sc[c] = (sc[c] * mm + sv[c]) / (mm + 2.0);"),
    ("Eq. 7 stops one exit point early", "for (int l0 = 1; l0 <= l; ++l0) {", "for (int l0 = 1; l0 < l; ++l0) {"),
    ("in-place forgetting halves", "if (TS[i] % W == 0) FT[i] /= 4;", "if (TS[i] % W == 0) FT[i] /= 2;"),
    ("fp16 exponent bias off by one", "expo - 15);", "expo - 14);"),
    ("tolerance scale loses its absolute values", "dot += fabs(v[k] * c[k]);", "dot += v[k] * c[k];"),
    ("tolerance scale ten times too large", "dot += fabs(v[k] * c[k]);\n        vv += v[k] * v[k];",
     "dot += fabs(v[k] * c[k]);\n        vv += 0.01 * v[k] * v[k];"),
    ("compaction keeps slots instead of frame ids", "live_ids[nl] = frame_ids[i];", "live_ids[nl] = (int32_t)i;"),
]


def _run_pins(tmp_path, source, tag):
    c = tmp_path / f"oracle_{tag}.c"
    so = tmp_path / f"liboracle_{tag}.so"
    c.write_text(source)
    subprocess.run(["gcc", "-O1", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", str(so), str(c), "-lm"], check=True)
    env = dict(os.environ, SMTM_ORACLE_LIB=str(so))
    r = subprocess.run([sys.executable, "-m", "pytest", str(ROOT / "tests" / "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], env=env, capture_output=True, text=True, cwd=str(ROOT))
    return r.returncode


def test_untouched_oracle_passes_in_the_child_process(tmp_path):
    assert _run_pins(tmp_path, SRC, "clean") == 0


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_notice_a_planted_mistake(tmp_path, name, old, new):
    assert SRC.count(old) >= 1, "the oracle no longer contains the text this mutant replaces"
    assert _run_pins(tmp_path, SRC.replace(old, new, 1), "mut") != 0, f"no pin noticed: {name}"
