"""Two checks of the checker itself (CPU only).

1. The C oracle built with AddressSanitizer + UndefinedBehaviorSanitizer passes its pins: no out-of-bounds
   access, no signed overflow, no misaligned access behind the numbers the GPU path is compared with.
2. Planted mistakes: the kind of slip a plausible re-typing of the oracle could contain (a dropped rounding
   term, a swapped operand, a transposed index, floor for ceiling ...).  Each edited copy of the source is
   compiled and the pins are run against it; every one of them must fail at least one pin.  The product path
   is not involved: the mistakes live in copies of oracle/blast_oracle.c only.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

from oracle import build as oracle_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PINS = os.path.join(ROOT, "tests", "test_oracle_pins.py")


def run_pins(lib_path, extra_env=None, stop_early=True):
    env = dict(os.environ)
    env["BLAST_ORACLE_LIB"] = lib_path
    env.update(extra_env or {})
    cmd = [sys.executable, "-m", "pytest", PINS, "-q", "-p", "no:cacheprovider"] + (["-x"] if stop_early else [])
    return subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True)


def test_pins_pass_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    lib = oracle_build.build_variant(str(tmp_path / "liboracle_san.so"), sanitize=True)
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("gcc ships no libasan here")
    preload = asan + (":" + os.environ["LD_PRELOAD"] if os.environ.get("LD_PRELOAD") else "")
    res = run_pins(lib, {"LD_PRELOAD": preload, "ASAN_OPTIONS": "detect_leaks=0:abort_on_error=1",
                         "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1", "OMP_NUM_THREADS": "4"}, stop_early=False)
    assert res.returncode == 0, res.stdout[-3000:] + res.stderr[-3000:]
    assert "AddressSanitizer" not in res.stderr and "runtime error" not in res.stderr, res.stderr[-3000:]


# (what the slip is, text in oracle/blast_oracle.c, replacement)
PLANTED = [
    ("ties keep the higher index", "if (a->idx < b->idx) return -1;", "if (a->idx < b->idx) return 1;"),
    ("drop count by floor instead of ceiling", "(s_bp * n_blocks + 9999) / 10000", "(s_bp * n_blocks) / 10000"),
    ("bf16 rounding half away from zero instead of half to even", "u += 0x7FFFu + lsb;", "u += 0x8000u;"),
    ("sign of the exponent in SiLU", "case 0: return g / (1.0 + exp(-g));", "case 0: return g / (1.0 + exp(g));"),
    ("blocks unpacked transposed", "= vals[(k * b + i) * b + j];", "= vals[(k * b + j) * b + i];"),
    ("row schedule not stable for equal counts", "if (row_ptr[q + 1] - row_ptr[q] >= cnt) break;",
     "if (row_ptr[q + 1] - row_ptr[q] > cnt) break;"),
    ("H read with the strides of the other layout", "d_vals, H, T, 1, T, Y);", "d_vals, H, 1, T, T, Y);"),
    ("activation applied to the up projection", "double h = oracle_act(act, G[p]) * U[p];",
     "double h = oracle_act(act, U[p]) * G[p];"),
    ("block score by absolute sum instead of sum of squares", "s += w * w;", "s += fabs(w);"),
    ("lowest scores kept instead of highest", "if (a->score > b->score) return -1;", "if (a->score > b->score) return 1;"),
]


def test_every_planted_mistake_fails_a_pin(tmp_path):
    text = open(oracle_build.SRC).read()
    libs = []
    for i, (what, old, new) in enumerate(PLANTED):
        assert text.count(old) == 1, f"anchor of planted mistake {i} ({what}) not found exactly once"
        libs.append(oracle_build.build_variant(str(tmp_path / f"liboracle_m{i}.so"), source_text=text.replace(old, new)))
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(lambda l: run_pins(l, {"OMP_NUM_THREADS": "2"}), libs))
    survivors = [PLANTED[i][0] for i, r in enumerate(results) if r.returncode == 0]
    assert not survivors, "no pin notices: " + "; ".join(survivors)
    # and the failures are test failures, not crashes of the runner
    for i, r in enumerate(results):
        assert "failed" in r.stdout or "error" in r.stdout.lower(), (PLANTED[i][0], r.stdout[-500:])
