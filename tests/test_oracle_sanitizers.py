"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): the pins that walk its
index arithmetic hardest -- literal Eq. 3 on rectangular / offset / GQA cases, ragged and empty segments,
chunk splits with length-1 and empty chunks, the packed and the colocated batch -- are rerun in a child
process against a sanitized build of the same source.  An out-of-bounds access, a use of uninitialised
stack memory that trips UBSan, a signed overflow or a misaligned load aborts that process."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PINS = ("literal_eq3 or zero_query or one_hot or chunked_then_merged or merge_identity or varlen or colocated "
        "or ring_schedule or paused_prefill or bf16_bits")


def test_oracle_pins_pass_under_asan_and_ubsan():
    libasan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    if not os.path.isabs(libasan) or not os.path.exists(libasan):
        pytest.skip("gcc has no AddressSanitizer runtime here")
    env = dict(os.environ)
    env["PEC_ORACLE_SANITIZE"] = "1"
    env["LD_PRELOAD"] = libasan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # the interpreter itself is not instrumented: no leak report for it, and no complaint about link order
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                          os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-k", PINS],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    tail = (res.stdout + res.stderr)[-4000:]
    assert res.returncode == 0, tail
    assert "passed" in res.stdout and os.path.exists(os.path.join(ROOT, "oracle", "libpec_oracle_san.so")), tail
