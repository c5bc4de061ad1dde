"""The C oracle under AddressSanitizer + UndefinedBehaviorSanitizer (no GPU): oracle/rt_oracle.c is rebuilt with
-fsanitize=address,undefined and a selection of its pins runs against that build in a child process (gcc's libasan has
to be first among the preloaded libraries, which only a fresh process can arrange).  Any out-of-bounds access, use
after free, signed overflow or misaligned access in the oracle aborts the child."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

PINS = [
    "tests/test_oracle_pins.py::test_p1_single_position_closed_form",
    "tests/test_oracle_pins.py::test_p8_tiled_equals_naive",
    "tests/test_oracle_pins.py::test_p8_chunked_schedule_equals_naive",
    "tests/test_oracle_pins.py::test_p9_update_tile_any_split_any_order_equals_direct_softmax",
    "tests/test_oracle_pins.py::test_p11_prefill_equals_prefill_then_decode",
    "tests/test_oracle_pins.py::test_p13_blocked_recurrence",
    "tests/test_oracle_pins.py::test_transformer_layer_matches_dense_causal_attention",
]


def _existing(pins):
    """Keeps the node ids whose function exists (a renamed pin must not turn this test into a silent no-op)."""
    src = open(os.path.join(ROOT, "tests", "test_oracle_pins.py")).read()
    keep = [p for p in pins if ("def %s(" % p.split("::")[1]) in src]
    return keep


@pytest.mark.slow
def test_oracle_pins_under_address_and_ub_sanitizers(tmp_path):
    from oracle import rt_oracle
    libasan = subprocess.run(["gcc", "-print-file-name=libasan.so"], stdout=subprocess.PIPE, text=True, check=True).stdout.strip()
    if not os.path.isabs(libasan) or not os.path.exists(libasan):
        pytest.skip("gcc has no libasan.so here")
    lib = rt_oracle.build_sanitized(str(tmp_path / "librt_oracle_asan.so"))
    pins = _existing(PINS)
    assert len(pins) == len(PINS), "the selected pins no longer exist: %s" % PINS
    env = dict(os.environ)
    env["RT_ORACLE_LIB"] = lib
    env["LD_PRELOAD"] = libasan + ((" " + env["LD_PRELOAD"]) if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "2"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + pins, cwd=ROOT, env=env,
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-4000:]
    assert "passed" in r.stdout and "ERROR: AddressSanitizer" not in r.stdout and "runtime error" not in r.stdout, r.stdout[-4000:]
