"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: oracle/jfa_oracle.c is compiled with
-fsanitize=address,undefined (any finding aborts) and the brute-force, library, finite-difference, stability and
guard-row pins run through that build.  Host code only."""
import os
import subprocess
import sys

import pytest

import oracle_variants as ov


def test_oracle_pins_under_asan_and_ubsan(tmp_path):
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("gcc has no libasan.so here")
    lib = ov.compile_oracle(ov.ORACLE_SRC, str(tmp_path / "liboracle_san.so"),
                            ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"])
    env = dict(os.environ)
    # the sanitizer runtime has to come first among the preloaded libraries; whatever was preloaded stays behind it
    env["LD_PRELOAD"] = " ".join(x for x in (asan, env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "2"
    r = subprocess.run([sys.executable, os.path.join(os.path.dirname(__file__), "oracle_variants.py"), lib,
                        "test_p1_", "test_p2_", "test_p2b_", "test_p5_", "test_p9_", "test_p10", "test_p11_", "test_pairs_"],
                       capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0 and "PINS PASSED" in r.stdout, f"stdout:\n{r.stdout[-3000:]}\nstderr:\n{r.stderr[-3000:]}"
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-3000:]
