"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU): a small C
program that includes the oracle's source calls every entry point on exactly-sized heap buffers; any access
past a buffer, leak, or undefined arithmetic fails the run.  Built once per input type, run in a subprocess."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("ctype", ["double", "float"])
def test_oracle_runs_clean_under_address_and_undefined_sanitizers(tmp_path, ctype):
    exe = os.path.join(str(tmp_path), f"oracle_san_{ctype}")
    cmd = ["gcc", "-O1", "-g", "-std=gnu99", "-fopenmp", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-static-libasan", f"-DCPO_IN_T={ctype}", f"-DCPO_PREFIX=cpo_san_",
           "-I", os.path.join(ROOT, "oracle"), os.path.join(ROOT, "tests", "oracle_sanitizer_main.c"), "-o", exe, "-lm"]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, OMP_NUM_THREADS="3", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert res.returncode == 0, res.stderr[-4000:]
    assert "ok" in res.stdout
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr[-4000:]
