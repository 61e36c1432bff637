"""The oracle's pins once more, against the oracle built with AddressSanitizer and UBSan (host code only): an
out-of-bounds access, a signed overflow or a bad shift anywhere in oracle/fxp_ref.cpp ends that run with a
report instead of passing by luck.  Runs in a child process, because the sanitizer runtime has to be the first
library a process loads."""
import os
import subprocess
import sys

from oracle import build as oracle_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_FILES = ["test_oracle_scale.py", "test_oracle_map.py", "test_oracle_philox.py", "test_oracle_gemm.py",
             "test_oracle_unmap.py", "test_oracle_layer.py", "test_oracle_conv.py", "test_oracle_bmm.py",
             "test_oracle_sgd16.py"]


def test_pins_pass_under_address_and_undefined_behaviour_sanitizers():
    oracle_build.build(force=True, sanitize=True)
    env = dict(os.environ)
    inherited = env.get("LD_PRELOAD", "")
    env["LD_PRELOAD"] = oracle_build.sanitizer_runtime() + (":" + inherited if inherited else "")
    env["FXP_REF_SANITIZE"] = "1"
    # the interpreter's own allocations are not the subject; findings in the oracle abort the run
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu"] + \
          [os.path.join(ROOT, "tests", f) for f in PIN_FILES]
    res = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=1500)
    tail = (res.stdout + res.stderr)[-4000:]
    assert res.returncode == 0, tail
    assert " passed" in res.stdout and "failed" not in res.stdout, tail
