"""The oracle's pins once more against a build of oracle/moe_oracle.c with AddressSanitizer and
UndefinedBehaviorSanitizer (host code only, no GPU): an out-of-bounds index, a signed overflow or a
misaligned access anywhere in the checker aborts the child process."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_FILES = ["tests/test_oracle_routing.py", "tests/test_oracle_numerics.py", "tests/test_oracle_adamw.py",
             "tests/test_oracle_dtd.py"]


@pytest.mark.skipif(os.environ.get("MOE_ORACLE_SANITIZE") == "1", reason="already inside the sanitized run")
def test_oracle_pins_under_asan_and_ubsan():
    from oracle import moe_oracle
    moe_oracle.build_sanitized()
    runtime = moe_oracle.sanitizer_runtime()
    if not os.path.isabs(runtime) or not os.path.exists(runtime):
        pytest.skip("gcc has no AddressSanitizer runtime here")
    env = dict(os.environ)
    env["MOE_ORACLE_SANITIZE"] = "1"
    pre = env.get("LD_PRELOAD", "")
    env["LD_PRELOAD"] = runtime + ((":" + pre) if pre else "")       # the sanitizer runtime must come first
    # the interpreter itself is not instrumented: its exit-time "leaks" are not the oracle's
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["OMP_NUM_THREADS"] = "4"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *PIN_FILES], cwd=ROOT, env=env,
                       capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "failed" not in r.stdout, tail
    # the sanitized library is the one such a process maps, and the sanitizer is live in it: an output
    # array one element too short (a mistake planted here, on the CPU) must abort the child
    probe = ("import numpy as np, ctypes as C\n"
             "from oracle import moe_oracle as o\n"
             "L = o.lib()\n"
             "assert 'libmoe_oracle_san.so' in open('/proc/self/maps').read()\n"
             "z = np.zeros(64); g = np.zeros(%d)\n"
             "L.orc_act_grad_array(64, z.ctypes.data, g.ctypes.data, 0)\n"
             "print('survived')\n")
    ok = subprocess.run([sys.executable, "-c", probe % 64], cwd=ROOT, env=env, capture_output=True, text=True, timeout=120)
    assert ok.returncode == 0 and "survived" in ok.stdout, ok.stderr[-2000:]
    bad = subprocess.run([sys.executable, "-c", probe % 63], cwd=ROOT, env=env, capture_output=True, text=True, timeout=120)
    assert bad.returncode != 0 and "AddressSanitizer" in bad.stderr and "survived" not in bad.stdout
