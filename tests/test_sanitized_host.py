"""Host halves under AddressSanitizer + UndefinedBehaviorSanitizer (opt-in: PTQ4VM_SANITIZE=1; the sanitized build of
the HIP sources takes about two minutes).  The C ABI's host code (argument checks, launch set-up, status strings)
is built with clang's sanitizers and tests/test_abi_host.py runs against it; the CPU oracle is built with gcc's
and its pins run against it.  Each run is a child process with the matching sanitizer runtime preloaded; any
report makes the run fail (halt_on_error)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
pytestmark = pytest.mark.skipif(os.environ.get("PTQ4VM_SANITIZE") != "1", reason="opt-in: set PTQ4VM_SANITIZE=1")


def _run(tests, runtime, extra_env):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1", **extra_env)
    env["LD_PRELOAD"] = " ".join(v for v in (env.get("LD_PRELOAD"), runtime) if v)
    env.pop("PTQ4VM_SANITIZE")  # the child must not recurse into this file
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", *tests], cwd=ROOT, env=env, capture_output=True, text=True)
    out = res.stdout + res.stderr
    assert res.returncode == 0 and "AddressSanitizer" not in out and "runtime error:" not in out, out[-4000:]


def test_c_abi_host_code_under_sanitizers():
    from paper_2412_20386_amd import build

    lib = build.build_sanitized()
    _run(["tests/test_abi_host.py"], build.sanitizer_runtime(), {"PTQ4VM_LIB": lib})


def test_oracle_under_sanitizers():
    import oracle.ptq4vm_oracle as oracle_c

    lib = oracle_c.build_sanitized()
    runtime = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True, check=True).stdout.strip()
    _run(["tests/test_oracle_pins.py", "tests/test_oracle_pins_widened.py"], runtime, {"PTQ4VM_ORACLE_LIB": lib})
