"""The oracle's pins once more against a build of oracle.c with -fsanitize=address,undefined (CPU only).

The sanitizer runtime has to be in the process before Python starts, so the pins run in a child process that
preloads it (in front of whatever the environment preloads already); ORACLE_SANITIZED=1 makes the oracle's loader
build and load the instrumented library.  An out-of-bounds access, a signed overflow or a misaligned pointer
anywhere in the oracle aborts the child.
"""
import glob
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_pins_pass_under_address_and_undefined_behaviour_sanitizers():
    asan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    assert os.path.isabs(asan) and os.path.exists(asan), "gcc has no AddressSanitizer runtime"
    env = dict(os.environ)
    env["ORACLE_SANITIZED"] = "1"
    env["LD_PRELOAD"] = ":".join(x for x in (asan, env.get("LD_PRELOAD", "")) if x)
    # Python's own allocations are not the subject; the runtime need not be first if something else is preloaded
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "2"
    pins = sorted(glob.glob(os.path.join(ROOT, "tests", "test_oracle_*.py")))
    pins = [p for p in pins if not p.endswith("test_oracle_sanitized.py")]
    assert len(pins) >= 8
    check = ("import oracle, sys; assert oracle.SANITIZED and oracle.lib()._name.endswith('liboracle_san.so'); "
             "import pytest; sys.exit(pytest.main(['-x', '-q', '-p', 'no:cacheprovider'] + sys.argv[1:]))")
    r = subprocess.run([sys.executable, "-c", check] + pins, cwd=ROOT, env=env, stdout=subprocess.PIPE,
                       stderr=subprocess.STDOUT, text=True, timeout=900)
    assert r.returncode == 0, r.stdout[-4000:]
    assert " passed" in r.stdout and "ERROR: AddressSanitizer" not in r.stdout and "runtime error" not in r.stdout
