"""The oracle's pins once more against a build of oracle/socket_oracle.c under AddressSanitizer
and UndefinedBehaviorSanitizer (host code, CPU only): an out-of-bounds index, a signed overflow
or a misaligned access in the reference would otherwise go unnoticed as long as its results
look right."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

from oracle import build as oracle_build  # noqa: E402


def test_oracle_pins_pass_under_address_and_undefined_behaviour_sanitizers():
    lib = oracle_build.build_sanitized()
    runtime = oracle_build.sanitizer_runtime()
    assert os.path.isabs(runtime) and os.path.exists(runtime), "gcc's libasan.so not found"
    env = dict(os.environ)
    env["SOCKET_ORACLE_LIB"] = lib
    env["LD_PRELOAD"] = " ".join(x for x in (runtime, env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=97"   # the interpreter's own leaks are not ours
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1:exitcode=98"
    env["OMP_NUM_THREADS"] = "1"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=900)
    assert r.returncode == 0, r.stdout[-4000:]
    assert "passed" in r.stdout and "AddressSanitizer" not in r.stdout and "runtime error" not in r.stdout, r.stdout[-4000:]
