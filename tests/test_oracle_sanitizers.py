"""The oracle's pins once more, with the oracle built under AddressSanitizer and UndefinedBehaviorSanitizer:
an out-of-bounds read or write, a use after free or undefined arithmetic in lsrm_oracle.c fails here even where
it happens not to change a result.  Runs in a child process with the sanitizer runtime preloaded (host code
only; nothing here touches a GPU)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_pins_under_address_and_undefined_behaviour_sanitizers():
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True, check=True).stdout.strip()
    assert os.path.isabs(asan) and os.path.exists(asan), "gcc's AddressSanitizer runtime is not installed"
    env = dict(os.environ)
    env["LSRM_ORACLE_SANITIZE"] = "1"
    # the runtime must come first in the preload list; whatever is preloaded already stays behind it
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # (the interpreter itself is not instrumented: its own allocations at exit are not leaks of the oracle)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    files = [os.path.join(ROOT, "tests", f) for f in ("test_oracle_routing.py", "test_oracle_route3d.py",
                                                       "test_oracle_attention.py")]
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *files],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (run.stdout + run.stderr)[-3000:]
    assert run.returncode == 0, tail
    assert "passed" in run.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail
