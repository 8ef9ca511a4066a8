"""The oracle's pins once more, against the AddressSanitizer + UndefinedBehaviorSanitizer build of the oracle
(CPU only): an out-of-bounds access, a use after free, a signed overflow or a misaligned access anywhere in the
checker stops the child run at once.  The child is a separate interpreter because the sanitizer runtime has to be
loaded before anything else."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_pins_pass_under_address_and_ub_sanitizers():
    from oracle import build_oracle
    lib = build_oracle.build(force=True, sanitize=True)
    assert os.path.exists(lib)
    runtime = subprocess.run(["g++", "-print-file-name=libasan.so"], check=True, capture_output=True,
                             text=True).stdout.strip()
    assert os.path.isabs(runtime) and os.path.exists(runtime), runtime
    env = dict(os.environ)
    env["COMPAMS_ORACLE_SANITIZE"] = "1"
    env["LD_PRELOAD"] = " ".join(x for x in (runtime, env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"       # the interpreter itself leaks by design
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                        os.path.join(ROOT, "tests", "test_oracle_wire.py")],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "failed" not in r.stdout, tail
    assert "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail
