"""The CPU checker once more under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU).

oracle.c is rebuilt with both sanitizers and its own pins are run against that build in a child
process (the sanitizer runtime has to be the first library the process loads, so it is preloaded
there).  An out-of-bounds access, a signed overflow or a misaligned load anywhere in the checker
aborts the child."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_checker_pins_hold_under_sanitizers():
    sys.path.insert(0, ROOT)
    from oracle.build import build, sanitizer_runtime
    build(sanitize=True)
    runtime = sanitizer_runtime()
    assert os.path.exists(runtime), "gcc ships no AddressSanitizer runtime here"
    env = dict(os.environ)
    env["ORACLE_SANITIZED"] = "1"
    env["LD_PRELOAD"] = ":".join(x for x in (runtime, env.get("LD_PRELOAD", "")) if x)
    # the interpreter and numpy are not instrumented: their allocations are not this test's business
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                          os.path.join(ROOT, "tests", "test_oracle_matching.py"),
                          os.path.join(ROOT, "tests", "test_oracle_scorer.py")],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    assert run.returncode == 0, run.stdout[-3000:] + run.stderr[-3000:]
    assert "passed" in run.stdout
