"""Host-side sanitizer leg: the checker's pins run once more against a build of sr_oracle.c that is
instrumented with AddressSanitizer and UndefinedBehaviorSanitizer (-O1, errors abort).

The instrumented library needs the sanitizer runtime to be the first library of the process, so the pins
run in a child interpreter that is started with the runtime preloaded (in front of whatever the
environment already preloads) and with SRO_SANITIZE=1, which makes `oracle.load()` take the instrumented
build.  An out-of-bounds table access in the edit distance, a read past a prefix in the signals, a stale
K/V pointer or a signed overflow in the exact-compare arithmetic would end the child with a report.
"""
import os
import subprocess
import sys

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PINS = ["tests/test_oracle_gate.py", "tests/test_oracle_signals.py", "tests/test_oracle_logprob.py",
        "tests/test_oracle_decoder.py", "tests/test_oracle_contract.py"]


def test_pins_pass_under_address_and_undefined_behaviour_sanitizers():
    oracle.build(sanitize=True)
    env = dict(os.environ)
    runtime = oracle.sanitizer_runtime()
    assert os.path.isabs(runtime) and os.path.exists(runtime), "gcc's libasan.so not found"
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=97"     # the interpreter itself leaks by design
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["SRO_SANITIZE"] = "1"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + PINS, cwd=ROOT, env=env,
                       capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "failed" not in r.stdout, tail
    assert "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail


def test_the_child_really_loads_the_instrumented_build():
    env = dict(os.environ)
    env["LD_PRELOAD"] = oracle.sanitizer_runtime() + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0"
    env["SRO_SANITIZE"] = "1"
    code = ("import oracle, sys; L = oracle.load(); "
            "maps = open('/proc/self/maps').read(); "
            "sys.exit(0 if '_san_' in maps and oracle.lev([1, 2, 3], [1, 3]) == 1 else 5)")
    r = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, (r.stdout + r.stderr)[-2000:]
