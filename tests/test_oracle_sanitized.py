"""The oracle's C file under AddressSanitizer + UndefinedBehaviorSanitizer: every pin of
tests/test_oracle_pins.py is run once more, in a child process, against a build of
oracle/longflow_oracle.c with -fsanitize=address,undefined in which any report aborts.
CPU only; the HIP library is not involved."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_oracle_pin_passes_under_address_and_undefined_behaviour_sanitizers():
    from oracle import longflow_oracle as oracle
    lib = oracle.build(force=True, sanitize=True)
    syms = subprocess.run(["nm", "-D", lib], capture_output=True, text=True, check=True).stdout
    assert "__asan_init" in syms and "__ubsan_handle" in syms          # the instrumentation is really in
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True, check=True).stdout.strip()
    assert os.path.isabs(asan), "gcc has no libasan"
    env = dict(os.environ)
    env["LFO_SANITIZE"] = "1"
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:halt_on_error=1"   # the interpreter's own leaks are not the subject
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert " passed" in r.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail
