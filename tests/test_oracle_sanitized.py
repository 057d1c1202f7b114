"""The oracle's pins once more against a build of the same C source with gcc's address and
undefined-behaviour sanitizers (host code only): a read past a buffer or an overflowing index in
the oracle aborts the child process instead of producing a plausible number."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_pins_pass_under_address_and_undefined_sanitizers():
    sys.path.insert(0, ROOT)
    import oracle
    lib = oracle.build_sanitized()
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True,
                          text=True).stdout.strip()
    assert os.path.isabs(asan), "gcc has no address-sanitizer runtime"
    env = dict(os.environ)
    # the interpreter is not instrumented, so the runtime has to be loaded first; whatever the
    # environment preloads already stays behind it
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["FSK_ORACLE_LIB"] = lib
    env["OMP_NUM_THREADS"] = "4"
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                          os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    assert run.returncode == 0, run.stdout[-3000:] + run.stderr[-3000:]
    assert " passed" in run.stdout
