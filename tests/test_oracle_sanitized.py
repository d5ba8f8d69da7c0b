"""The oracle's C source under AddressSanitizer and UndefinedBehaviorSanitizer: every pin of
tests/test_oracle_pins.py is run once more, in a child process, against a sanitized build of
oracle/sgc_oracle.c (any out-of-bounds access, use after free, signed overflow or misaligned access in
the oracle aborts the child). CPU only."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_pins_pass_under_address_and_undefined_behaviour_sanitizers():
    from oracle import oracle as orc

    so = orc.build_sanitized()
    asan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    assert os.path.isabs(asan) and os.path.exists(asan), "gcc's libasan.so not found"
    env = dict(os.environ)
    env["SGC_ORACLE_LIB"] = so
    # the sanitizer runtime must come first among the preloaded libraries; whatever is preloaded already stays
    env["LD_PRELOAD"] = asan + ((":" + env["LD_PRELOAD"]) if env.get("LD_PRELOAD") else "")
    # python itself is not instrumented: its (intentional) leaks at exit are not findings of the oracle
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                          os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (run.stdout + run.stderr)[-3000:]
    assert run.returncode == 0, tail
    assert " passed" in run.stdout and "failed" not in run.stdout, tail
