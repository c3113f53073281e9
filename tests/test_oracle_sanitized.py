"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer: the whole pin set (every
layout, dtype, subset and degenerate case the pins feed it) runs once more in a child process
against a build of oracle/lamina_oracle.c with -fsanitize=address,undefined, where any
out-of-bounds access, misaligned or overflowing arithmetic aborts the run.  CPU only."""
import ctypes
import os
import subprocess
import sys

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_pin_set_is_clean_under_address_and_undefined_behaviour_sanitizers():
    lib = oracle.build(sanitize=True)
    probe = ("import ctypes, oracle; l = oracle._load(); "
             "assert oracle.sanitized() and getattr(l, '__asan_init') is not None; "
             "print('sanitized oracle loaded:', l._name)")
    env = oracle.sanitizer_env()
    res = subprocess.run([sys.executable, "-c", probe], cwd=ROOT, env=env, capture_output=True,
                         text=True, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert os.path.basename(lib) in res.stdout
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                          os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                          os.path.join(ROOT, "tests", "test_workloads.py")],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    text = res.stdout + res.stderr
    assert res.returncode == 0, text[-4000:]
    assert "AddressSanitizer" not in text and "runtime error" not in text, text[-4000:]
    assert " passed" in text


def test_the_plain_build_is_not_the_sanitized_one():
    # the parity tests and the benchmark's CPU baseline use the plain -O2 build
    assert not oracle.sanitized()
    assert not hasattr(ctypes.CDLL(oracle.build()), "__asan_init")
