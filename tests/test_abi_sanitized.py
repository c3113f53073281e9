"""The HOST half of the HIP library under AddressSanitizer and UndefinedBehaviorSanitizer: the
library is built once more with the sanitizers applied to host code only (the device code is
compiled as always), and the tests that exercise its argument checks, configuration checks and
workspace arithmetic without a GPU run against that build in a child process, where any
out-of-bounds access, use after free or overflowing arithmetic in the library's host code
aborts the run.  CPU only."""
import os
import subprocess
import sys

from paper_2405_01814_amd import lamina

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_code_is_clean_under_address_and_undefined_behaviour_sanitizers():
    env = lamina.host_sanitizer_env()
    probe = ("import ctypes; from paper_2405_01814_amd import lamina; l = lamina.load(); "
             "assert lamina.host_sanitized() and l._name == lamina.HOSTSAN_LIB_PATH; "
             "print('loaded', l._name)")
    res = subprocess.run([sys.executable, "-c", probe], cwd=ROOT, env=env, capture_output=True,
                         text=True, timeout=900)
    assert res.returncode == 0, (res.stdout + res.stderr)[-4000:]
    assert os.path.basename(lamina.HOSTSAN_LIB_PATH) in res.stdout
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                          os.path.join(ROOT, "tests", "test_abi.py")],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    text = res.stdout + res.stderr
    assert res.returncode == 0, text[-4000:]
    assert "AddressSanitizer" not in text and "runtime error" not in text, text[-4000:]
    assert " passed" in text


def test_the_ordinary_build_is_not_the_sanitized_one():
    assert not lamina.host_sanitized()
    assert lamina.load()._name == lamina.LIB_PATH
