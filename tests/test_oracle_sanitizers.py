"""Host sanitizers on the oracle (CPU only): AddressSanitizer + UndefinedBehaviorSanitizer on a C driver that
reaches every oracle function and its edge cases, and the oracle's own pin tests once more on a library built
with the undefined-behaviour sanitizer."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE = os.path.join(ROOT, "oracle")


def test_driver_is_clean_under_asan_and_ubsan(tmp_path):
    cc = shutil.which("gcc")
    if cc is None:
        pytest.skip("no gcc")
    exe = tmp_path / "sanitize_driver"
    # the sanitizer runtime is linked statically: nothing has to be preloaded into the process
    subprocess.run([cc, "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
                    os.path.join(ORACLE, "sanitize_driver.c"), os.path.join(ORACLE, "atomo_oracle.c"), "-lm",
                    "-o", str(exe)], check=True)
    run = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, run.stderr[-2000:]
    assert "clean" in run.stdout and "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr


def test_pins_pass_on_a_ubsan_build_of_the_oracle():
    env = dict(os.environ, ATOMO_ORACLE_SANITIZE="undefined")
    pins = [os.path.join(ROOT, "tests", name) for name in
            ("test_oracle_philox.py", "test_oracle_probabilities.py", "test_oracle_svd.py", "test_oracle_lq.py")]
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *pins],
                         capture_output=True, text=True, env=env, cwd=ROOT, timeout=900)
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-2000:]
    assert "runtime error" not in run.stderr
