"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer on the host: a C driver calls every entry point
with small random shapes (column remap, warm-up, all generator modes, sparse lists with repeats, the two comparison
methods).  Any out-of-bounds access, leak or undefined operation makes the run fail."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitized")
    build = subprocess.run(["gcc", "-std=c11", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                            "-fno-omit-frame-pointer", "-ffp-contract=off", "-DORA_REAL=double",
                            os.path.join(ROOT, "oracle", "laa_oracle.c"), os.path.join(HERE, "oracle_sanitizer_driver.c"),
                            "-o", exe, "-lm"], capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    run = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0 and "oracle sanitizer run: ok" in run.stdout, run.stdout + run.stderr
