"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU): a small C
driver (oracle/sanitize_check.c) is built together with oracle/path_oracle.c under
-fsanitize=address,undefined and calls every entry point on exact-size buffers; any report fails the run."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "sanitize_check")
    # (the sanitizer runtimes are linked statically, so that nothing depends on the order of preloaded libraries)
    cmd = ["gcc", "-O1", "-g", "-fopenmp", "-std=c11", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan",
           "-fno-omit-frame-pointer", os.path.join(ROOT, "oracle", "sanitize_check.c"), os.path.join(ROOT, "oracle", "path_oracle.c"),
           "-o", exe, "-lm"]
    subprocess.run(cmd, check=True)
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0"
    env["OMP_NUM_THREADS"] = "4"
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "oracle sanitizer run: ok" in r.stdout
