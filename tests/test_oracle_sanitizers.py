"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): every entry point driven
on small awkward shapes in exactly-sized buffers by tests/oracle_sanitize_driver.cpp."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="no g++")
def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "oracle_sanitize"
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-ffp-contract=off", "-fno-fast-math", "-pthread",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-I", os.path.join(ROOT, "oracle"), os.path.join(ROOT, "oracle", "svdq_oracle.cpp"),
           os.path.join(ROOT, "tests", "oracle_sanitize_driver.cpp"), "-o", str(exe)]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    # the environment is passed on untouched; the sanitizer runtime is only told not to insist on being the first
    # library of the process (another preloaded library may stand before it)
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0"
    p = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=300)
    if p.returncode != 0 and "does not come first in initial library list" in p.stderr:
        pytest.skip("another preloaded library keeps the sanitizer runtime from starting in this environment")
    assert p.returncode == 0, p.stdout + p.stderr
    assert "oracle sanitizer drive: ok" in p.stdout
