"""Builds the host-only part of the library with AddressSanitizer + UBSan (plain g++, no GPU code) and runs a
driver that writes the per-call metadata into buffers of exactly the computed size."""

import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_logic_under_sanitizers(tmp_path):
    exe = str(tmp_path / "host_asan")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(ROOT, "paper_2504_02921_amd", "csrc"),
           os.path.join(ROOT, "tests", "host_asan_driver.cpp"),
           os.path.join(ROOT, "paper_2504_02921_amd", "csrc", "hr_host.cpp"), "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    env = dict(os.environ)
    env.pop("LD_PRELOAD", None)          # the sanitizer runtime must come first in the link order
    r = subprocess.run([exe], capture_output=True, text=True, env=env)
    assert r.returncode == 0, (r.stdout + r.stderr)[-2000:]
    assert "clean under sanitizers" in r.stdout
