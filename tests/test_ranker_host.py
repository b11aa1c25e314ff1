"""The key-based register rankers, compiled for the host, against plain selections (tests/native/ranker_host_check.hip)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="needs hipcc to compile the host check")
def test_key_based_rankers_match_plain_selection(tmp_path):
    exe = str(tmp_path / "ranker_host_check")
    src = os.path.join(ROOT, "tests", "native", "ranker_host_check.hip")
    cmd = [HIPCC, "-O1", "-std=c++17", "--offload-arch=gfx950", "-I" + os.path.join(ROOT, "include"),
           "-I" + os.path.join(ROOT, "paper_2202_00774_amd", "csrc"), "-o", exe, src]
    subprocess.run(cmd, check=True, capture_output=True, timeout=300)
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, run.stdout[-2000:]
    assert "total mismatches 0" in run.stdout
