"""The host entry points (packing, sharding maps, streaming packer, sharding selection, exact
solver) built with AddressSanitizer and UndefinedBehaviorSanitizer and driven with random and
degenerate inputs by host_sanitizer_harness.cpp.  Host code only: no GPU, no HIP runtime."""
import shutil
import subprocess
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parents[1]


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_entry_points_under_sanitizers(tmp_path):
    exe = tmp_path / "harness"
    build = subprocess.run(
        ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
         f"-I{ROOT / 'include'}", f"-I{ROOT / 'paper_2503_17924_amd' / 'csrc'}",
         str(ROOT / "tests" / "host_sanitizer_harness.cpp"),
         str(ROOT / "paper_2503_17924_amd" / "csrc" / "wlb_host.cpp"), "-o", str(exe)],
        capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-2000:]
    run = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, (run.stdout + run.stderr)[-4000:]
    assert "host entry points: ok" in run.stdout
