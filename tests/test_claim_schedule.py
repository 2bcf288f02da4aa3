"""The claim schedule of the streaming kernels (chunks shifted to the reference stream's line phase) tiles the buffer
exactly: a host-only C++ check compiled with hipcc against the library's own headers.  No GPU needed."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not os.path.exists(HIPCC) and shutil.which("hipcc") is None, reason="hipcc not installed")
def test_claims_tile_the_buffer(tmp_path):
    exe = str(tmp_path / "claim_schedule_check")
    src = os.path.join(ROOT, "tests", "claim_schedule_check.hip")
    inc = os.path.join(ROOT, "paper_2412_01152_amd", "csrc")
    r = subprocess.run([HIPCC if os.path.exists(HIPCC) else "hipcc", "--offload-arch=gfx950", "-O2", "-std=c++17",
                        f"-I{inc}", src, "-o", exe], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0 and r.stdout.startswith("ok:"), r.stdout[-2000:]
    print(r.stdout)
