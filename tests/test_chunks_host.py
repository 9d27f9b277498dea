"""Host check of the LDS chunk geometry of the filter-gradient kernels (compiled with the host compiler, no GPU)."""
import os
import subprocess
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_wgrad_chunks_fit_their_lds_limits():
    src = os.path.join(ROOT, "tests", "host_checks", "chunk_check.cpp")
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "chunk_check")
        subprocess.run(["g++", "-O1", "-std=c++17", "-I", os.path.join(ROOT, "include"),
                        "-I", os.path.join(ROOT, "paper_2409_09083_amd", "csrc"), src, "-o", exe], check=True)
        out = subprocess.run([exe], capture_output=True, text=True)
        assert out.returncode == 0, out.stdout
        assert out.stdout.startswith("ok")
