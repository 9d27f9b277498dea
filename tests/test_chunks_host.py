"""Host checks of the LDS geometry of the matrix-core kernels (compiled with the host compiler, no GPU)."""
import os
import subprocess
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _build_and_run(name):
    src = os.path.join(ROOT, "tests", "host_checks", name + ".cpp")
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, name)
        subprocess.run(["g++", "-O1", "-std=c++17", "-I", os.path.join(ROOT, "include"),
                        "-I", os.path.join(ROOT, "paper_2409_09083_amd", "csrc"), src, "-o", exe], check=True)
        out = subprocess.run([exe], capture_output=True, text=True)
        assert out.returncode == 0, out.stdout
        assert out.stdout.startswith("ok")


def test_wgrad_chunks_fit_their_lds_limits():
    _build_and_run("chunk_check")


def test_conv_tiles_fit_their_lds_limits_and_cover_every_pixel_once():
    _build_and_run("conv_tile_check")
