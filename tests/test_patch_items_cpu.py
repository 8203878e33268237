"""Host logic of the LDS-patch convolution kernels: the work-item decoding (a header the kernels
include) walked on the CPU for every grid size, including grids of fewer than 8 workgroups that
no CU mask of this GPU can produce."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_tile_is_visited_exactly_once_for_every_grid(tmp_path):
    exe = str(tmp_path / "patch_items_check")
    subprocess.run(["g++", "-O1", "-std=c++17", "-Wall", "-I", os.path.join(ROOT, "paper_2406_09425_amd", "csrc"),
                    os.path.join(ROOT, "tests", "cpp", "patch_items_check.cpp"), "-o", exe], check=True)
    r = subprocess.run([exe], capture_output=True, text=True)
    assert r.returncode == 0 and r.stdout.startswith("ok "), r.stdout + r.stderr
    assert int(r.stdout.split()[1]) > 10000
