"""The index maps of the GEMM launches, checked on the CPU: the header that holds them has no HIP dependency, so
the same code the kernels compile is built here with g++ and run over a sweep of shapes (tests/tile_walk_main.cpp:
workgroup -> tile: every tile exactly once, grid size, the XCDs in step over the columns; the block-by-block operand
layout: a bijection with contiguous 8-column pieces and contiguous 256 x 64 blocks)."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_tile_walk_and_blocked_layout(tmp_path):
    exe = str(tmp_path / "tile_walk")
    subprocess.run(["g++", "-O1", "-std=c++17", "-Wall", "-Werror", "-I", os.path.join(ROOT, "paper_2410_17765_amd", "csrc"),
                    os.path.join(ROOT, "tests", "tile_walk_main.cpp"), "-o", exe], check=True)
    out = subprocess.run([exe], check=False, capture_output=True, text=True)
    assert out.returncode == 0, out.stdout
    assert out.stdout.startswith("ok ")
