"""Host-side check of the grouped GEMM's work distribution: tests/tile_schedule_check.hip includes the index
arithmetic the kernels use (csrc/ffn_tiles.h, compiled for the host) and walks every workgroup id of thousands of
random launches: every (bucket, row tile, column tile, k tile) owned exactly once, partial-tile slots unique,
the fix-up consistent with the split, the host's grid large enough.  No GPU is needed or touched."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_k_tile_of_every_tile_has_exactly_one_owner(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    exe = str(tmp_path / "tile_schedule_check")
    build = subprocess.run([hipcc, "--offload-arch=gfx950", "-O2", "-std=c++17", "-I" + os.path.join(ROOT, "include"),
                            "-I" + os.path.join(ROOT, "paper_2502_06643_amd", "csrc"),
                            os.path.join(ROOT, "tests", "tile_schedule_check.hip"), "-o", exe],
                           capture_output=True, text=True, timeout=300)
    assert build.returncode == 0, build.stderr[-2000:]
    run = subprocess.run([exe, "4000"], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0 and run.stdout.startswith("ok:"), run.stdout[-2000:] + run.stderr[-2000:]
