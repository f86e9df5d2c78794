"""Builds and runs the CPU emulation of the GEMM workgroup program (operand
loaders, LDS staging, MFMA index maps, epilogues, split-k) under
AddressSanitizer, against direct convolution loops.  No GPU involved."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_gemm_workgroup_program_on_cpu(tmp_path):
    exe = str(tmp_path / "gemm_emu")
    src = os.path.join(HERE, "emu", "gemm_emu.cpp")
    subprocess.run(["g++", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-o", exe, src], check=True, timeout=900)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert "ALL OK" in r.stdout and "FAIL" not in r.stdout


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_tile_transforms_of_the_3x3_layers_on_cpu(tmp_path):
    """The per-thread programs of the F(4x4, 3x3) transforms (input, taps, output, output gradient, tap
    gradient), run for every thread with exactly-sized buffers under AddressSanitizer: forward,
    backward-data and backward-weight against direct convolution loops in double precision."""
    exe = str(tmp_path / "winograd_emu")
    src = os.path.join(HERE, "emu", "winograd_emu.cpp")
    subprocess.run(["g++", "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-o", exe, src], check=True, timeout=600)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert "ALL OK" in r.stdout and "FAIL" not in r.stdout
