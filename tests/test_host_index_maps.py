"""Host logic of the four-step path: the index maps shared by kernels and host code, compiled for the host only."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not os.path.exists(HIPCC) and shutil.which("hipcc") is None, reason="hipcc not found")
def test_entry_order_and_spectrum_pairing(tmp_path):
    """`big_position` and `spectrum_pair` (csrc/mix_pow2.h), the functions the column kernel's forward-only and
    inverse-only modes and the pair <-> half-spectra kernels index the scratch with: for every plan the lines those
    kernels walk cover every bin up to N/2 and every scratch entry exactly once, in bounds."""
    exe = tmp_path / "index_maps"
    csrc = os.path.join(ROOT, "paper_2502_18394_amd", "csrc")
    cmd = [HIPCC if os.path.exists(HIPCC) else "hipcc", "--cuda-host-only", "-x", "hip", "-std=c++17", "-O1", "-I", csrc,
           os.path.join(ROOT, "tests", "host", "index_maps.cpp"), "-o", str(exe)]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-3000:]
    run = subprocess.run([str(exe)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    print(run.stdout)
    assert run.returncode == 0, run.stdout
    assert " 0 failures" in run.stdout
