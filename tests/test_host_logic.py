"""Host-side logic of the library that needs no GPU: the block-id decoding of the kernels, compiled for the host
from the library's own header."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_block_decode_is_a_bijection_and_keeps_units_on_few_xcds(tmp_path):
    exe = tmp_path / "decode_check"
    hipcc = "/opt/rocm/bin/hipcc" if os.path.exists("/opt/rocm/bin/hipcc") else "hipcc"
    subprocess.run([hipcc, "-O1", "-std=c++17", "--offload-arch=gfx950", "-Wno-unused-command-line-argument",
                    "-I", os.path.join(ROOT, "paper_2206_08888_amd", "csrc"),
                    os.path.join(ROOT, "tests", "host", "decode_check.cpp"), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0 and "bad 0" in out.stdout, out.stdout[-2000:]
    assert "agents 8, 9 on 4 and 4 XCDs; critics 16..19 on 2 2 2 2" in out.stdout
