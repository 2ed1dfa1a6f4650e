"""The ring GEMM kernels must not spill: their next-weights touch parks a value in a register that
the compiler believes is already written, and a spill of it (or of anything else in the K loop) would
go unnoticed at run time.  Compiles the kernel file to gfx950 assembly (no GPU needed) and reads the
resource usage the compiler reports per kernel."""
import os
import re
import subprocess
import tempfile

from paper_2006_09503_amd import build as B


def test_ring_gemm_kernels_use_no_scratch_and_fit_two_waves_per_simd():
    src = os.path.join(B.CSRC, "gemm_bf16.hip")
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "gemm_bf16.s")
        flags = [f for f in B.FLAGS if f != "-fPIC"]
        subprocess.run([B.HIPCC, *flags, "--cuda-device-only", "-S", src, "-o", out], check=True,
                       stderr=subprocess.DEVNULL)
        text = open(out).read()
    kernels = re.findall(r"\.name:\s+(\S+)\n(.*?)\.wavefront_size", text, flags=re.S)
    ring = [(n, body) for n, body in kernels if "gemm_bf16_ring_kernel" in n]
    assert len(ring) >= 10
    for name, body in ring:
        field = lambda k: int(re.search(r"\." + k + r":\s+(\d+)", body).group(1))
        assert field("private_segment_fixed_size") == 0, name       # no scratch: nothing spilled
        assert field("vgpr_spill_count") == 0 and field("sgpr_spill_count") == 0, name
        assert field("vgpr_count") <= 256, name                     # 8 waves per workgroup = 2 per SIMD
