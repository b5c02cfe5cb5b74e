"""Build-time guard: kernels that use the inline-asm MFMA form must compile without register spills
(a spill copy next to an asm MFMA would escape the compiler's hazard handling)."""
import os
import re
import subprocess
import tempfile

from paper_2503_07680_amd import build as B


def kernel_metadata(asm_text):
    out = {}
    for m in re.finditer(r"\.name:\s+(\S+)\n(?:.*\n)*?\s+\.vgpr_spill_count:\s+(\d+)", asm_text):
        out[m.group(1)] = int(m.group(2))
    return out


def test_asm_mfma_kernels_have_no_vgpr_spills():
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "bwd.s")
        cmd = [B._hipcc()] + B.HIP_FLAGS + ["-S", "--cuda-device-only", os.path.join(B.CSRC, "bwd.hip"), "-o", out]
        subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
        meta = kernel_metadata(open(out).read())
        text = open(out).read()
    dkdv = {k: v for k, v in meta.items() if "bwd_dkdv_kernel" in k or "bwd_dq_kernel" in k}
    assert len(dkdv) == 6, meta
    for name, spills in dkdv.items():
        assert spills == 0, (name, spills)
        # nor copies between two sets of accumulator registers (the key-tile kernel issues every update
        # of dK / dV from one place so that the compiler keeps them in place)
        body = text[text.index("\n" + name + ":"):]
        body = body[:body.index(".end_amdhsa_kernel")]
        assert "v_accvgpr_mov" not in body, name
