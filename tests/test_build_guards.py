"""Build-time guard: in kernels that use the inline-asm MFMA form no register spill or reload may sit among
the MFMAs (a spill copy next to an asm MFMA would escape the compiler's hazard handling: the compiler does
not see what the asm writes and when).  A value parked in scratch once per work item, in the item's
prologue far ahead of the first MFMA, is harmless and allowed."""
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
        body = text[text.index("\n" + name + ":"):]
        body = body[:body.index(".end_amdhsa_kernel")]
        ins = [l.split()[0] for l in body.splitlines()
               if l.startswith("\t") and l.strip() and not l.strip().startswith((";", "."))]
        mfma = [i for i, op in enumerate(ins) if op.startswith("v_mfma")]
        scratch = [i for i, op in enumerate(ins) if op.startswith("scratch_")]
        assert mfma, name
        # nothing between the first MFMA and 64 instructions behind the last one (MFMA results are long
        # written by then), and no more than a handful of parked values altogether
        assert all(i < mfma[0] or i > mfma[-1] + 64 for i in scratch), (name, scratch, mfma[0], mfma[-1])
        assert spills <= 4, (name, spills)
        # nor copies between two sets of accumulator registers (the key-tile kernel issues every update
        # of dK / dV from one place so that the compiler keeps them in place)
        body = text[text.index("\n" + name + ":"):]
        body = body[:body.index(".end_amdhsa_kernel")]
        assert "v_accvgpr_mov" not in body, name
