"""Build-time guard: in kernels that use the inline-asm MFMA form no register spill or reload may sit among
the MFMAs (a spill copy next to an asm MFMA would escape the compiler's hazard handling: the compiler does
not see what the asm writes and when).  A value parked in scratch once per work item, in the item's
prologue far ahead of the first MFMA, is harmless and allowed.  Nor may any vector instruction touch the result
registers of an asm MFMA before the result exists: the compiler inserts such a read when it joins the score
registers of two code paths by copies (it has happened: wrong dK on every pack of short samples), and no
run-time check tells it from rounding noise on long ones."""
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


_ASM_CACHE = {}


def backward_asm():
    if "text" not in _ASM_CACHE:
        with tempfile.TemporaryDirectory() as tmp:
            out = os.path.join(tmp, "bwd.s")
            cmd = [B._hipcc()] + B.HIP_FLAGS + ["-S", "--cuda-device-only", os.path.join(B.CSRC, "bwd.hip"), "-o", out]
            subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
            _ASM_CACHE["text"] = open(out).read()
    return _ASM_CACHE["text"]


def kernel_instructions(text, name):
    body = text[text.index("\n" + name + ":"):]
    body = body[:body.index(".end_amdhsa_kernel")]
    return [l.strip() for l in body.splitlines()
            if l.startswith("\t") and l.strip() and not l.strip().startswith((";", "."))]


def early_reads_of_asm_mfma_results(ins, need=18):
    """Instructions that name a register of an asm MFMA's destination tuple (the asm form writes vector
    registers, v[a:b]; the builtin form writes accumulation registers here) fewer than `need` wait states
    behind that MFMA.  Another MFMA ends the window (a chain on the same accumulator is interlocked by the
    hardware); scalar instructions and s_nop count as wait states, every other instruction as one."""
    found = []
    for k, l in enumerate(ins):
        m = re.match(r"v_mfma_f32_32x32x16_bf16 v\[(\d+):(\d+)\]", l)
        if not m:
            continue
        lo, hi = int(m.group(1)), int(m.group(2))
        waited = 0
        for l2 in ins[k + 1:k + 1 + need]:
            if l2.startswith("v_mfma"):
                break
            if l2.startswith("s_nop"):
                waited += int(l2.split()[1]) + 1
                continue
            if not l2.startswith("s_"):
                regs = [int(x) for x in re.findall(r"\bv(\d+)\b", l2)]
                regs += [r for a, b in re.findall(r"v\[(\d+):(\d+)\]", l2) for r in range(int(a), int(b) + 1)]
                if any(lo <= r <= hi for r in regs) and waited < need:
                    found.append((l, l2, waited))
                    break
            waited += 1
            if waited >= need:
                break
    return found


def test_the_hazard_scan_sees_a_planted_early_copy():
    good = ["v_mfma_f32_32x32x16_bf16 v[8:23], v[0:3], v[4:7], v[8:23]", "s_nop 15", "s_nop 3", "v_mov_b32_e32 v40, v9"]
    assert early_reads_of_asm_mfma_results(good) == []
    chain = ["v_mfma_f32_32x32x16_bf16 v[8:23], v[0:3], v[4:7], v[8:23]",
             "v_mfma_f32_32x32x16_bf16 v[8:23], v[0:3], v[4:7], v[8:23]"]
    assert early_reads_of_asm_mfma_results(chain) == []
    bad = ["v_mfma_f32_32x32x16_bf16 v[8:23], v[0:3], v[4:7], v[8:23]", "s_nop 1", "v_mov_b64_e32 v[86:87], v[22:23]"]
    assert len(early_reads_of_asm_mfma_results(bad)) == 1
    builtin = ["v_mfma_f32_32x32x16_bf16 a[0:15], v[0:3], v[4:7], a[0:15]", "v_accvgpr_read_b32 v1, a0"]
    assert early_reads_of_asm_mfma_results(builtin) == []      # the compiler's own MFMAs: its business


def test_nothing_touches_an_asm_mfma_result_before_it_exists():
    text = backward_asm()
    names = [k for k in kernel_metadata(text) if "bwd_dkdv_kernel" in k or "bwd_dq_kernel" in k]
    assert len(names) == 6, names
    for name in names:
        ins = kernel_instructions(text, name)
        assert any(re.match(r"v_mfma_f32_32x32x16_bf16 v\[", l) for l in ins), name   # the asm form is in use
        assert early_reads_of_asm_mfma_results(ins) == [], name


def test_asm_mfma_kernels_have_no_vgpr_spills():
    text = backward_asm()
    meta = kernel_metadata(text)
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
