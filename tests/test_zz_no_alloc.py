"""hbp_varlen_attn_bwd_static (the backward that takes no workspace: its scratch is a static device array
inside the library) against hbp_varlen_attn_bwd on the same inputs, through the C ABI: two calls in a row,
the second on a smaller problem, so that what the first left in the array would show if it were read."""
import ctypes

import numpy as np
import pytest

import paper_2503_07680_amd as H
from parity_util import Case, run_gpu, compare


def static_backward(pa, dev):
    """dQ, dK, dV of the static entry point into fresh buffers pre-filled with a sentinel."""
    import torch
    dq, dk, dv = (torch.full_like(t, 7.0) for t in (pa.dq, pa.dk, pa.dv))
    H.hbp_varlen_attn_bwd_static(pa.desc, dev["q"], dev["k"], dev["v"], pa.o, pa.lse, dev["do"], pa.cu_dev,
                                 pa.q_tiles_dev, len(pa.q_tiles), pa.kv_tiles_dev, len(pa.kv_tiles), dq, dk, dv,
                                 None, None, int(torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    return dq, dk, dv


@pytest.mark.gpu
def test_static_scratch_backward_equals_the_workspace_backward_on_two_calls_in_a_row():
    import torch
    # first call: 2 kv heads, so the key-tile kernel writes partial sums (the largest scratch layout);
    # second call: a smaller pack with another head size and no partial sums
    big = Case([700, 130, 1, 333, 257], 1421, 8, 2, 128, 128, seed=71, name="static-first")
    small = Case([200, 60, 31], 291, 8, 8, 64, 64, seed=72, name="static-second")
    for case in (big, small):
        pa, dev, out = run_gpu(case)                       # forward + workspace backward
        assert H.hbp_workspace_bytes(pa.desc, H.HBP_BWD) <= H.HBP_STATIC_SCRATCH_BYTES
        dq, dk, dv = static_backward(pa, dev)
        assert torch.equal(dq, pa.dq) and torch.equal(dk, pa.dk) and torch.equal(dv, pa.dv)
        got = dict(out, dq=dq.float().cpu().numpy(), dk=dk.float().cpu().numpy(), dv=dv.float().cpu().numpy())
        compare(case, pa, got, label="static scratch")     # and the oracle's bars
    # once more on the first problem: the array now holds the smaller call's leftovers
    pa, dev, out = run_gpu(big)
    dq, dk, dv = static_backward(pa, dev)
    assert torch.equal(dq, pa.dq) and torch.equal(dk, pa.dk) and torch.equal(dv, pa.dv)


def test_static_scratch_backward_rejects_what_does_not_fit_before_touching_the_device():
    lib = H.load_library()
    fake = 0x1000   # never dereferenced
    d = H.AttnDesc(total_tokens=131072, n_samples=2, n_q_heads=128, n_kv_heads=8, d_qk=128, d_v=128)
    assert H.hbp_workspace_bytes(d, H.HBP_BWD) > H.HBP_STATIC_SCRATCH_BYTES
    st = lib.hbp_varlen_attn_bwd_static(ctypes.byref(d), fake, fake, fake, fake, fake, fake, fake, fake, 1, fake, 1,
                                        fake, fake, fake, None, None, None)
    assert st == H.HBP_ERR_STATIC_LIMIT and "static" in H.hbp_status_string(st)
    # the largest benchmark pack (64 heads x 131072 tokens, 8 kv heads) fits exactly
    d4 = H.AttnDesc(total_tokens=131072, n_samples=2, n_q_heads=64, n_kv_heads=8, d_qk=128, d_v=128)
    assert H.hbp_workspace_bytes(d4, H.HBP_BWD) <= H.HBP_STATIC_SCRATCH_BYTES
    # argument checks come first, as in the workspace form
    assert lib.hbp_varlen_attn_bwd_static(None, fake, fake, fake, fake, fake, fake, fake, fake, 1, fake, 1,
                                          fake, fake, fake, None, None, None) == 1
    d0 = H.AttnDesc(total_tokens=0, n_samples=0, n_q_heads=4, n_kv_heads=2, d_qk=64, d_v=64)
    assert lib.hbp_varlen_attn_bwd_static(ctypes.byref(d0), None, None, None, None, None, None, None, None, 0,
                                          None, 0, None, None, None, None, None, None) == 0
