"""The C++ auto-selection against the oracle: every integer exact, the times as returned by the profile."""
import math

import numpy as np
import pytest

import paper_2503_07680_amd as H
from oracle import auto_selection as au

K = 1024


def cost_model_profile(seed, hidden=4096, layers=32, mem_cap=80.0):
    """A synthetic profile in the shape of the paper's: iteration time from the per-layer cost model of
    the appendix (24 B s h^2 + 4 B sum s_i^2, with recomputation for checkpointed layers and an
    all-to-all term growing with the SP degree), remaining memory linear in the checkpointed layers.
    Deterministic in (seed, l, sp, ckpt); used for BOTH sides, it holds none of the method's steps."""
    r = np.random.default_rng([31, seed])
    jitter = {}

    def j(l, sp):
        if (l, sp) not in jitter:
            jitter[(l, sp)] = 1.0 + 0.02 * r.standard_normal()
        return jitter[(l, sp)]

    def memory(l, sp, c):
        ktok = l / sp / 1024                        # thousands of tokens per rank
        kept, ckpt = 0.09 * ktok, 0.012 * ktok      # GB per layer: activations kept / checkpoint only
        return mem_cap - 50.0 - kept * (layers - c) - ckpt * c

    def time(l, sp, c):                             # GPU-seconds per million tokens
        compute = (1.0 + l / (6.0 * hidden)) * (1.0 + c / (3.0 * layers))
        comm = 0.0 if sp == 1 else 0.08 * (sp - 1) / sp + 0.004 * sp * (8192.0 / l)
        overhead = 0.6 * 8192.0 / l                 # fixed cost per iteration, spread over its tokens
        return (compute + comm + overhead) * j(l, sp)

    return memory, time


CASES = [
    ([8 * K, 16 * K, 32 * K, 64 * K, 128 * K], [1, 2, 4, 8, 16], 20, 32, 0),
    ([4 * K, 32 * K, 128 * K], [1, 2, 4, 8], 8, 32, 1),
    ([2 * K, 4 * K, 8 * K], [1, 2], 0, 32, 2),
    ([32 * K], [1, 2, 4, 8, 16, 32], 20, 32, 3),
    ([1000, 3001, 100000], [3, 1, 7], 4, 30, 4),
    ([8 * K, 16 * K, 256 * K, 512 * K], [1, 2, 4, 8, 16], 20, 32, 5),
    ([8 * K, 2048 * K], [1, 2], 20, 32, 6),                      # nothing fits at the longest length
    ([4 * K, 8 * K, 16 * K, 2048 * K], [1, 2, 64], 20, 32, 7),
]


@pytest.mark.parametrize("lengths,sps,c_min,c_max,seed", CASES)
def test_matches_oracle(lengths, sps, c_min, c_max, seed):
    mem, tim = cost_model_profile(seed)
    try:
        want = au.auto_selection(lengths, sps, c_min, c_max, mem, tim)
    except ValueError:
        want = None
    mem2, tim2 = cost_model_profile(seed)
    if want is None:
        with pytest.raises(H.HbpError):
            H.hbp_auto_select(lengths, sps, c_min, c_max, mem2, tim2)
        return
    groups, per, j = H.hbp_auto_select(lengths, sps, c_min, c_max, mem2, tim2)
    assert [int(g["l"]) for g in groups] == want["groups"]
    assert [int(g["sp"]) for g in groups] == want["sp"]
    assert [int(g["ckpt"]) for g in groups] == want["ckpt"]
    assert j == want["j"]
    for p, s, t, l in zip(per, want["strategies"], want["times"], lengths):
        assert int(p["l"]) == l
        if s is None:
            assert p["feasible"] == 0
        else:
            assert p["feasible"] == 1 and (int(p["sp"]), int(p["ckpt"])) == s and float(p["time"]) == t


def test_the_cases_cover_both_stage2_branches_and_an_infeasible_length():
    seen = set()
    for lengths, sps, c_min, c_max, seed in CASES:
        mem, tim = cost_model_profile(seed)
        try:
            w = au.auto_selection(lengths, sps, c_min, c_max, mem, tim)
        except ValueError:
            seen.add("longest infeasible")
            continue
        seen.add(len(w["groups"]))
        seen.add("best is not the first" if w["j"] > 0 else "best is the first")
        if any(c > 0 for c in w["ckpt"]):
            seen.add("checkpointing")
    assert {2, 3, 4, "longest infeasible", "best is not the first", "best is the first", "checkpointing"} <= seen, seen


def test_papers_tables_through_the_c_abi():
    best = {8 * K: (2, 8, 2.69), 16 * K: (1, 28, 2.65), 32 * K: (8, 8, 2.83), 64 * K: (4, 28, 3.01),
            128 * K: (8, 28, 3.05)}   # appendix table of the best strategy per packing length
    mem = lambda l, sp, c: 1.5 * (c - best[l][1]) if sp >= best[l][0] else -5.0
    tim = lambda l, sp, c: best[l][2] * (1.0 + 0.1 * abs(math.log2(sp / best[l][0])))
    groups, per, j = H.hbp_auto_select(sorted(best), [1, 2, 4, 8, 16], 20, 32, mem, tim)
    assert [(int(g["l"]), int(g["sp"])) for g in groups] == [(16 * K, 1), (128 * K, 8)] and j == 1
    assert [(int(p["sp"]), int(p["ckpt"])) for p in per] == [best[l][:2] for l in sorted(best)]


def test_argument_errors():
    ok = (lambda l, sp, c: 1.0, lambda l, sp, c: 1.0)
    for lengths, sps, c0, c1 in [([], [1], 1, 2), ([8], [], 1, 2), ([8, 8], [1], 1, 2), ([16, 8], [1], 1, 2),
                                 ([0, 8], [1], 1, 2), ([8], [0], 1, 2), ([8], [1], 2, 2), ([8], [1], -1, 2)]:
        with pytest.raises(H.HbpError):
            H.hbp_auto_select(lengths, sps, c0, c1, *ok)
    with pytest.raises(H.HbpError):   # nothing fits at the longest length
        H.hbp_auto_select([8, 16], [1], 1, 2, lambda l, sp, c: -1.0 if l == 16 else 1.0, ok[1])
