"""fp64 CPU oracle for packed varlen causal attention and the pack planner.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()`` and by the
``cpu_baseline`` leg of ``bench.py``.  The product package never imports it, and it never
imports the product package.
"""
from .attention import (attn_fwd, attn_bwd_dq, attn_bwd_dkdv, prob_row, build_oracle,
                        oracle_threads)
from .plan import pack_plan, pack_cost, balance_ratio
from . import balance_packing
from . import loss
from . import auto_selection

__all__ = ["attn_fwd", "attn_bwd_dq", "attn_bwd_dkdv", "prob_row", "build_oracle",
           "oracle_threads", "pack_plan", "pack_cost", "balance_ratio", "balance_packing", "loss",
           "auto_selection"]
