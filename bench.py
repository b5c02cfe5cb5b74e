#!/usr/bin/env python3
"""Benchmark of the packed varlen causal attention hot path (plan -> forward -> backward) on one MI355X.

One "step" = one forward + one backward over one synthetic pack, inputs resident in HBM.
Prints ONE JSON line: useful TFLOP/s (only in-sample causal pairs are counted:
fwd 2(d_qk+d_v), bwd 2(3 d_qk+2 d_v) flop per pair and head), the roofline of the dominant kernel
(the backward key-tile kernel) timed live with HIP events, the per-CU busy-time spread from the
kernels' own profile records, and the fp64 oracle timed on the host as a CPU baseline.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA (published)

TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_table.md")
DOMINANT_KERNEL_SOURCES = ("bwd.hip", "common.hpp")   # what the backward key-tile kernel is compiled from


def kernel_sources_digest() -> str:
    """First 12 hex digits of the SHA-256 over the dominant kernel's source files: the key that ties a
    measured traffic figure to the build it was measured on."""
    import hashlib
    h = hashlib.sha256()
    for name in DOMINANT_KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2503_07680_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:12]


def measured_traffic_bytes(config: int, seed: int):
    """HBM bytes of one launch of the dominant kernel from the rocprofv3 counter runs recorded in
    profiles/hbm_traffic_table.md (FETCH_SIZE and WRITE_SIZE in KiB per dispatch, each with its calibration
    factor), or None when the table has no row for this workload, seed and kernel source digest."""
    digest = kernel_sources_digest()
    try:
        lines = open(TRAFFIC_TABLE).read().splitlines()
    except OSError:
        return None
    for line in lines:
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) != 7 or not cells[0].isdigit():
            continue
        cfg, sd, dig, fetch_kib, fetch_x, write_kib, write_x = cells
        if int(cfg) == config and int(sd) == seed and dig == digest:
            return int((float(fetch_kib) * float(fetch_x) + float(write_kib) * float(write_x)) * 1024)
    return None


class HipEvents:
    """hipEvent_t handles through the HIP runtime (timing on the stream the kernels run on)."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def create(self) -> int:
        ev = ctypes.c_void_p()
        rc = self.hip.hipEventCreate(ctypes.byref(ev))
        if rc != 0:
            raise RuntimeError("hipEventCreate failed: %d" % rc)
        return ev.value

    def record(self, ev: int, stream: int):
        rc = self.hip.hipEventRecord(ev, stream)
        if rc != 0:
            raise RuntimeError("hipEventRecord failed: %d" % rc)

    def sync(self, ev: int):
        self.hip.hipEventSynchronize(ev)

    def elapsed_ms(self, a: int, b: int) -> float:
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
        if rc != 0:
            raise RuntimeError("hipEventElapsedTime failed: %d" % rc)
        return float(ms.value)


class PowerSampler:
    """Board power from the amdgpu hwmon node, polled from a host thread while the timed steps run (the
    kernels sit at the board's power limit, which is what bounds them).  Reports nothing
    when the node cannot be read."""

    def __init__(self, period_s: float = 0.004):
        import glob
        import threading
        self.period = period_s
        self.samples = []
        self.stop = False
        nodes = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input"))
        self.node = nodes[0] if nodes else None
        self.cap_w = None
        if self.node:
            try:
                self.cap_w = int(open(self.node.replace("power1_input", "power1_cap")).read()) / 1e6
            except (OSError, ValueError):
                pass
        self.thread = threading.Thread(target=self._run, daemon=True) if self.node else None

    def _run(self):
        while not self.stop:
            try:
                self.samples.append((time.perf_counter(), int(open(self.node).read()) / 1e6))
            except (OSError, ValueError):
                return
            time.sleep(self.period)

    def start(self):
        if self.thread:
            self.thread.start()

    def finish(self, t0: float, t1: float):
        self.stop = True
        if not self.thread:
            return None
        self.thread.join()
        w = [p for (t, p) in self.samples if t0 <= t <= t1]
        if not w:
            return None
        return {"mean_w": float(np.mean(w)), "max_w": float(np.max(w)), "cap_w": self.cap_w, "samples": len(w),
                "source": "hwmon power1_input during the timed steps"}


def busy_spread(rec: np.ndarray):
    """Per-CU busy time from per-workgroup records -> (max-min)/max, the ABR form, #CUs seen."""
    hw, xcc = rec["hw_id"], rec["xcc_id"] & 0xF
    cu_key = (xcc.astype(np.int64) << 16) | (((hw >> 13) & 7).astype(np.int64) << 8) | \
             (((hw >> 12) & 1).astype(np.int64) << 4) | ((hw >> 8) & 0xF).astype(np.int64)
    used = rec["n_items"] > 0
    keys = np.unique(cu_key[used])
    busy = np.array([rec["busy_ticks"][used & (cu_key == kq)].sum() for kq in keys], dtype=np.float64)
    if len(busy) == 0:
        return None
    span = float(rec["last_tick"][used].max() - rec["first_tick"][used].min())
    return {"cus_seen": int(len(keys)), "spread": float((busy.max() - busy.min()) / busy.max()),
            "abr": float((busy.max() - busy).sum() / (busy.max() * len(busy))),
            "kernel_span_ms": span / 1e5, "max_cu_busy_ms": float(busy.max()) / 1e5,
            "workgroups": int(used.sum())}


def cpu_baseline(w, cu, target_pairs=2.0e8):
    """Time the fp64 oracle (fwd + dQ + dK/dV) on a bounded sub-pack of the same workload."""
    import hbp_workloads as wl
    import oracle
    g = w.n_q_heads // w.n_kv_heads
    lens = np.diff(cu)
    keep = [i for i in range(len(lens)) if lens[i] <= 4096]
    if keep:
        sub_lens = [int(lens[i]) for i in keep]
        starts = [int(cu[i]) for i in keep]
        what = "%d samples of <=4096 tokens taken whole from the pack" % len(keep)
    else:
        sub_lens = [4096 for _ in lens]
        starts = [int(cu[i]) for i in range(len(lens))]
        what = "first 4096 tokens of each sample"
    pairs = sum(s * (s + 1) // 2 for s in sub_lens)
    n_groups = int(max(1, min(w.n_kv_heads, round(target_pairs / max(pairs * g, 1)))))
    q_heads = list(range(n_groups * g))
    kv_heads = list(range(n_groups))
    T = int(cu[-1])
    rows = np.concatenate([np.arange(a, a + s) for a, s in zip(starts, sub_lens)])
    pick = lambda t, hs: wl.bf16_bits_to_f32(wl.workload_tensor_bits(w, t, T, hs)[rows])
    q, do, k, v = pick("q", q_heads), pick("do", q_heads), pick("k", kv_heads), pick("v", kv_heads)
    sub_cu = np.concatenate([[0], np.cumsum(sub_lens)]).astype(np.int32)
    t0 = time.perf_counter()
    oracle.attn_fwd(q, k, v, sub_cu)
    oracle.attn_bwd_dq(q, k, v, do, sub_cu)
    oracle.attn_bwd_dkdv(q, k, v, do, sub_cu)
    dt = time.perf_counter() - t0
    flops = len(q_heads) * pairs * (2 * (w.d_qk + w.d_v) + 2 * (3 * w.d_qk + 2 * w.d_v))
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.oracle_threads(),
            "kind": "oracle", "seconds": dt, "cpu_model": cpu_model(),
            "sample": "%s (%d tokens, %d causal pairs), %d query heads / %d kv heads, fwd+bwd in fp64; a sub-pack "
                      "sized for 10-30 s of oracle time, not the subset the parity tests compare"
                      % (what, int(sum(sub_lens)), pairs, len(q_heads), len(kv_heads))}


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def planner_timing(n=1_000_000):
    """Host side: the multi-level Balance Packing planner over a synthetic dataset of n lengths
    (lognormal(600, 1.2) clipped to [16, 131072], four packing groups); the paper quotes about 5 s per
    million samples for its whole-dataset packing (Appendix, packing time), on other hardware."""
    import paper_2503_07680_amd as H
    r = np.random.default_rng(0)
    lengths = np.clip(np.rint(np.exp(r.normal(np.log(600.0), 1.2, n))), 16, 131072).astype(np.int32)
    groups, per_batch, sp = [4096, 16384, 32768, 131072], [32, 8, 4, 1], [1, 2, 4, 8]
    H.hbp_balance_packing(lengths[:1000], groups, per_batch, sp, 0)
    t0 = time.perf_counter()
    batches, packs, items, m = H.hbp_balance_packing(lengths, groups, per_batch, sp, 0)
    dt = time.perf_counter() - t0
    return {"samples": n, "seconds": dt, "samples_per_s": n / dt, "n_packs": int(len(packs)),
            "n_batches": int(len(batches)), "metrics": m, "packing_groups": groups}


def auto_select_timing():
    """Host side: Hierarchical Groups Auto-Selection over the paper's candidate lengths and SP degrees with
    a table profile in the shape of the appendix tables (the library calls back for every profile point;
    the time is that of the selection logic plus the Python callbacks)."""
    import paper_2503_07680_amd as H
    K = 1024
    best = {8 * K: (2, 8, 2.69), 16 * K: (1, 28, 2.65), 32 * K: (8, 8, 2.83), 64 * K: (4, 28, 3.01),
            128 * K: (8, 28, 3.05)}
    calls = [0]

    def memory(l, sp, c):
        calls[0] += 1
        return 1.5 * (c - best[l][1]) if sp >= best[l][0] else -5.0

    def iter_time(l, sp, c):
        calls[0] += 1
        return best[l][2] * (1.0 + 0.1 * abs(np.log2(sp / best[l][0])))

    t0 = time.perf_counter()
    groups, per, j = H.hbp_auto_select(sorted(best), [1, 2, 4, 8, 16], 20, 32, memory, iter_time)
    dt = time.perf_counter() - t0
    return {"candidate_lengths": sorted(best), "sp_degrees": [1, 2, 4, 8, 16], "profile_calls": calls[0],
            "seconds": dt, "groups": [int(g["l"]) for g in groups], "group_sp": [int(g["sp"]) for g in groups]}


def packed_ce_timing(ev, stream, T=8192, V=128256, n_samples=12, reps=10):
    """The HBM-bound companion kernel: cross-entropy + gradient with the stable normaliser over T tokens
    of a LLaMA-3-sized vocabulary (synthetic logits N(0, 2), 30 % of the tokens without loss).
    Algorithmic bytes: the loss rows are read once, every gradient row is written once."""
    import torch
    import paper_2503_07680_amd as H
    g = torch.Generator(device="cuda").manual_seed(0)
    logits = (2.0 * torch.randn((T, V), generator=g, device="cuda", dtype=torch.float32)).to(torch.bfloat16)
    labels = torch.randint(0, V, (T,), generator=g, device="cuda", dtype=torch.int32)
    labels[torch.rand((T,), generator=g, device="cuda") < 0.3] = -100
    cu = torch.linspace(0, T, n_samples + 1, device="cuda").to(torch.int32)
    dl = torch.empty((T, V), dtype=torch.bfloat16, device="cuda")
    loss = torch.zeros(1, device="cuda")
    ws = torch.empty(H.hbp_packed_ce_workspace_bytes(T, n_samples), dtype=torch.uint8, device="cuda")
    n_valid = int((labels >= 0).sum().item())
    t_ave = n_valid / n_samples
    pairs = [(ev.create(), ev.create()) for _ in range(reps)]
    for i in range(-2, reps):
        if i >= 0:
            H.hbp_set_kernel_events(H.HBP_LOSS, *pairs[i])
        H.hbp_packed_ce(logits, 0, T, V, labels, cu, n_samples, H.HBP_LOSS_STABLE, t_ave, dl, loss, None, ws, stream)
    torch.cuda.synchronize()
    H.hbp_set_kernel_events(H.HBP_LOSS, None, None)
    ms = np.array([ev.elapsed_ms(a, b) for a, b in pairs])
    nbytes = (n_valid + T) * V * 2
    return {"workload": "T=%d tokens x V=%d, %d samples, %d loss tokens, stable normaliser" % (T, V, n_samples, n_valid),
            "kernel_ms_avg": float(ms.mean()), "kernel_ms_min": float(ms.min()), "algorithmic_bytes": nbytes,
            "roofline": {"bound": "hbm", "achieved": nbytes / (ms.mean() * 1e-3) / 1e9, "peak": 8000.0,
                         "unit": "GB/s", "frac": nbytes / (ms.mean() * 1e-3) / 1e9 / 8000.0},
            "loss": float(loss.item())}


def plan_timing(w, pa):
    """Host planning of this pack (both worklists through hbp_pack_plan) and the upload of
    cu_seqlens and the worklists: outside the timed region, reported on their own."""
    import torch
    import paper_2503_07680_amd as H
    reps, per_call = 20, []
    for i in range(reps + 3):
        t0 = time.perf_counter()
        H.hbp_pack_plan(w.lengths, w.pack_len, pa.rows_fwd, H.HBP_TILES_QUERY)
        H.hbp_pack_plan(w.lengths, w.pack_len, pa.rows_bwd, H.HBP_TILES_KEY)
        if i >= 3:
            per_call.append((time.perf_counter() - t0) * 1e3)
    plan_ms = float(np.median(per_call))
    host = [torch.from_numpy(a).pin_memory() for a in (pa.cu, pa.q_tiles, pa.kv_tiles)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        devs = [h.to(pa.device, non_blocking=True) for h in host]
    torch.cuda.synchronize()
    h2d_ms = (time.perf_counter() - t0) * 1e3 / reps
    return {"pack_plan_host_ms": plan_ms, "worklist_h2d_ms": h2d_ms,
            "n_query_tiles": int(len(pa.q_tiles)), "n_key_tiles": int(len(pa.kv_tiles)),
            "bytes_uploaded": int(sum(h.numel() * h.element_size() for h in host))}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3, help="workload 1..5 (default 3: the mixed 32K pack)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--heads", default="",
                    help="Hq/Hkv override, e.g. 32/32: the chosen workload's lengths with another head layout")
    ap.add_argument("--row-pad", type=int, default=0,
                    help="extra elements (multiple of 8) at the end of every token row of Q, K, V, O and the "
                         "gradients (strides in the descriptor); default 0 = dense [T, H, dim]")
    ap.add_argument("--graph", action="store_true",
                    help="also time the same steps replayed from one captured HIP graph (reported as "
                         "graph_replay; `value` stays the eager figure)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one 256 MiB device-to-device copy (known size) to scale rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); --gpus %d is not "
              "supported. Use --gpus 1." % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import hbp_workloads as wl
    import paper_2503_07680_amd as H
    from paper_2503_07680_amd.runner import PackedAttention

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    H.load_library()
    w = wl.workload(args.config, args.seed)
    if args.heads:
        import dataclasses
        hq, hkv = (int(x) for x in args.heads.split("/"))
        w = dataclasses.replace(w, n_q_heads=hq, n_kv_heads=hkv, note=w.note + "; heads overridden to %d/%d" % (hq, hkv))
    pa = PackedAttention(w.lengths, w.pack_len, w.n_q_heads, w.n_kv_heads, w.d_qk, w.d_v, with_profile=True,
                         row_pad=args.row_pad)
    T = pa.T
    dev = {t: pa.to_device_bf16(wl.workload_tensor_bits(w, t, T)) for t in ("q", "k", "v", "do")}
    lens = np.diff(pa.cu).astype(np.int64)
    pairs = int((lens * (lens + 1) // 2).sum())
    fwd_flops = w.n_q_heads * pairs * 2 * (w.d_qk + w.d_v)
    bwd_flops = w.n_q_heads * pairs * 2 * (3 * w.d_qk + 2 * w.d_v)

    ev = HipEvents()
    stream = int(torch.cuda.current_stream().cuda_stream)
    K = args.steps
    f_ev = [(ev.create(), ev.create()) for _ in range(K)]
    b_ev = [(ev.create(), ev.create()) for _ in range(K)]
    q_ev = [(ev.create(), ev.create()) for _ in range(K)]
    e0, e1 = ev.create(), ev.create()

    def step(i=None):
        if i is not None:
            H.hbp_set_kernel_events(H.HBP_FWD, *f_ev[i])
            H.hbp_set_kernel_events(H.HBP_BWD, *b_ev[i])
            H.hbp_set_kernel_events(H.HBP_BWD_DQ, *q_ev[i])
        pa.forward(dev["q"], dev["k"], dev["v"])
        pa.backward(dev["q"], dev["k"], dev["v"], dev["do"])

    power = PowerSampler()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    power.start()
    ev.record(e0, stream)
    t_host = time.perf_counter()
    for i in range(K):
        step(i)
    ev.record(e1, stream)
    torch.cuda.synchronize()
    t_host_end = time.perf_counter()
    host_ms = (t_host_end - t_host) * 1e3
    board_power = power.finish(t_host, t_host_end)
    H.hbp_set_kernel_events(H.HBP_FWD, None, None)
    H.hbp_set_kernel_events(H.HBP_BWD, None, None)
    H.hbp_set_kernel_events(H.HBP_BWD_DQ, None, None)
    total_ms = ev.elapsed_ms(e0, e1)
    ms_per_step = total_ms / K
    fwd_k = np.array([ev.elapsed_ms(a, b) for a, b in f_ev])
    bwd_k = np.array([ev.elapsed_ms(a, b) for a, b in b_ev])
    dq_k = np.array([ev.elapsed_ms(a, b) for a, b in q_ev])

    graph_info = None
    if args.graph:
        # the same step recorded once and replayed K times: what is left of the launch overhead
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step()
        for _ in range(args.warmup):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K):
            g.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / K
        graph_info = {"ms_per_step": graph_ms,
                      "useful_tflops": (fwd_flops + bwd_flops) / (graph_ms * 1e-3) / 1e12}

    # one extra, untimed, profiled step: per-CU busy time
    pa.forward(dev["q"], dev["k"], dev["v"], profile=True)
    pa.backward(dev["q"], dev["k"], dev["v"], dev["do"], profile=True)
    torch.cuda.synchronize()
    spread_f = busy_spread(pa.profile_records(H.HBP_FWD))
    spread_b = busy_spread(pa.profile_records(H.HBP_BWD))
    spread_q = busy_spread(pa.profile_records(H.HBP_BWD_DQ))

    # second roofline denominator: what the matrix pipes of this part sustain on MFMA-only code
    # (every SIMD busy, ~4 ms, same process right after the timed steps, so under the same power state)
    sink = torch.empty(256 * 512, dtype=torch.float32, device="cuda")
    p0, p1 = ev.create(), ev.create()
    n_probe = 120000
    H.hbp_mfma_probe(256, 20000, sink, stream)   # warm
    ev.record(p0, stream)
    H.hbp_mfma_probe(256, n_probe, sink, stream)
    ev.record(p1, stream)
    torch.cuda.synchronize()
    sustained_tf = 256 * 8 * n_probe * 32768 / (ev.elapsed_ms(p0, p1) * 1e-3) / 1e12

    if args.calib_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()

    value = (fwd_flops + bwd_flops) / (ms_per_step * 1e-3) / 1e12
    # flops of the launches themselves: the dK/dV kernel does 4 of the backward's products
    # (S, dP, dV, dK), the dQ kernel 3 (S and dP again, dQ); only 5 of those 7 count as useful
    per_pair = lambda n_qk, n_v: w.n_q_heads * pairs * 2 * (n_qk * w.d_qk + n_v * w.d_v)
    dkdv_flops, dq_flops = per_pair(2, 2), per_pair(2, 1)
    bwd_tf = dkdv_flops / (bwd_k.mean() * 1e-3) / 1e12
    dq_tf = dq_flops / (dq_k.mean() * 1e-3) / 1e12
    fwd_tf = fwd_flops / (fwd_k.mean() * 1e-3) / 1e12
    out = {
        "metric": "useful TFLOP/s fwd+bwd packed varlen attention (1 GPU) + % of bf16 MFMA peak",
        "value": value, "unit": "TFLOP/s", "pct_of_bf16_mfma_peak": 100.0 * value / PEAK_BF16_TFLOPS,
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "config %d: %s (%s)" % (args.config, w.name, w.note), "seed": args.seed,
                   "total_tokens": T, "n_samples": pa.n_samples, "n_q_heads": w.n_q_heads,
                   "n_kv_heads": w.n_kv_heads, "d_qk": w.d_qk, "d_v": w.d_v, "causal_pairs": pairs,
                   "pack_cost_sum_s2": pa.pack_cost, "row_pad": args.row_pad, "useful_tflop_fwd": fwd_flops / 1e12,
                   "useful_tflop_bwd": bwd_flops / 1e12},
        "useful_tflops_4gemm_bwd": (fwd_flops + dkdv_flops) / (ms_per_step * 1e-3) / 1e12,
        "kernels": {"fwd_ms_avg": float(fwd_k.mean()), "fwd_ms_min": float(fwd_k.min()),
                    "fwd_ms_median": float(np.median(fwd_k)), "bwd_dkdv_ms_median": float(np.median(bwd_k)),
                    "bwd_dq_ms_median": float(np.median(dq_k)),
                    "fwd_tflops": fwd_tf, "bwd_dkdv_ms_avg": float(bwd_k.mean()),
                    "bwd_dkdv_ms_min": float(bwd_k.min()), "bwd_dkdv_tflops": bwd_tf,
                    "bwd_dq_ms_avg": float(dq_k.mean()), "bwd_dq_ms_min": float(dq_k.min()),
                    "bwd_dq_tflops": dq_tf,
                    "host_ms_per_step": host_ms / K},
        "roofline": {"kernel": "bwd_dkdv_kernel (key-tile persistent kernel; S, dP, dV, dK products)",
                     "bound": "mfma", "flop_per_launch": dkdv_flops,
                     "achieved": bwd_tf, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": bwd_tf / PEAK_BF16_TFLOPS,
                     "sustained_mfma_only_tflops": sustained_tf, "frac_of_sustained": bwd_tf / sustained_tf,
                     "traffic": None if (args.heads or args.row_pad) else measured_traffic_bytes(args.config, args.seed),
                     "traffic_key": {"config": args.config, "seed": args.seed, "kernel_sources_sha256_12": kernel_sources_digest(),
                                     "table": "profiles/hbm_traffic_table.md"}},
        "busy_time_spread": {"fwd": spread_f, "bwd_dkdv": spread_b, "bwd_dq": spread_q},
        "board_power": board_power,
    }
    if graph_info:
        out["graph_replay"] = graph_info
    out["plan"] = plan_timing(w, pa)
    out["balance_packing"] = planner_timing()
    out["auto_selection"] = auto_select_timing()
    del dev
    out["packed_ce"] = packed_ce_timing(ev, stream)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, pa.cu)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
