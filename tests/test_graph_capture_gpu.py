"""The entry points under HIP graph capture: forward, backward and the packed cross-entropy are recorded
once and replayed several times, with eager launches and synchronisations in between; every replay
must reproduce the eager results bit for bit (the kernels write every output once, without atomics,
and reset their own work-queue counters with kernels, not memsets)."""
import numpy as np
import pytest

import hbp_workloads as wl

pytestmark = pytest.mark.gpu


def test_replays_of_a_captured_step_match_eager_bit_for_bit():
    import torch
    import paper_2503_07680_amd as H
    from paper_2503_07680_amd.runner import PackedAttention

    lengths, Hq, Hkv, d, e = [700, 300, 1500, 60, 1, 415], 4, 2, 128, 128
    pa = PackedAttention(lengths, sum(lengths), Hq, Hkv, d, e)
    pa.alloc_backward()
    T = pa.T
    host = {s: {w: wl.tensor_bits(s, w, T, {"q": Hq, "k": Hkv, "v": Hkv, "do": Hq}[w],
                                  {"q": d, "k": d, "v": e, "do": e}[w], 1.0, None) for w in ("q", "k", "v", "do")}
            for s in (11, 12)}
    dev = {w: pa.to_device_bf16(host[11][w]) for w in ("q", "k", "v", "do")}

    V, n_samples = 4096, pa.n_samples
    r = np.random.default_rng(5)
    logit_sets = {s: torch.from_numpy(wl.f32_to_bf16_bits(r.normal(0, 2, (T, V)).astype(np.float32)).view(np.int16)).cuda()
                  for s in (11, 12)}
    logits = logit_sets[11].clone()
    labels_np = r.integers(0, V, T).astype(np.int32)
    labels_np[r.random(T) < 0.3] = -100
    labels = torch.from_numpy(labels_np).cuda()
    dlogits = torch.zeros((T, V), dtype=torch.int16, device="cuda")
    loss = torch.zeros(1, device="cuda")
    ws = torch.empty(H.hbp_packed_ce_workspace_bytes(T, n_samples), dtype=torch.uint8, device="cuda")

    def load(s):
        for w in dev:
            dev[w].copy_(pa.to_device_bf16(host[s][w]))
        logits.copy_(logit_sets[s])

    def step():
        stream = int(torch.cuda.current_stream().cuda_stream)
        pa.forward(dev["q"], dev["k"], dev["v"])
        pa.backward(dev["q"], dev["k"], dev["v"], dev["do"])
        H.hbp_packed_ce(logits, 0, T, V, labels, pa.cu_dev, n_samples, H.HBP_LOSS_STABLE, 100.0, dlogits, loss, None,
                        ws, stream)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (pa.o, pa.lse, pa.dq, pa.dk, pa.dv, dlogits, loss)]

    def clear():
        for t in (pa.o, pa.lse, pa.dq, pa.dk, pa.dv, dlogits, loss):
            t.zero_()

    eager = {}
    for s in (11, 12):
        load(s)
        clear()
        step()
        eager[s] = snapshot()

    load(11)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()

    for s in (11, 12, 11, 12):
        load(s)            # eager copies between the replays
        clear()            # eager fills
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for a, b in zip(got, eager[s]):
            assert torch.equal(a.contiguous().view(torch.uint8), b.contiguous().view(torch.uint8))
        step()             # an eager step of the same work between replays
        torch.cuda.synchronize()


def test_the_workspace_free_backward_replays_from_a_graph():
    """hbp_varlen_attn_bwd_static is meant for code under graph capture: after one eager call (which looks up
    the static array's address on this device) it is recorded together with the forward and replayed on two
    inputs, with eager work in between; every replay must equal the eager workspace backward bit for bit."""
    import torch
    import paper_2503_07680_amd as H
    from paper_2503_07680_amd.runner import PackedAttention

    lengths, Hq, Hkv, d, e = [900, 130, 1, 333], 8, 2, 128, 128      # 2 kv heads: partial sums + reduce kernel
    pa = PackedAttention(lengths, sum(lengths), Hq, Hkv, d, e)
    pa.alloc_backward()
    T = pa.T
    dims = {"q": (Hq, d), "k": (Hkv, d), "v": (Hkv, e), "do": (Hq, e)}
    host = {s: {w: wl.tensor_bits(s, w, T, dims[w][0], dims[w][1], 1.0, None) for w in dims} for s in (21, 22)}
    dev = {w: pa.to_device_bf16(host[21][w]) for w in dims}
    dq, dk, dv = torch.zeros_like(pa.dq), torch.zeros_like(pa.dk), torch.zeros_like(pa.dv)

    def static_step():
        stream = int(torch.cuda.current_stream().cuda_stream)
        pa.forward(dev["q"], dev["k"], dev["v"])
        H.hbp_varlen_attn_bwd_static(pa.desc, dev["q"], dev["k"], dev["v"], pa.o, pa.lse, dev["do"], pa.cu_dev,
                                     pa.q_tiles_dev, len(pa.q_tiles), pa.kv_tiles_dev, len(pa.kv_tiles), dq, dk, dv,
                                     None, None, stream)

    eager = {}
    for s in (21, 22):
        for w in dev:
            dev[w].copy_(pa.to_device_bf16(host[s][w]))
        pa.forward(dev["q"], dev["k"], dev["v"])
        pa.backward(dev["q"], dev["k"], dev["v"], dev["do"])
        torch.cuda.synchronize()
        eager[s] = [t.clone() for t in (pa.dq, pa.dk, pa.dv)]
    static_step()                      # first call on this device, outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        static_step()
    for s in (21, 22, 21):
        for w in dev:
            dev[w].copy_(pa.to_device_bf16(host[s][w]))
        for t in (dq, dk, dv):
            t.fill_(5.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip((dq, dk, dv), eager[s]):
            assert torch.equal(a, b)
        pa.backward(dev["q"], dev["k"], dev["v"], dev["do"])      # eager work between the replays
        torch.cuda.synchronize()
