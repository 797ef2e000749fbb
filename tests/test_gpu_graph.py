"""The entry points under HIP graph capture: they allocate nothing, synchronise nothing and enqueue only kernels on
the caller's stream, so a captured call must replay to the same result -- several times, with eager work and
synchronisations between the replays."""
import numpy as np
import pytest

import sla_inputs as si
from gpu_util import GLA, GDN, RETNET, to_device

pytestmark = pytest.mark.gpu


def _forward_args(variant, d, dtype):
    g, _ = to_device(d, dtype, variant)
    return g


@pytest.mark.parametrize("variant,segments", [(GLA, 1), (RETNET, 3), (GDN, 1)])
def test_forward_replays_identically(variant, segments):
    import torch
    import paper_2602_01744_amd as sla

    B, T, H, dk, dv = 2, 900, 4, 128, 128
    d = si.custom(variant, "bf16", B=B, T=T, H=H, dk=dk, dv=dv, seed=2700 + variant)
    g = _forward_args(variant, d, "bf16")
    s0 = torch.from_numpy(si.initial_state(B, H, dk, dv, seed=27)).cuda()
    args = (variant, g["q"], g["k"], g["v"], g["q_logits"], g["k_logits"], g["log_decay"], g["beta"], s0)
    ref_out, ref_fin = sla.forward(*args, segments=segments)
    torch.cuda.synchronize()

    out = torch.empty_like(ref_out)
    fin = torch.empty_like(ref_fin)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    p = sla.SlaParams(variant, sla.BF16, B, T, H, dk, dv, 0, 0, segments)
    ws = torch.empty(max(sla.sla_workspace_bytes(p, cus), 16), dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):  # one eager call on the capture stream first (one-time kernel set-up)
        sla.forward(*args, out=out, final_state=fin, segments=segments, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        sla.forward(*args, out=out, final_state=fin, segments=segments, workspace=ws)
    for rep in range(4):
        out.zero_(); fin.zero_(); ws.fill_(rep)  # eager work between replays; stale workspace contents
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref_out) and torch.equal(fin, ref_fin), f"replay {rep}"


def test_decode_steps_replay_identically():
    """Eight decode steps captured as one graph; two replays continue the recurrence exactly like eager steps."""
    import torch
    import paper_2602_01744_amd as sla

    B, H, dk, dv, N = 4, 8, 128, 128, 8
    d = si.custom(GLA, "bf16", B=B, T=1, H=H, dk=dk, dv=dv, seed=2800)
    g = _forward_args(GLA, d, "bf16")
    sq = lambda t: t[:, 0].contiguous()
    q, k, v, ql, kl, ld = (sq(g[n]) for n in ("q", "k", "v", "q_logits", "k_logits", "log_decay"))
    s0 = torch.from_numpy(si.initial_state(B, H, dk, dv, seed=28)).cuda()

    eager_state = s0.clone()
    for _ in range(2 * N):
        eager_out = sla.decode_step(GLA, q, k, v, ql, kl, ld, None, eager_state)
    torch.cuda.synchronize()

    state = s0.clone()
    out = torch.empty_like(eager_out)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for _ in range(N):
            sla.decode_step(GLA, q, k, v, ql, kl, ld, None, state, out=out)
    state.copy_(s0)  # capture runs nothing: start from the seeded state
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    _ = state.sum().item()  # eager work and a synchronisation between the replays
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(state, eager_state) and torch.equal(out, eager_out)


@pytest.mark.parametrize("variant", [RETNET, GLA, GDN])
def test_training_step_replays_identically(variant):
    """Gate logits, forward and backward captured as one graph (raw entry points, buffers allocated up front); the
    workspace is dirtied between replays."""
    import torch
    import paper_2602_01744_amd as sla

    B, T, H, dk, dv = 2, 300, 4, 128, 128
    d = si.custom(variant, "bf16", B=B, T=T, H=H, dk=dk, dv=dv, seed=2900 + variant)
    g = _forward_args(variant, d, "bf16")
    gw = si.gate_weights(H, dk, seed=2901)
    wq, wk = torch.from_numpy(gw["w_gq"]).cuda(), torch.from_numpy(gw["w_gk"]).cuda()
    dout = torch.from_numpy(si.cotangents(B, T, H, dk, dv, seed=2902)["d_out"]).to(torch.bfloat16).cuda()
    p = sla.SlaParams(variant, sla.BF16, B, T, H, dk, dv, 0, 0, 1)
    ql = torch.empty((B, T, H), dtype=torch.float32, device="cuda")
    kl = torch.empty_like(ql)
    out = torch.empty_like(g["v"])
    fin = torch.empty((B, H, dk, dv), dtype=torch.float32, device="cuda")
    grads = [torch.empty_like(g["q"]), torch.empty_like(g["k"]), torch.empty_like(g["v"]), torch.empty_like(ql),
             torch.empty_like(kl)]
    dld = torch.empty_like(g["log_decay"]) if variant != RETNET else None
    dbeta = torch.empty_like(g["beta"]) if variant == GDN else None
    need = sla.sla_backward_gdn_workspace_bytes(p) if variant == GDN else sla.sla_backward_workspace_bytes(p)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    ptr = lambda t: None if t is None else t.data_ptr()

    def step(stream):
        assert sla.sla_gate_logits(p, ptr(g["q"]), ptr(g["k"]), ptr(wq), ptr(wk), ptr(ql), ptr(kl), stream) == 0
        assert sla.sla_forward(p, ptr(g["q"]), ptr(g["k"]), ptr(g["v"]), ptr(ql), ptr(kl), ptr(g["log_decay"]),
                               ptr(g["beta"]), None, ptr(out), ptr(fin), stream) == 0
        if variant == GDN:
            assert sla.sla_backward_gdn(p, ptr(g["q"]), ptr(g["k"]), ptr(g["v"]), ptr(ql), ptr(kl),
                                        ptr(g["log_decay"]), ptr(g["beta"]), None, ptr(dout), None,
                                        *(ptr(t) for t in grads), ptr(dld), ptr(dbeta), None, ptr(ws), ws.numel(),
                                        stream) == 0
            return
        assert sla.sla_backward(p, ptr(g["q"]), ptr(g["k"]), ptr(g["v"]), ptr(ql), ptr(kl), ptr(g["log_decay"]), None,
                                ptr(dout), None, *(ptr(t) for t in grads), ptr(dld), None, ptr(ws), ws.numel(),
                                stream) == 0

    step(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    everything = [ql, kl, out, fin] + grads + [t for t in (dld, dbeta) if t is not None]
    ref = [t.clone() for t in everything]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(side.cuda_stream)
    for rep in range(3):
        for t in everything:
            t.zero_()
        ws.fill_(rep + 1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for t, r in zip(everything, ref):
            assert torch.equal(t, r), f"replay {rep}"
