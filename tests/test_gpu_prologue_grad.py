"""GPU parity of the prologue's backward and of the feature map's L2 option against oracle/sla_prologue.py."""
import numpy as np
import pytest

import sla_inputs as si
from gpu_util import GLA, rel_err
from oracle import sla_prologue as op

pytestmark = pytest.mark.gpu

# fp32 tensors: fp32 accumulation against fp64, hardware exp2 / rsq (1 ulp); bf16 tensors: one rounding of the output
TOL = {"f32": 1e-5, "bf16": 6e-3}


def _dev(a, dtype):
    import torch

    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def _host(t):
    import torch

    return t.to(torch.float32).cpu().numpy().astype(np.float64)


def _round(a, dtype):
    return si.round_to_bf16(a.astype(np.float32)) if dtype == "bf16" else a.astype(np.float32)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("head_width,C", [(0, 72), (32, 128), (64, 256), (128, 384)])
@pytest.mark.parametrize("K", [1, 4])
def test_feature_map_l2_forward_and_backward(dtype, head_width, C, K):
    import paper_2602_01744_amd as sla

    rng = np.random.default_rng(3000 + C + K)
    B, T = 2, 150  # three segments of 64 tokens, the last ragged
    x = _round(rng.normal(size=(B, T, C)), dtype)
    w = rng.normal(size=(C, K)).astype(np.float32) * 0.5
    dy = _round(rng.normal(size=(B, T, C)), dtype)
    eps = 1e-6
    xd, wd, dyd = _dev(x, dtype), _dev(w, "f32"), _dev(dy, dtype)
    y = sla.short_conv_silu_l2(xd, wd, head_width, eps)
    dx, dw = sla.short_conv_silu_l2_backward(xd, wd, dyd, head_width, eps)
    ry = op.short_conv_silu_l2(x, w, head_width, eps)
    rdx, rdw = op.short_conv_silu_l2_backward(x, w, dy, head_width, eps)
    ey, ex, ew = rel_err(_host(y), ry), rel_err(_host(dx), rdx), rel_err(_host(dw), rdw)
    print(f"[feature map] {dtype} C={C} head={head_width} K={K}: y {ey:.2e} dx {ex:.2e} dw {ew:.2e}", flush=True)
    assert ey <= TOL[dtype] and ex <= TOL[dtype] and ew <= 1e-5, (ey, ex, ew)
    if head_width == 0:  # the plain entry point is the same function
        y0 = sla.short_conv_silu(xd, wd)
        assert rel_err(_host(y0), ry) <= TOL[dtype]
    # the two-stage sum over tokens is bitwise reproducible
    dx2, dw2 = sla.short_conv_silu_l2_backward(xd, wd, dyd, head_width, eps)
    assert bool((dw2 == dw).all()) and bool((dx2 == dx).all())


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("H,dk", [(1, 64), (5, 128), (16, 32), (16, 128), (64, 64)])
def test_gate_logits_backward(dtype, H, dk):
    import paper_2602_01744_amd as sla

    rng = np.random.default_rng(3100 + H + dk)
    B, T = 2, 333
    x = _round(rng.normal(size=(B, T, H, dk)), dtype)
    w = si.gate_weights(H, dk, seed=3101)["w_gq"]
    dl = rng.normal(size=(B, T, H)).astype(np.float32)
    dx0 = _round(rng.normal(size=(B, T, H, dk)), dtype)  # what the mixer's backward left in dq
    dxd = _dev(dx0, dtype)
    dw = sla.gate_logits_backward(_dev(x, dtype), _dev(w, "f32"), _dev(dl, "f32"), dxd)
    rdx, rdw = op.gate_logits_backward(x, w, dl)
    ex, ew = rel_err(_host(dxd), dx0.astype(np.float64) + rdx), rel_err(_host(dw), rdw)
    print(f"[gate logits bwd] {dtype} H={H} dk={dk}: dx {ex:.2e} dw {ew:.2e}", flush=True)
    assert ex <= TOL[dtype] and ew <= 1e-5, (ex, ew)


def test_prologue_and_mixer_gradients_chain():
    """Gate logits -> forward -> backward -> gate projections' backward on one small GLA problem: the logit
    cotangents that sla_backward returns, pushed through the projections, against the two oracles chained."""
    import torch

    import paper_2602_01744_amd as sla
    from gpu_util import to_device
    from oracle import sla_backward as ob
    from oracle import sla_numpy as on

    B, T, H, dk, dv = 1, 100, 4, 128, 128
    d = si.custom(GLA, "bf16", B=B, T=T, H=H, dk=dk, dv=dv, seed=3200)
    gw = si.gate_weights(H, dk, seed=3201)
    cot = si.cotangents(B, T, H, dk, dv, seed=3202)
    g, _ = to_device(d, "bf16", GLA)
    wq, wk = torch.from_numpy(gw["w_gq"]).cuda(), torch.from_numpy(gw["w_gk"]).cuda()
    ql, kl = sla.gate_logits(g["q"], g["k"], wq, wk)
    dout = torch.from_numpy(cot["d_out"]).to(torch.bfloat16).cuda()
    gr = sla.backward(GLA, g["q"], g["k"], g["v"], ql, kl, g["log_decay"], dout)
    dwq = sla.gate_logits_backward(g["q"], wq, gr["dq_head_logits"], gr["dq"])
    dwk = sla.gate_logits_backward(g["k"], wk, gr["dk_head_logits"], gr["dk"])
    torch.cuda.synchronize()
    # oracle chain on the same (bf16-representable) inputs, logits in fp64 rounded to the fp32 the GPU passes on
    rql = on.gate_logits(d["q"], gw["w_gq"]).astype(np.float32)
    rkl = on.gate_logits(d["k"], gw["w_gk"]).astype(np.float32)
    ref = ob.backward(GLA, d["q"], d["k"], d["v"], rql, rkl, d["log_decay"], cot["d_out"])
    pq, rwq = op.gate_logits_backward(d["q"], gw["w_gq"], ref["dq_logits"])
    pk, rwk = op.gate_logits_backward(d["k"], gw["w_gk"], ref["dk_logits"])
    assert rel_err(_host(gr["dq"]), ref["dq"] + pq) <= 2e-2
    assert rel_err(_host(gr["dk"]), ref["dk"] + pk) <= 2e-2
    assert rel_err(_host(dwq), rwq) <= 2e-2 and rel_err(_host(dwk), rwk) <= 2e-2
