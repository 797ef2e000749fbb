"""GPU parity of sla_gate_logits (the projection in front of Eq. 4) against the oracle's statement of it, and of
the chain gate logits -> forward against the oracle run on the oracle's own logits."""
import numpy as np
import pytest

import sla_inputs as si
from gpu_util import GLA, RETNET, TOL, rel_err, to_device
from oracle import sla_numpy

pytestmark = pytest.mark.gpu


def run(d, w, dtype, both=True):
    import torch
    import paper_2602_01744_amd as sla

    g, _ = to_device(d, dtype, GLA)
    wq = torch.from_numpy(w["w_gq"]).cuda()
    wk = torch.from_numpy(w["w_gk"]).cuda()
    ql, kl = sla.gate_logits(g["q"], g["k"] if both else None, wq, wk if both else None, dv=d["v"].shape[-1])
    torch.cuda.synchronize()
    return ql.cpu().numpy().astype(np.float64), None if kl is None else kl.cpu().numpy().astype(np.float64)


# fp32 accumulation of dk products of bf16 / fp32 inputs against fp64: summation order only
LOGIT_TOL = 1e-5


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("H,dk", [(1, 64), (3, 64), (4, 128), (5, 128), (16, 128), (64, 64), (64, 128), (16, 32), (5, 32)])
def test_gate_logits_parity(dtype, H, dk):
    B, T = 2, 203
    d = si.custom(GLA, dtype, B=B, T=T, H=H, dk=dk, dv=64, seed=1000 + H + dk)
    w = si.gate_weights(H, dk, seed=1001 + H)
    ql, kl = run(d, w, dtype)
    rq, rk = sla_numpy.gate_logits(d["q"], w["w_gq"]), sla_numpy.gate_logits(d["k"], w["w_gk"])
    eq, ek = rel_err(ql, rq), rel_err(kl, rk)
    print(f"[gate logits] {dtype} H={H} dk={dk} q_err={eq:.2e} k_err={ek:.2e}", flush=True)
    assert eq <= LOGIT_TOL and ek <= LOGIT_TOL


@pytest.mark.parametrize("T", [1, 2, 3, 4, 5, 17])
def test_gate_logits_short_and_read_gate_only(T):
    d = si.custom(GLA, "bf16", B=1, T=T, H=4, dk=128, dv=64, seed=1100 + T)
    w = si.gate_weights(4, 128, seed=1101)
    ql, kl = run(d, w, "bf16", both=False)
    assert kl is None
    assert rel_err(ql, sla_numpy.gate_logits(d["q"], w["w_gq"])) <= LOGIT_TOL


@pytest.mark.parametrize("variant", [RETNET, GLA])
def test_prologue_then_forward(variant):
    """Logits from the GPU prologue feed the GPU forward; the oracle computes its own logits from the same
    weights.  Checks that the two entry points agree on the layout of the logits."""
    import torch
    import paper_2602_01744_amd as sla
    import oracle

    B, T, H, dk, dv = 2, 150, 8, 128, 128
    d = si.custom(variant, "bf16", B=B, T=T, H=H, dk=dk, dv=dv, seed=1200 + variant)
    w = si.gate_weights(H, dk, seed=1201)
    g, _ = to_device(d, "bf16", variant)
    ql, kl = sla.gate_logits(g["q"], g["k"], torch.from_numpy(w["w_gq"]).cuda(), torch.from_numpy(w["w_gk"]).cuda(), dv=dv)
    out, fin = sla.forward(variant, g["q"], g["k"], g["v"], ql, kl, g["log_decay"])
    torch.cuda.synchronize()
    rq = sla_numpy.gate_logits(d["q"], w["w_gq"]).astype(np.float32)
    rk = sla_numpy.gate_logits(d["k"], w["w_gk"]).astype(np.float32)
    ro, rf = oracle.forward(variant, d["q"], d["k"], d["v"], rq, rk, d["log_decay"], None, None)
    assert rel_err(out.float().cpu().numpy().astype(np.float64), ro) <= TOL["bf16"]
    assert rel_err(fin.cpu().numpy().astype(np.float64), rf) <= TOL["bf16"]


def test_full_size():
    w0 = si.workload("gla_train")
    d = si.generate(w0)
    w = si.gate_weights(w0.H, w0.dk, seed=1300)
    ql, kl = run(d, w, "bf16")
    rows = slice(0, 2)  # the oracle on two batch rows
    assert rel_err(ql[rows], sla_numpy.gate_logits(d["q"][rows], w["w_gq"])) <= LOGIT_TOL
    assert rel_err(kl[rows], sla_numpy.gate_logits(d["k"][rows], w["w_gk"])) <= LOGIT_TOL


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("taps", [1, 2, 3, 4])
@pytest.mark.parametrize("B,T,C", [(2, 203, 256), (1, 64, 8), (3, 1, 64), (1, 129, 2048)])
def test_short_conv_silu_parity(dtype, taps, B, T, C):
    import torch
    import paper_2602_01744_amd as sla

    r = np.random.default_rng(1500 + taps + T)
    x = r.standard_normal(size=(B, T, C)).astype(np.float32)
    if dtype == "bf16":
        x = si.round_to_bf16(x)
    w = (r.standard_normal(size=(C, taps)) / np.sqrt(taps)).astype(np.float32)
    xt = torch.from_numpy(x).to(torch.bfloat16 if dtype == "bf16" else torch.float32).cuda()
    y = sla.short_conv_silu(xt, torch.from_numpy(w).cuda())
    torch.cuda.synchronize()
    got = y.float().cpu().numpy().astype(np.float64)
    want = sla_numpy.short_conv_silu(x, w)
    # fp32: summation order and the hardware exp2 (1 ulp); bf16: the output is rounded to bf16 (2^-9 relative)
    tol = 1e-5 if dtype == "f32" else 4e-3
    assert rel_err(got, want) <= tol


def test_short_conv_silu_full_size():
    import torch
    import paper_2602_01744_amd as sla

    w0 = si.workload("gdn")  # the delta-rule workload's q: [B, T, H * dk]
    r = np.random.default_rng(1600)
    C = w0.H * w0.dk
    x = si.round_to_bf16(r.standard_normal(size=(w0.B, w0.T, C)).astype(np.float32))
    w = (r.standard_normal(size=(C, 4)) / 2).astype(np.float32)
    y = sla.short_conv_silu(torch.from_numpy(x).to(torch.bfloat16).cuda(), torch.from_numpy(w).cuda())
    torch.cuda.synchronize()
    got = y[:1].float().cpu().numpy().astype(np.float64)  # the oracle on batch row 0
    assert rel_err(got, sla_numpy.short_conv_silu(x[:1], w)) <= 4e-3
