"""SLA_FLAG_HEAD_MAJOR: the forward on [B,H,T,d] tensors must give, bit for bit, the result it gives on the same
values in the [B,T,H,d] layout (the arithmetic is the same, only addresses differ), and that result is held to the
oracle by the other parity tests."""
import numpy as np
import pytest

import sla_inputs as si
from gpu_util import GDN, GLA, RETNET, to_device

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("variant", [RETNET, GLA, GDN])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("segments", [1, 3])
def test_head_major_matches_token_major(variant, dtype, segments):
    import torch
    import paper_2602_01744_amd as sla

    if variant == GDN and segments > 1:
        pytest.skip("the delta rule runs one pass")
    B, T, H, dk, dv = 2, 900, 5, 128, 128
    d = si.custom(variant, dtype, B=B, T=T, H=H, dk=dk, dv=dv, seed=3100 + variant)
    g, _ = to_device(d, dtype, variant)
    s0 = torch.from_numpy(si.initial_state(B, H, dk, dv, seed=31)).cuda()
    ref_out, ref_fin = sla.forward(variant, g["q"], g["k"], g["v"], g["q_logits"], g["k_logits"], g["log_decay"],
                                   g["beta"], s0, segments=segments)
    hm = lambda t: t.permute(0, 2, 1, 3).contiguous()
    ld = hm(g["log_decay"]) if variant == GLA else g["log_decay"]
    out, fin = sla.forward(variant, hm(g["q"]), hm(g["k"]), hm(g["v"]), g["q_logits"], g["k_logits"], ld, g["beta"], s0,
                           segments=segments, head_major=True)
    torch.cuda.synchronize()
    assert out.shape == (B, H, T, dv)
    assert torch.equal(out.permute(0, 2, 1, 3), ref_out) and torch.equal(fin, ref_fin)


def test_head_major_widths_and_ragged_length():
    import torch
    import paper_2602_01744_amd as sla

    for dk, dv, T in ((64, 256, 203), (128, 64, 17), (64, 64, 1)):
        d = si.custom(GLA, "bf16", B=3, T=T, H=4, dk=dk, dv=dv, seed=3200 + dk + dv)
        g, _ = to_device(d, "bf16", GLA)
        ref_out, ref_fin = sla.forward(GLA, g["q"], g["k"], g["v"], g["q_logits"], g["k_logits"], g["log_decay"])
        hm = lambda t: t.permute(0, 2, 1, 3).contiguous()
        out, fin = sla.forward(GLA, hm(g["q"]), hm(g["k"]), hm(g["v"]), g["q_logits"], g["k_logits"],
                               hm(g["log_decay"]), head_major=True)
        torch.cuda.synchronize()
        assert torch.equal(out.permute(0, 2, 1, 3), ref_out) and torch.equal(fin, ref_fin)


@pytest.mark.parametrize("variant", [RETNET, GLA])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_backward_head_major_matches_token_major(variant, dtype):
    import torch
    import paper_2602_01744_amd as sla

    B, T, H, dk, dv = 2, 203, 5, 128, 64
    d = si.custom(variant, dtype, B=B, T=T, H=H, dk=dk, dv=dv, seed=3300 + variant)
    g, tdt = to_device(d, dtype, variant)
    cot = si.cotangents(B, T, H, dk, dv, seed=3301, final_state=True)
    dout = torch.from_numpy(cot["d_out"]).to(tdt).cuda()
    dsf = torch.from_numpy(cot["d_final_state"]).cuda()
    s0 = torch.from_numpy(si.initial_state(B, H, dk, dv, seed=33)).cuda()
    ref = sla.backward(variant, g["q"], g["k"], g["v"], g["q_logits"], g["k_logits"], g["log_decay"], dout, s0, dsf,
                       want_d_initial_state=True)
    hm = lambda t: t.permute(0, 2, 1, 3).contiguous()
    ld = hm(g["log_decay"]) if variant == GLA else g["log_decay"]
    got = sla.backward(variant, hm(g["q"]), hm(g["k"]), hm(g["v"]), g["q_logits"], g["k_logits"], ld, hm(dout), s0, dsf,
                       want_d_initial_state=True, head_major=True)
    torch.cuda.synchronize()
    for n in ("dq", "dk", "dv", "dlog_decay"):
        if ref[n] is not None and ref[n].dim() == 4:
            assert torch.equal(got[n].permute(0, 2, 1, 3), ref[n]), n
    for n in ("dq_head_logits", "dk_head_logits", "d_initial_state"):
        assert torch.equal(got[n], ref[n]), n


@pytest.mark.timeout(600)
def test_head_major_full_size_against_the_oracle():
    """The headline workload with its wide tensors laid out [B,H,T,d], compared with the CPU oracle directly (not only
    with the other layout's result): out, final state, and the worst (batch, head) slice."""
    import torch
    import paper_2602_01744_amd as sla
    from gpu_util import TOL, rel_err, run_oracle, worst_slice_err

    w = si.workload("gla_train")
    d = si.generate(w)
    g, _ = to_device(d, w.dtype, w.variant)
    hm = lambda t: t.permute(0, 2, 1, 3).contiguous()
    out, fin = sla.forward(w.variant, hm(g["q"]), hm(g["k"]), hm(g["v"]), g["q_logits"], g["k_logits"],
                           hm(g["log_decay"]), head_major=True)
    torch.cuda.synchronize()
    o = out.permute(0, 2, 1, 3).to(torch.float32).cpu().numpy().astype(np.float64)
    f = fin.cpu().numpy().astype(np.float64)
    ro, rf = run_oracle(w.variant, d)
    tol = TOL[w.dtype]
    assert rel_err(o, ro) <= tol and rel_err(f, rf) <= tol
    assert worst_slice_err(o, ro, 2) <= tol and worst_slice_err(f, rf, 1) <= tol
