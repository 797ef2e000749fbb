"""GPU parity of the segment-parallel schedule (pre-pass, combine, main pass) against the CPU oracle and
against the single fused pass."""
import numpy as np
import pytest

import sla_inputs as si
from gpu_util import GDN, GLA, RETNET, check, rel_err, run_gpu

pytestmark = pytest.mark.gpu

SEG_VARIANTS = [RETNET, GLA]


def _name(v):
    return si.VARIANT_NAMES[v]


@pytest.mark.parametrize("variant", SEG_VARIANTS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("segments", [2, 3, 5])
def test_segments_match_oracle_ragged(variant, dtype, segments):
    # T = 1100: segments of 576, 384, 256 tokens with a ragged last one; initial state given
    d = si.custom(variant, dtype, B=2, T=1100, H=3, dk=128, dv=128, seed=1300 + variant)
    s0 = si.initial_state(2, 3, 128, 128, seed=11)
    check(variant, d, dtype, s0, label=f"{_name(variant)} T=1100", segments=segments)


@pytest.mark.parametrize("variant", SEG_VARIANTS)
@pytest.mark.parametrize("dk,dv,dv_split", [(64, 64, 16), (64, 128, 32), (128, 64, 64)])
def test_segments_head_widths_and_slices(variant, dk, dv, dv_split):
    for dtype in ("f32", "bf16"):
        d = si.custom(variant, dtype, B=1, T=777, H=2, dk=dk, dv=dv, seed=1400 + dk + dv)
        check(variant, d, dtype, None, dv_split, label=f"{_name(variant)} dk={dk} dv={dv}", segments=3)


@pytest.mark.parametrize("variant", SEG_VARIANTS)
def test_segments_agree_with_single_pass(variant):
    """Same inputs through both schedules: fp32 results agree to rounding of the chained states."""
    d = si.custom(variant, "f32", B=2, T=1536, H=4, dk=128, dv=128, seed=1500)
    s0 = si.initial_state(2, 4, 128, 128, seed=12)
    o1, f1 = run_gpu(variant, d, "f32", s0)
    for segments in (2, 4, 6):
        o2, f2 = run_gpu(variant, d, "f32", s0, segments=segments)
        assert rel_err(o2, o1) <= 2e-5, segments
        assert rel_err(f2, f1) <= 2e-5, segments
    # the library's own choice (few rows: it will cut) and a fixed schedule are bitwise reproducible
    o3, f3 = run_gpu(variant, d, "f32", s0, segments=0)
    o4, f4 = run_gpu(variant, d, "f32", s0, segments=0)
    np.testing.assert_array_equal(o3, o4)
    np.testing.assert_array_equal(f3, f4)
    assert rel_err(o3, o1) <= 2e-5 and rel_err(f3, f1) <= 2e-5


def test_segments_strong_decay_gla():
    """Strong decay: the segment decay products underflow towards zero; the chained states must stay finite."""
    d = si.custom(GLA, "bf16", B=1, T=1024, H=2, dk=128, dv=64, seed=1600)
    rng = np.random.default_rng(6)
    ld = -rng.uniform(0.0, 4.0, size=d["log_decay"].shape).astype(np.float32)
    ld[:, :, :, :8] = -4.0
    d["log_decay"] = si.round_to_bf16(ld)
    s0 = si.initial_state(1, 2, 128, 64, seed=13)
    check(GLA, d, "bf16", s0, label="gla strong decay, segments", segments=4)


def test_short_sequences_fall_back_to_one_pass():
    # T below two minimum segments: the request is reduced to one pass and must still be right
    d = si.custom(GLA, "bf16", B=1, T=200, H=2, dk=64, dv=64, seed=1700)
    check(GLA, d, "bf16", label="gla T=200 segments=4", segments=4)


def test_final_state_may_alias_initial_state_with_segments():
    import torch
    import paper_2602_01744_amd as sla
    from gpu_util import to_device

    d = si.custom(GLA, "bf16", B=2, T=1024, H=4, dk=64, dv=64, seed=1800)
    g, _ = to_device(d, "bf16", GLA)
    s0 = torch.from_numpy(si.initial_state(2, 4, 64, 64, seed=14)).cuda()
    ref_out, ref_fin = sla.forward(GLA, g["q"], g["k"], g["v"], g["q_logits"], g["k_logits"], g["log_decay"], None,
                                   s0.clone(), segments=4)
    st = s0.clone()
    out, fin = sla.forward(GLA, g["q"], g["k"], g["v"], g["q_logits"], g["k_logits"], g["log_decay"], None, st,
                           final_state=st, segments=4)
    torch.cuda.synchronize()
    assert torch.equal(out, ref_out) and torch.equal(fin, ref_fin)


def test_delta_rule_has_no_segment_schedule():
    import paper_2602_01744_amd as sla

    d = si.custom(GDN, "bf16", B=1, T=512, H=2, dk=64, dv=64, seed=1900)
    with pytest.raises(sla.SlaError) as e:
        run_gpu(GDN, d, "bf16", segments=2)
    assert e.value.status == -3
    check(GDN, d, "bf16", label="gdn segments=0 (one pass)", segments=0)


def test_workspace_too_small():
    import torch
    import paper_2602_01744_amd as sla
    from gpu_util import to_device

    d = si.custom(RETNET, "bf16", B=1, T=1024, H=2, dk=64, dv=64, seed=2000)
    g, _ = to_device(d, "bf16", RETNET)
    tiny = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(sla.SlaError) as e:
        sla.forward(RETNET, g["q"], g["k"], g["v"], g["q_logits"], g["k_logits"], g["log_decay"], None, None,
                    segments=4, workspace=tiny)
    assert e.value.status == -6
    # the library's own choice falls back to one pass instead
    o, f = sla.forward(RETNET, g["q"], g["k"], g["v"], g["q_logits"], g["k_logits"], g["log_decay"], None, None,
                       segments=0, workspace=tiny)
    o1, f1 = sla.forward(RETNET, g["q"], g["k"], g["v"], g["q_logits"], g["k_logits"], g["log_decay"], None, None)
    torch.cuda.synchronize()
    assert torch.equal(o, o1) and torch.equal(f, f1)
