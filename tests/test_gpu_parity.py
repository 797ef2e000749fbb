"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest

import sla_inputs as si
from gpu_util import GDN, GLA, RETNET, TOL, check, rel_err, run_gpu, run_oracle

pytestmark = pytest.mark.gpu

VARIANTS = [RETNET, GLA, GDN]


def _name(v):
    return si.VARIANT_NAMES[v]


# ------------------------------------------------------------------ the benchmark definition's small case
def test_config1_gla_tiny_fp32():
    w = si.workload("gla_tiny")
    check(w.variant, si.generate(w), w.dtype, label="gla_tiny")


# ------------------------------------------------------------------ several tiles + ragged tails, all slice widths
@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("dv_split", [16, 32, 64])
def test_ragged_multi_tile(variant, dtype, dv_split):
    d = si.custom(variant, dtype, B=2, T=203, H=5, dk=128, dv=128, seed=100 + variant)
    s0 = si.initial_state(2, 5, 128, 128, seed=7)
    check(variant, d, dtype, s0, dv_split, label=f"{_name(variant)} T=203 H=5 d=128")


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("dk,dv", [(64, 64), (64, 128), (128, 64), (32, 64), (32, 128)])
def test_head_widths(variant, dk, dv):
    for dtype in ("f32", "bf16"):
        d = si.custom(variant, dtype, B=1, T=130, H=3, dk=dk, dv=dv, seed=200 + dk + dv)
        check(variant, d, dtype, label=f"{_name(variant)} dk={dk} dv={dv}")


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("dk", [64, 128])
def test_wide_values(variant, dk):
    """dv = 256 (the paper's 340M-class GLA shape has dk = 128, dv = 256): four 64-column slices per head."""
    for dtype in ("f32", "bf16"):
        d = si.custom(variant, dtype, B=1, T=150, H=2, dk=dk, dv=256, seed=250 + dk)
        s0 = si.initial_state(1, 2, dk, 256, seed=8)
        check(variant, d, dtype, s0, label=f"{_name(variant)} dk={dk} dv=256")


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("T", [1, 2, 15, 16, 17, 63, 64, 65])
def test_short_sequences(variant, T):
    d = si.custom(variant, "bf16", B=2, T=T, H=4, dk=128, dv=64, seed=300 + T)
    check(variant, d, "bf16", label=f"{_name(variant)} T={T}")


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("H", [1, 2, 7, 16, 32, 64])
def test_head_counts(variant, H):
    d = si.custom(variant, "bf16", B=1, T=96, H=H, dk=64, dv=64, seed=400 + H)
    check(variant, d, "bf16", label=f"{_name(variant)} H={H}")


# ------------------------------------------------------------------ gating modes and invariants on the device
@pytest.mark.parametrize("variant", VARIANTS)
def test_read_gate_only(variant):
    d = si.custom(variant, "bf16", B=1, T=150, H=4, dk=128, dv=128, seed=500, dual_gates=False)
    assert d["k_logits"] is None
    check(variant, d, "bf16", label=f"{_name(variant)} read-gate only")


@pytest.mark.parametrize("variant", VARIANTS)
def test_saturated_logits_give_exact_zeros(variant):
    """Thm 4.2 limit: a saturated gate selects one head; the others must be exactly zero."""
    H, sel = 4, 1
    d = si.custom(variant, "bf16", B=1, T=100, H=H, dk=128, dv=128, seed=600)
    sat = np.zeros_like(d["q_logits"]); sat[..., sel] = 1e4
    d["q_logits"] = sat; d["k_logits"] = sat.copy()
    o, f, ro, rf = check(variant, d, "bf16", label=f"{_name(variant)} saturated")
    others = [h for h in range(H) if h != sel]
    assert np.all(o[:, :, others] == 0.0)
    assert np.all(f[:, others] == 0.0)


@pytest.mark.parametrize("variant", VARIANTS)
def test_uniform_logits_scale_by_head_count(variant):
    H = 4
    d = si.custom(variant, "bf16", B=1, T=80, H=H, dk=64, dv=64, seed=700)
    d["q_logits"] = np.full_like(d["q_logits"], 0.3); d["k_logits"] = np.full_like(d["k_logits"], -1.2)
    o, f = run_gpu(variant, d, "bf16")
    d1 = dict(d); d1["k_logits"] = None
    o1, f1 = run_gpu(variant, d1, "bf16")
    # write gate 1/H scales state and output by exactly 1/H (a power of two: exact in every rounding)
    np.testing.assert_array_equal(f * H, f1)
    np.testing.assert_allclose(o * H, o1, rtol=2 ** -7, atol=1e-6)


def test_winner_take_all_mismatch_blocks_flow():
    """Thm 4.3: tokens written under one winning head are invisible to queries that pick another."""
    H = 4
    d = si.custom(GLA, "bf16", B=1, T=70, H=H, dk=64, dv=64, seed=800)
    wq = np.zeros_like(d["q_logits"]); wq[..., 0] = 1e4
    wk = np.zeros_like(d["k_logits"]); wk[..., 2] = 1e4
    d["q_logits"], d["k_logits"] = wq, wk
    o, f = run_gpu(GLA, d, "bf16")
    assert np.all(o == 0.0)
    assert np.abs(f[:, 2]).max() > 0


# ------------------------------------------------------------------ state carry
@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("split", [16, 37, 64, 100])
def test_chained_calls_match_single_call(variant, split):
    T = 140
    d = si.custom(variant, "f32", B=1, T=T, H=2, dk=64, dv=64, seed=900)
    o, f = run_gpu(variant, d, "f32")

    def cut(lo, hi):
        c = {}
        for key, a in d.items():
            if a is None or (key == "log_decay" and variant == RETNET):
                c[key] = a
            else:
                c[key] = np.ascontiguousarray(a[:, lo:hi])
        return c

    o1, f1 = run_gpu(variant, cut(0, split), "f32")
    o2, f2 = run_gpu(variant, cut(split, T), "f32", initial_state=f1.astype(np.float32))
    assert rel_err(np.concatenate([o1, o2], 1), o) <= 1e-5
    assert rel_err(f2, f) <= 1e-5


def test_zero_length_passes_state_through():
    import torch
    import paper_2602_01744_amd as sla

    s0 = torch.from_numpy(si.initial_state(2, 3, 64, 64, seed=3)).cuda()
    e = lambda *s, dt=torch.float32: torch.empty(s, dtype=dt, device="cuda")
    out, fin = sla.forward(GLA, e(2, 0, 3, 64), e(2, 0, 3, 64), e(2, 0, 3, 64), e(2, 0, 3), None, e(2, 0, 3, 64), None, s0)
    torch.cuda.synchronize()
    assert torch.equal(fin, s0)
    out, fin = sla.forward(GLA, e(2, 0, 3, 64), e(2, 0, 3, 64), e(2, 0, 3, 64), e(2, 0, 3), None, e(2, 0, 3, 64), None, None)
    torch.cuda.synchronize()
    assert torch.count_nonzero(fin).item() == 0


# ------------------------------------------------------------------ robustness
def test_strong_decay_within_documented_range():
    """log-decay down to -4 per token (documented bound: -5): the 1/p factors reach e^64 and must not overflow."""
    d = si.custom(GLA, "bf16", B=1, T=100, H=2, dk=128, dv=64, seed=1000)
    rng = np.random.default_rng(5)
    ld = -rng.uniform(0.0, 4.0, size=d["log_decay"].shape).astype(np.float32)
    ld[:, :, :, :8] = -4.0
    d["log_decay"] = si.round_to_bf16(ld)
    check(GLA, d, "bf16", label="gla strong decay")
    d32 = dict(d);
    check(GLA, d32, "f32", label="gla strong decay fp32")


@pytest.mark.parametrize("variant", VARIANTS)
def test_bitwise_determinism(variant):
    d = si.custom(variant, "bf16", B=2, T=300, H=4, dk=128, dv=128, seed=1100)
    o1, f1 = run_gpu(variant, d, "bf16")
    o2, f2 = run_gpu(variant, d, "bf16")
    np.testing.assert_array_equal(o1, o2)
    np.testing.assert_array_equal(f1, f2)
    o3, f3 = run_gpu(variant, d, "bf16", dv_split=16)
    np.testing.assert_array_equal(o1, o3)  # the slice width is a schedule, not a result
    np.testing.assert_array_equal(f1, f3)


def test_final_state_may_be_skipped_and_may_alias_initial_state():
    import torch
    import paper_2602_01744_amd as sla
    from gpu_util import to_device

    d = si.custom(GLA, "bf16", B=1, T=90, H=2, dk=64, dv=64, seed=1200)
    g, _ = to_device(d, "bf16", GLA)
    s0 = torch.from_numpy(si.initial_state(1, 2, 64, 64, seed=4)).cuda()
    ref_out, ref_fin = sla.forward(GLA, g["q"], g["k"], g["v"], g["q_logits"], g["k_logits"], g["log_decay"], None, s0.clone())
    out, none = sla.forward(GLA, g["q"], g["k"], g["v"], g["q_logits"], g["k_logits"], g["log_decay"], None, s0.clone(),
                            want_final_state=False)
    assert none is None
    st = s0.clone()
    out2, fin2 = sla.forward(GLA, g["q"], g["k"], g["v"], g["q_logits"], g["k_logits"], g["log_decay"], None, st, final_state=st)
    torch.cuda.synchronize()
    assert torch.equal(out, ref_out) and torch.equal(out2, ref_out) and torch.equal(fin2, ref_fin)


def test_device_status_word_reports_out_of_range_decay():
    """The sticky device status word: zero after ordinary calls (no hand-over wait ever expired), and a GLA block
    whose accumulated decay leaves the documented range sets SLA_DEVICE_DECAY_RANGE; the reset clears it."""
    import paper_2602_01744_amd as sla

    rc, _ = sla.sla_device_status(reset=True)
    assert rc == 0
    for variant in VARIANTS:
        d = si.custom(variant, "bf16", B=2, T=200, H=4, dk=128, dv=128, seed=1900 + variant)
        run_gpu(variant, d, "bf16")
        run_gpu(variant, d, "f32")
    rc, word = sla.sla_device_status()
    assert rc == 0 and word == 0, word
    # log-decay -8 per token on a few key dimensions: 16 tokens accumulate e^-128, below e^-80
    d = si.custom(GLA, "bf16", B=1, T=64, H=2, dk=128, dv=64, seed=1950)
    ld = d["log_decay"].copy()
    ld[:, :, :, :4] = -8.0
    d["log_decay"] = si.round_to_bf16(ld)
    run_gpu(GLA, d, "bf16")
    rc, word = sla.sla_device_status(reset=True)
    assert rc == 0 and word == sla.DEVICE_DECAY_RANGE, word
    rc, word = sla.sla_device_status()
    assert rc == 0 and word == 0, word


@pytest.mark.parametrize("variant", [RETNET, GDN])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_scalar_decay_of_any_strength(variant, dtype):
    """RetNet and the delta rule take any decay <= 0.  Their kernels keep the state divided by a pending decay
    factor and fold it in when it gets small: weak decay (folded every few hundred tokens), strong decay (every
    block) and changes between the two within a sequence must all agree with the oracle."""
    d = si.custom(variant, dtype, B=2, T=700, H=5, dk=128, dv=64, seed=2000 + variant)
    rng = np.random.default_rng(21)
    if variant == RETNET:
        d["log_decay"] = np.array([-1e-4, -0.05, -0.9, -3.0, -7.0], dtype=np.float32)
    else:
        ld = -rng.choice([1e-4, 0.02, 0.3, 2.0, 6.0], size=d["log_decay"].shape).astype(np.float32)
        ld[:, 200:330] = -1e-3   # a long stretch of weak decay after strong ones, then strong again
        ld[:, 330:360] = -5.0
        d["log_decay"] = ld
    s0 = si.initial_state(2, 5, 128, 64, seed=22)
    check(variant, d, dtype, s0, label=f"{si.VARIANT_NAMES[variant]} mixed decay strengths")


@pytest.mark.parametrize("variant", VARIANTS)
def test_narrow_keys_ragged_segments_and_state(variant):
    """dk = 32 (the H = 16 point of the head ablation at fixed model width): half of a producer wave's lanes own no
    key dimension.  Ragged length, an initial state, every slice width, and the segment schedule."""
    d = si.custom(variant, "bf16", B=2, T=333, H=16, dk=32, dv=64, seed=2100 + variant)
    s0 = si.initial_state(2, 16, 32, 64, seed=23)
    for dv_split in (0, 16, 32):
        check(variant, d, "bf16", s0, dv_split, label=f"{_name(variant)} dk=32 dv=64 H=16")
    check(variant, d, "f32", s0, label=f"{_name(variant)} dk=32 dv=64 H=16 fp32")
    if variant != GDN:
        d = si.custom(variant, "bf16", B=1, T=900, H=4, dk=32, dv=64, seed=2200 + variant)
        check(variant, d, "bf16", label=f"{_name(variant)} dk=32, 3 segments", segments=3)
