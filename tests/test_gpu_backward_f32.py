"""GPU parity of the backward pass on fp32 tensors (sla_backward with dtype SLA_F32: RetNet and GLA, token by token in
fp32 vector arithmetic) against the gradient oracle.  Tolerance: the forward's fp32 bar, max|x - x*| / max|x*| <= 1e-4
per gradient tensor and per (batch, head) slice: every operand is fp32 end to end, so what remains is summation order
and the 1-ulp hardware exponential."""
import numpy as np
import pytest

import sla_inputs as si
from gpu_util import GLA, RETNET, TOL
from test_gpu_backward import check_backward

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("variant", [RETNET, GLA])
def test_small_block_aligned(variant):
    d = si.custom(variant, "f32", B=1, T=32, H=2, dk=64, dv=64, seed=1900 + variant)
    cot = si.cotangents(1, 32, 2, 64, 64, seed=1901)
    check_backward(variant, d, cot, label=f"f32 {si.VARIANT_NAMES[variant]} T=32 d=64", dtype="f32")


@pytest.mark.parametrize("variant", [RETNET, GLA])
@pytest.mark.parametrize("states", [False, True])
def test_ragged_multi_tile(variant, states):
    B, T, H, dk, dv = 2, 203, 5, 128, 128
    d = si.custom(variant, "f32", B=B, T=T, H=H, dk=dk, dv=dv, seed=1910 + variant)
    cot = si.cotangents(B, T, H, dk, dv, seed=1911, final_state=states)
    s0 = si.initial_state(B, H, dk, dv, seed=19) if states else None
    check_backward(variant, d, cot, s0, want_ds0=states, dtype="f32",
                   label=f"f32 {si.VARIANT_NAMES[variant]} T=203 H=5 states={states}")


@pytest.mark.parametrize("variant", [RETNET, GLA])
@pytest.mark.parametrize("dk,dv", [(64, 64), (64, 128), (128, 64), (128, 256), (64, 256)])
def test_head_widths(variant, dk, dv):
    d = si.custom(variant, "f32", B=1, T=130, H=3, dk=dk, dv=dv, seed=1920 + dk + dv)
    cot = si.cotangents(1, 130, 3, dk, dv, seed=1921, final_state=True)
    s0 = si.initial_state(1, 3, dk, dv, seed=20)
    check_backward(variant, d, cot, s0, want_ds0=True, dtype="f32",
                   label=f"f32 {si.VARIANT_NAMES[variant]} dk={dk} dv={dv}")


@pytest.mark.parametrize("variant", [RETNET, GLA])
@pytest.mark.parametrize("T", [1, 15, 16, 17, 65])
def test_short_sequences(variant, T):
    d = si.custom(variant, "f32", B=2, T=T, H=4, dk=128, dv=64, seed=1930 + T)
    cot = si.cotangents(2, T, 4, 128, 64, seed=1931 + T, final_state=True)
    check_backward(variant, d, cot, None, want_ds0=True, dtype="f32", label=f"f32 {si.VARIANT_NAMES[variant]} T={T}")


@pytest.mark.parametrize("variant", [RETNET, GLA])
def test_read_gate_only(variant):
    d = si.custom(variant, "f32", B=1, T=90, H=7, dk=64, dv=128, seed=1950)
    d["k_logits"] = None
    cot = si.cotangents(1, 90, 7, 64, 128, seed=1951)
    got, _ = check_backward(variant, d, cot, dtype="f32", label=f"f32 {si.VARIANT_NAMES[variant]} read gate only")
    assert got["dk_head_logits"] is None


def test_any_decay_is_in_range():
    # the decay is applied token by token, so log-decays far below the block form's bound of -5 are fine
    B, T, H = 1, 100, 2
    d = si.custom(GLA, "f32", B=B, T=T, H=H, dk=64, dv=64, seed=1970)
    r = np.random.default_rng(1971)
    d["log_decay"] = (-40.0 * r.random(size=d["log_decay"].shape)).astype(np.float32)
    cot = si.cotangents(B, T, H, 64, 64, seed=1972)
    check_backward(GLA, d, cot, dtype="f32", label="f32 decay in [-40, 0]")


def test_long_sequence_decay_gradient():
    """dlog_decay sums q dq - k dk over every later token, two sums that nearly cancel: the running sum is kept in
    fp64, so the error of the earliest tokens stays at the fp32 bar."""
    B, T, H, dk, dv = 1, 4096 + 40, 2, 128, 128
    d = si.custom(GLA, "f32", B=B, T=T, H=H, dk=dk, dv=dv, seed=1977)
    cot = si.cotangents(B, T, H, dk, dv, seed=1978, final_state=True)
    s0 = si.initial_state(B, H, dk, dv, seed=1979)
    got, ref = check_backward(GLA, d, cot, s0=s0, want_ds0=True, dtype="f32", label=f"f32 long T={T}")
    scale = np.abs(ref["dlog_decay"]).max()
    early = np.abs(got["dlog_decay"][:, :512] - ref["dlog_decay"][:, :512]).max() / scale
    assert early <= TOL["f32"]


def test_segments_are_refused():
    import paper_2602_01744_amd as sla

    p = sla.SlaParams(GLA, sla.F32, 1, 1024, 2, 64, 64, 0, 0, 2)
    assert sla.sla_backward_workspace_bytes(p) == 0
    d = si.custom(GLA, "f32", B=1, T=1024, H=2, dk=64, dv=64, seed=1980)
    cot = si.cotangents(1, 1024, 2, 64, 64, seed=1981)
    with pytest.raises(sla.SlaError):
        check_backward(GLA, d, cot, dtype="f32", segments=2)


@pytest.mark.parametrize("name", ["gla_train", "retnet_train"])
def test_full_size(name):
    """The bench shapes (B=8, T=2048, H=16, d=128) held as fp32 tensors; every batch row against the C gradient oracle."""
    w = si.workload(name)
    d = si.generate(w)
    cot = si.cotangents(w.B, w.T, w.H, w.dk, w.dv, seed=w.seed + 50)
    check_backward(w.variant, d, cot, label=f"f32 {name}", c_oracle=True, dtype="f32")
