"""GPU parity of the backward passes for key heads of width 32 (dk = 32, dv = 64: the H = 16 point of the head-count
ablation at fixed width), which run zero-padded to width 64: same oracle, same bars as the other widths."""
import numpy as np
import pytest

import sla_inputs as si
from gpu_util import GDN, GLA, RETNET
from test_gpu_backward import check_backward
from test_gpu_backward_gdn import check_backward_gdn

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("variant", [RETNET, GLA])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("dv", [64, 128])
def test_retnet_gla(variant, dtype, dv):
    B, T, H, dk = 2, 203, 5, 32
    d = si.custom(variant, dtype, B=B, T=T, H=H, dk=dk, dv=dv, seed=2900 + variant + dv)
    cot = si.cotangents(B, T, H, dk, dv, seed=2901, final_state=True)
    s0 = si.initial_state(B, H, dk, dv, seed=29)
    check_backward(variant, d, cot, s0, want_ds0=True, dtype=dtype,
                   label=f"dk=32 {dtype} {si.VARIANT_NAMES[variant]} dv={dv}")


@pytest.mark.parametrize("variant", [RETNET, GLA])
def test_without_states(variant):
    d = si.custom(variant, "bf16", B=1, T=70, H=16, dk=32, dv=64, seed=2910 + variant)
    cot = si.cotangents(1, 70, 16, 32, 64, seed=2911)
    check_backward(variant, d, cot, label=f"dk=32 {si.VARIANT_NAMES[variant]} H=16 no states")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_delta_rule(dtype):
    B, T, H, dk, dv = 2, 203, 3, 32, 64
    d = si.custom(GDN, dtype, B=B, T=T, H=H, dk=dk, dv=dv, seed=2920)
    cot = si.cotangents(B, T, H, dk, dv, seed=2921, final_state=True)
    s0 = si.initial_state(B, H, dk, dv, seed=2922)
    check_backward_gdn(d, cot, s0=s0, want_ds0=True, dtype=dtype, label=f"dk=32 {dtype} gdn")


def test_paper_shape_h16():
    """gla_paper_h16 (B=8, T=4096, H=16, dk=32, dv=64), every batch row against the C gradient oracle."""
    w = si.workload("gla_paper_h16")
    d = si.generate(w)
    cot = si.cotangents(w.B, w.T, w.H, w.dk, w.dv, seed=w.seed + 50)
    check_backward(w.variant, d, cot, label="gla_paper_h16", c_oracle=True)
