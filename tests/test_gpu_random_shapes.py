"""Seeded random shapes through every entry point family: forward, backward (single pass and segments; bf16 and fp32
tensors) and the delta rule's backward, each against the oracle at the usual bars.  The draws cover ragged lengths around block and
chunk boundaries, every supported head width, odd head counts, optional write gates and state cotangents."""
import numpy as np
import pytest

import sla_inputs as si
from gpu_util import GDN, GLA, RETNET, check
from test_gpu_backward import check_backward
from test_gpu_backward_gdn import check_backward_gdn

pytestmark = pytest.mark.gpu


def draw(seed):
    r = np.random.default_rng(seed)
    return dict(
        B=int(r.integers(1, 4)),
        T=int(r.choice([1, 7, 15, 16, 17, 31, 33, 63, 64, 65, 100, 255, 257, 300, 511, 513, 700])),
        H=int(r.choice([1, 2, 3, 5, 8, 12])),
        dk=int(r.choice([32, 64, 128])),
        dv=int(r.choice([64, 128, 256])),
        states=bool(r.integers(0, 2)),
        k_logits=bool(r.integers(0, 4) > 0),
    )


@pytest.mark.parametrize("seed", range(3000, 3012))
@pytest.mark.parametrize("variant", [RETNET, GLA, GDN])
def test_forward(variant, seed):
    c = draw(seed + 100 * variant)
    dtype = "bf16" if seed % 3 else "f32"
    d = si.custom(variant, dtype, B=c["B"], T=c["T"], H=c["H"], dk=c["dk"], dv=c["dv"], seed=seed)
    if not c["k_logits"]:
        d["k_logits"] = None
    s0 = si.initial_state(c["B"], c["H"], c["dk"], c["dv"], seed=seed + 1) if c["states"] else None
    check(variant, d, dtype, initial_state=s0, label=f"random {c}")


@pytest.mark.parametrize("seed", range(3100, 3112))
@pytest.mark.parametrize("variant", [RETNET, GLA])
def test_backward(variant, seed):
    c = draw(seed + 100 * variant)
    dtype = "bf16" if seed % 3 else "f32"
    d = si.custom(variant, dtype, B=c["B"], T=c["T"], H=c["H"], dk=c["dk"], dv=c["dv"], seed=seed)
    if not c["k_logits"]:
        d["k_logits"] = None
    cot = si.cotangents(c["B"], c["T"], c["H"], c["dk"], c["dv"], seed=seed + 1, final_state=c["states"])
    s0 = si.initial_state(c["B"], c["H"], c["dk"], c["dv"], seed=seed + 2) if c["states"] else None
    # the segment schedule: bf16 tensors, key heads of 64 and up
    segments = 2 if (seed % 2 and c["T"] >= 511 and dtype == "bf16" and c["dk"] >= 64) else 1
    check_backward(variant, d, cot, s0=s0, want_ds0=c["states"], label=f"random {dtype} {c} segments={segments}",
                   segments=segments, dtype=dtype)


@pytest.mark.parametrize("seed", range(3200, 3212))
def test_backward_gdn(seed):
    c = draw(seed)
    dtype = "bf16" if seed % 3 else "f32"
    d = si.custom(GDN, dtype, B=c["B"], T=c["T"], H=c["H"], dk=c["dk"], dv=c["dv"], seed=seed)
    if not c["k_logits"]:
        d["k_logits"] = None
    cot = si.cotangents(c["B"], c["T"], c["H"], c["dk"], c["dv"], seed=seed + 1, dtype=dtype, final_state=c["states"])
    s0 = si.initial_state(c["B"], c["H"], c["dk"], c["dv"], seed=seed + 2) if c["states"] else None
    check_backward_gdn(d, cot, s0=s0, want_ds0=c["states"], label=f"random {c}", dtype=dtype)
