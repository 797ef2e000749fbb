"""GPU parity at the full sizes of the benchmark definition, in the launch configuration bench.py times
(default slice width).  The C oracle finishes each of these in seconds on the machine's host cores, so whole
tensors are compared, not samples."""
import numpy as np
import pytest

import sla_inputs as si
from gpu_util import check, rel_err, run_gpu

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]


@pytest.mark.parametrize("name", ["retnet", "gla_train", "gdn", "retnet_train", "gdn_train", "gla_paper_h16", "gdn_paper_h4"])
def test_full_size_workload(name):
    w = si.workload(name)
    check(w.variant, si.generate(w), w.dtype, label=f"full {name}")


@pytest.mark.parametrize("name", ["retnet", "gla_long", "gla_paper_h4", "gla_paper_h8", "retnet_paper_h4"])
def test_full_size_segmented(name):
    """The 32-sequence workloads in the schedule bench.py times: the library's own choice of segments."""
    import torch
    import paper_2602_01744_amd as sla

    w = si.workload(name)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    p = sla.SlaParams(w.variant, 1 if w.dtype == "bf16" else 0, w.B, w.T, w.H, w.dk, w.dv, 0, 0, 0)
    assert sla.sla_segments(p, cus) > 1
    check(w.variant, si.generate(w), w.dtype, label=f"full {name}, segments chosen by the library", segments=0)


def test_full_size_long_context():
    """B=1, T=65536, H=32: 1024 chunks of state carry in the winner-take-all regime (peaked logits)."""
    w = si.workload("gla_long")
    d = si.generate(w)
    o, f, ro, rf = check(w.variant, d, w.dtype, label="full gla_long")
    # the losing heads of a segment get gates of about e^-6: their outputs are small but must still be right
    # relative to their own scale, head by head
    for h in range(0, w.H, 5):
        assert rel_err(o[:, :, h], ro[:, :, h]) <= 2e-2
    del o, ro
    # split-call chaining at full size: state carry through initial_state is exact to fp32 rounding
    half = w.T // 2 + 37  # not a multiple of the block or of the staging chunk

    def cut(lo, hi):
        return {k: (None if a is None else np.ascontiguousarray(a[:, lo:hi])) for k, a in d.items()}

    o1, f1 = run_gpu(w.variant, cut(0, half), w.dtype)
    o2, f2 = run_gpu(w.variant, cut(half, w.T), w.dtype, initial_state=f1.astype(np.float32))
    assert rel_err(f2, rf) <= 2e-2
    assert rel_err(f2, f) <= 1e-2
