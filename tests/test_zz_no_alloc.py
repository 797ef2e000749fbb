"""sla_forward_static (the entry point that allocates nothing: its segment workspace is a buffer inside the
library's device image) against sla_forward_ws with a caller-owned workspace, through the C ABI.

Both run the same kernels on the same schedule, so the results must be bit-identical; the oracle comparison is
added on top.  Two calls in a row share the one static buffer, the second with a smaller input: nothing of the
first call's contents may leak into it."""
import numpy as np
import pytest

import sla_inputs as si
from gpu_util import GLA, RETNET, TOL, rel_err, run_oracle, to_device

pytestmark = pytest.mark.gpu


def _both(variant, d, dtype, segments, initial_state=None):
    import torch

    import paper_2602_01744_amd as sla

    g, tdt = to_device(d, dtype, variant)
    B, T, H, dk = g["q"].shape
    dv = g["v"].shape[-1]
    dev = g["q"].device
    s0 = None if initial_state is None else torch.from_numpy(np.ascontiguousarray(initial_state, dtype=np.float32)).to(dev)
    params = sla.SlaParams(variant, sla.BF16 if dtype == "bf16" else sla.F32, B, T, H, dk, dv, 0, 0, segments)
    cus = torch.cuda.get_device_properties(dev).multi_processor_count
    need = sla.sla_workspace_bytes(params, cus)
    assert 0 < need <= sla.sla_static_scratch_bytes(), need
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    ptr = lambda t: None if t is None else t.data_ptr()
    stream = torch.cuda.current_stream(dev).cuda_stream
    res = []
    for static in (False, True):
        out = torch.full((B, T, H, dv), float("nan"), dtype=tdt, device=dev)
        fin = torch.full((B, H, dk, dv), float("nan"), dtype=torch.float32, device=dev)
        args = (params, ptr(g["q"]), ptr(g["k"]), ptr(g["v"]), ptr(g["q_logits"]), ptr(g["k_logits"]),
                ptr(g["log_decay"]), ptr(g["beta"]), ptr(s0), ptr(out), ptr(fin))
        if static:
            rc = sla.sla_forward_static(*args, stream)
        else:
            rc = sla.sla_forward_ws(*args, ptr(ws), need, stream)
        assert rc == 0, sla.sla_status_string(rc)
        torch.cuda.synchronize()
        res.append((out.to(torch.float32).cpu().numpy(), fin.cpu().numpy()))
    return res


def _check(variant, d, dtype, segments, initial_state, label):
    (o_ws, f_ws), (o_st, f_st) = _both(variant, d, dtype, segments, initial_state)
    np.testing.assert_array_equal(o_st, o_ws, err_msg=f"{label}: out differs from sla_forward_ws")
    np.testing.assert_array_equal(f_st, f_ws, err_msg=f"{label}: final state differs from sla_forward_ws")
    ro, rf = run_oracle(variant, d, initial_state)
    eo, ef = rel_err(o_st.astype(np.float64), ro), rel_err(f_st.astype(np.float64), rf)
    print(f"[no-alloc] {label}: out_err={eo:.3e} state_err={ef:.3e}", flush=True)
    assert eo <= TOL[dtype] and ef <= TOL[dtype], (label, eo, ef)


@pytest.mark.parametrize("variant,dtype", [(GLA, "bf16"), (RETNET, "f32")])
def test_static_scratch_matches_workspace_two_calls(variant, dtype):
    import paper_2602_01744_amd as sla

    assert sla.sla_init() == 0
    name = si.VARIANT_NAMES[variant]
    big = si.custom(variant, dtype, B=2, T=1536, H=4, dk=128, dv=128, seed=4100 + variant)
    s0 = si.initial_state(2, 4, 128, 128, seed=41)
    _check(variant, big, dtype, 4, s0, f"{name} {dtype} T=1536, 4 segments")
    small = si.custom(variant, dtype, B=1, T=700, H=2, dk=128, dv=64, seed=4200 + variant)
    _check(variant, small, dtype, 2, None, f"{name} {dtype} T=700, 2 segments (after the larger call)")


def test_static_scratch_one_pass_shapes_and_limit():
    """Shapes that run as one fused pass use no scratch (the delta rule among them); a segment request beyond the
    buffer is refused with SLA_ERR_SCRATCH and writes nothing."""
    import torch

    import paper_2602_01744_amd as sla
    from gpu_util import GDN

    d = si.custom(GDN, "bf16", B=2, T=200, H=4, dk=128, dv=128, seed=4300)
    g, tdt = to_device(d, "bf16", GDN)
    dev = g["q"].device
    out = torch.empty((2, 200, 4, 128), dtype=tdt, device=dev)
    fin = torch.empty((2, 4, 128, 128), dtype=torch.float32, device=dev)
    params = sla.SlaParams(GDN, sla.BF16, 2, 200, 4, 128, 128, 0, 0, 0)
    ptr = lambda t: None if t is None else t.data_ptr()
    rc = sla.sla_forward_static(params, ptr(g["q"]), ptr(g["k"]), ptr(g["v"]), ptr(g["q_logits"]), ptr(g["k_logits"]),
                                ptr(g["log_decay"]), ptr(g["beta"]), None, ptr(out), ptr(fin),
                                torch.cuda.current_stream(dev).cuda_stream)
    assert rc == 0
    torch.cuda.synchronize()
    ro, rf = run_oracle(GDN, d, None)
    assert rel_err(out.to(torch.float32).cpu().numpy().astype(np.float64), ro) <= TOL["bf16"]
    assert rel_err(fin.cpu().numpy().astype(np.float64), rf) <= TOL["bf16"]

    # 32 segments of 256 tokens, 32 heads: 32 * 32 * 128 * 128 floats = 64 MiB of entry states
    B, T, H = 1, 8192, 32
    q = torch.zeros((B, T, H, 128), dtype=torch.bfloat16, device=dev)
    lg = torch.zeros((B, T, H), dtype=torch.float32, device=dev)
    canary = torch.full((B, T, H, 128), 7.0, dtype=torch.bfloat16, device=dev)
    params = sla.SlaParams(GLA, sla.BF16, B, T, H, 128, 128, 0, 0, 32)
    rc = sla.sla_forward_static(params, q.data_ptr(), q.data_ptr(), q.data_ptr(), lg.data_ptr(), lg.data_ptr(),
                                q.data_ptr(), None, None, canary.data_ptr(), None,
                                torch.cuda.current_stream(dev).cuda_stream)
    assert rc == -7, rc
    torch.cuda.synchronize()
    assert bool((canary == 7.0).all())
