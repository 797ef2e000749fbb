"""Helpers shared by the GPU parity tests: move seeded numpy inputs to the device, call the C ABI
through the binding, run the CPU oracle on the same arrays and compare."""
from __future__ import annotations

import numpy as np

import oracle
import sla_inputs as si

RETNET, GLA, GDN = 0, 1, 2

# Tolerances of the parity gate (max |x - x*| / max |x*| per output tensor).
# fp32: operands stay fp32 through the matrix cores, differences are summation order and the
#       hardware exp2/rcp (1 ulp): 1e-4 leaves two orders of margin.
# bf16: operands are rounded to bf16 (2^-9 relative) three times on the way (decay-folded q/k, the
#       masked scores, the state used for the read-out); accumulation and the state are fp32.
TOL = {"f32": 1e-4, "bf16": 2e-2}


to_device = si.to_device  # numpy inputs -> device tensors (marshalling only)


def run_gpu(variant, d, dtype, initial_state=None, dv_split=0, want_final_state=True, segments=1):
    import torch
    import paper_2602_01744_amd as sla

    g, _ = to_device(d, dtype, variant)
    s0 = None if initial_state is None else torch.from_numpy(np.ascontiguousarray(initial_state, dtype=np.float32)).to("cuda:0")
    out, fin = sla.forward(variant, g["q"], g["k"], g["v"], g["q_logits"], g["k_logits"], g["log_decay"], g["beta"],
                           s0, dv_split=dv_split, want_final_state=want_final_state, segments=segments)
    torch.cuda.synchronize()
    o = out.to(torch.float32).cpu().numpy().astype(np.float64)
    f = None if fin is None else fin.cpu().numpy().astype(np.float64)
    return o, f


def run_oracle(variant, d, initial_state=None):
    return oracle.forward(variant, d["q"], d["k"], d["v"], d["q_logits"], d["k_logits"], d["log_decay"], d["beta"],
                          initial_state)


def rel_err(x, ref):
    denom = float(np.max(np.abs(ref)))
    if denom == 0.0:
        return float(np.max(np.abs(x)))
    return float(np.max(np.abs(x - ref))) / denom


def worst_slice_err(x, ref, head_axis):
    """Largest max-abs-error / max-abs-reference over (batch, head) slices: every head is held to the tolerance on
    its own scale, so a head with small outputs (a low gate) cannot hide behind a loud one."""
    axes = tuple(i for i in range(ref.ndim) if i not in (0, head_axis))
    num = np.max(np.abs(x - ref), axis=axes)
    den = np.max(np.abs(ref), axis=axes)
    with np.errstate(divide="ignore", invalid="ignore"):
        r = np.where(den > 0, num / den, 0.0)
    return float(np.max(r))


def check(variant, d, dtype, initial_state=None, dv_split=0, tol=None, label="", segments=1):
    tol = TOL[dtype] if tol is None else tol
    o, f = run_gpu(variant, d, dtype, initial_state, dv_split, segments=segments)
    ro, rf = run_oracle(variant, d, initial_state)
    assert np.all(np.isfinite(o)), f"{label}: non-finite output"
    assert np.all(np.isfinite(f)), f"{label}: non-finite state"
    eo, ef = rel_err(o, ro), rel_err(f, rf)
    so, sf = worst_slice_err(o, ro, 2), worst_slice_err(f, rf, 1)
    print(f"[parity] {label} dtype={dtype} dv_split={dv_split} segments={segments} out_err={eo:.3e} state_err={ef:.3e} "
          f"worst_head_out={so:.3e} worst_head_state={sf:.3e}", flush=True)
    assert eo <= tol, f"{label}: output error {eo:.3e} > {tol}"
    assert ef <= tol, f"{label}: state error {ef:.3e} > {tol}"
    assert so <= tol, f"{label}: output error of the worst (batch, head) slice {so:.3e} > {tol}"
    assert sf <= tol, f"{label}: state error of the worst (batch, head) slice {sf:.3e} > {tol}"
    return o, f, ro, rf
