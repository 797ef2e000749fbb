"""GPU parity of the backward pass (sla_backward through the C ABI) against the gradient oracle on the same
seeded inputs and cotangents.  Tolerance: the forward's bf16 bar, max|x - x*| / max|x*| <= 2e-2 per gradient
tensor (operands are rounded to bf16 on the way to the matrix cores, accumulation is fp32, and every gradient
is itself returned in bf16 except the logit and state gradients)."""
import numpy as np
import pytest

import sla_inputs as si
import oracle
from gpu_util import GLA, RETNET, TOL, rel_err, to_device, worst_slice_err
from oracle import sla_backward as ob

pytestmark = pytest.mark.gpu

NAMES = {"dq": "dq", "dk": "dk", "dv": "dv", "dq_head_logits": "dq_logits", "dk_head_logits": "dk_logits",
         "dlog_decay": "dlog_decay", "d_initial_state": "dinitial_state"}


def run_backward(variant, d, cot, s0=None, want_ds0=False, segments=1, dtype="bf16"):
    import torch
    import paper_2602_01744_amd as sla

    g, tdt = to_device(d, dtype, variant)
    dev = torch.device("cuda:0")
    up = lambda a, dt: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dt).to(dev)
    res = sla.backward(variant, g["q"], g["k"], g["v"], g["q_logits"], g["k_logits"], g["log_decay"],
                       up(cot["d_out"], tdt), up(s0, torch.float32), up(cot["d_final_state"], torch.float32),
                       want_d_initial_state=want_ds0, segments=segments)
    torch.cuda.synchronize()
    return {n: None if t is None else t.to(torch.float32).cpu().numpy().astype(np.float64) for n, t in res.items()}


# Worst (batch, head) slice, each on its own scale, at the same bar.  The quantities that are small by cancellation
# where a head's own values are (logit gradients; the GLA decay gradient, a difference of two running sums) are held
# to the bar on the scale of their batch row instead.
SLICE_TOL = {}


def check_backward(variant, d, cot, s0=None, want_ds0=False, label="", batch_rows=None, segments=1, c_oracle=False,
                   dtype="bf16"):
    """c_oracle: the reference is the C gradient oracle (whole workloads in seconds) instead of the numpy one.
    dtype: the tensors' element type; the bar is TOL[dtype]."""
    got = run_backward(variant, d, cot, s0, want_ds0, segments, dtype)
    rows = slice(None) if batch_rows is None else batch_rows
    sub = lambda a: None if a is None else (a if a.ndim == 1 else a[rows])
    fn = oracle.backward if c_oracle else ob.backward
    ref = fn(variant, sub(d["q"]), sub(d["k"]), sub(d["v"]), sub(d["q_logits"]), sub(d["k_logits"]),
             sub(d["log_decay"]), sub(cot["d_out"]), sub(s0), sub(cot["d_final_state"]))
    errs, slices = {}, {}
    for n, rn in NAMES.items():
        x, r = got[n], ref[rn]
        if n == "dlog_decay" and variant == RETNET:
            assert x is None
            continue
        if n == "d_initial_state" and not want_ds0:
            continue
        if r is None:
            assert x is None, n
            continue
        x = x[rows]
        assert np.all(np.isfinite(x)), f"{label}: non-finite {n}"
        errs[n] = rel_err(x, r)
        if n.endswith("_head_logits") or n == "dlog_decay":
            # a head's logit gradient is G (dG - sum_h G dG), small by cancellation where the gate is: held to the
            # tolerance on the scale of its batch row, not on its own
            slices[n] = max(rel_err(x[i], r[i]) for i in range(r.shape[0]))
        else:
            slices[n] = worst_slice_err(x, r, 1 if n == "d_initial_state" else 2)
    print(f"[backward parity] {label} " + " ".join(f"{n}={e:.2e}/{slices[n]:.2e}" for n, e in errs.items()), flush=True)
    for n, e in errs.items():
        assert e <= TOL[dtype], f"{label}: {n} error {e:.3e} > {TOL[dtype]}"
        bar = SLICE_TOL.get(n, TOL[dtype])
        assert slices[n] <= bar, f"{label}: {n} error of the worst (batch, head) slice {slices[n]:.3e} > {bar}"
    return got, ref


@pytest.mark.parametrize("variant", [RETNET, GLA])
def test_small_block_aligned(variant):
    d = si.custom(variant, "bf16", B=1, T=32, H=2, dk=64, dv=64, seed=900 + variant)
    cot = si.cotangents(1, 32, 2, 64, 64, seed=901)
    check_backward(variant, d, cot, label=f"{si.VARIANT_NAMES[variant]} T=32 d=64")


@pytest.mark.parametrize("variant", [RETNET, GLA])
@pytest.mark.parametrize("states", [False, True])
def test_ragged_multi_tile(variant, states):
    B, T, H, dk, dv = 2, 203, 5, 128, 128
    d = si.custom(variant, "bf16", B=B, T=T, H=H, dk=dk, dv=dv, seed=910 + variant)
    cot = si.cotangents(B, T, H, dk, dv, seed=911, final_state=states)
    s0 = si.initial_state(B, H, dk, dv, seed=9) if states else None
    check_backward(variant, d, cot, s0, want_ds0=states, label=f"{si.VARIANT_NAMES[variant]} T=203 H=5 states={states}")


@pytest.mark.parametrize("variant", [RETNET, GLA])
@pytest.mark.parametrize("dk,dv", [(64, 64), (64, 128), (128, 64), (128, 256), (64, 256)])
def test_head_widths(variant, dk, dv):
    d = si.custom(variant, "bf16", B=1, T=130, H=3, dk=dk, dv=dv, seed=920 + dk + dv)
    cot = si.cotangents(1, 130, 3, dk, dv, seed=921, final_state=True)
    s0 = si.initial_state(1, 3, dk, dv, seed=10)
    check_backward(variant, d, cot, s0, want_ds0=True, label=f"{si.VARIANT_NAMES[variant]} dk={dk} dv={dv}")


@pytest.mark.parametrize("variant", [RETNET, GLA])
@pytest.mark.parametrize("T", [1, 2, 15, 16, 17, 63, 65])
def test_short_sequences(variant, T):
    d = si.custom(variant, "bf16", B=2, T=T, H=4, dk=128, dv=64, seed=930 + T)
    cot = si.cotangents(2, T, 4, 128, 64, seed=931 + T, final_state=True)
    check_backward(variant, d, cot, None, want_ds0=True, label=f"{si.VARIANT_NAMES[variant]} T={T}")


@pytest.mark.parametrize("variant", [RETNET, GLA])
@pytest.mark.parametrize("H", [1, 7, 64])
def test_head_counts(variant, H):
    d = si.custom(variant, "bf16", B=1, T=70, H=H, dk=64, dv=64, seed=940 + H)
    cot = si.cotangents(1, 70, H, 64, 64, seed=941)
    check_backward(variant, d, cot, label=f"{si.VARIANT_NAMES[variant]} H={H}")


@pytest.mark.parametrize("variant", [RETNET, GLA])
def test_read_gate_only(variant):
    d = si.custom(variant, "bf16", B=1, T=90, H=4, dk=64, dv=128, seed=950)
    d["k_logits"] = None
    cot = si.cotangents(1, 90, 4, 64, 128, seed=951)
    got, _ = check_backward(variant, d, cot, label=f"{si.VARIANT_NAMES[variant]} read gate only")
    assert got["dk_head_logits"] is None


def test_saturated_gates_give_exact_zero_gradients():
    # one-hot gates (Sec. 4.2's saturated limit): heads that are never selected get exactly zero dq, dk, dv
    B, T, H = 1, 48, 4
    d = si.custom(GLA, "bf16", B=B, T=T, H=H, dk=64, dv=64, seed=960)
    d["q_logits"][:] = 0.0
    d["q_logits"][..., 1] = 1.0e4
    d["k_logits"][:] = 0.0
    d["k_logits"][..., 1] = 1.0e4
    cot = si.cotangents(B, T, H, 64, 64, seed=961)
    got, ref = check_backward(GLA, d, cot, label="saturated gates")
    for h in (0, 2, 3):
        assert np.all(got["dq"][:, :, h] == 0.0) and np.all(got["dk"][:, :, h] == 0.0)
        assert np.all(got["dv"][:, :, h] == 0.0)


def test_strong_decay_domain():
    # log-decay down to -5 per step: the block-local factors span e^{+-80}
    B, T, H = 1, 100, 2
    d = si.custom(GLA, "bf16", B=B, T=T, H=H, dk=64, dv=64, seed=970)
    r = np.random.default_rng(971)
    d["log_decay"] = si.round_to_bf16((-5.0 * r.random(size=d["log_decay"].shape)).astype(np.float32))
    cot = si.cotangents(B, T, H, 64, 64, seed=972)
    check_backward(GLA, d, cot, label="decay in [-5, 0]")


@pytest.mark.parametrize("T,dv,states", [(4096, 128, False), (8192 + 40, 128, True), (2048 + 512, 256, True)])
def test_long_sequences_keep_the_decay_gradient_accurate(T, dv, states):
    """dlog_decay at token t sums q dq - k dk over every later token, two sums that nearly cancel: without the
    exact re-anchoring every 512 tokens its error grows with the sequence length and passes the bar near 4k tokens."""
    B, H, dk = 1, 2, 128
    d = si.custom(GLA, "bf16", B=B, T=T, H=H, dk=dk, dv=dv, seed=77)
    cot = si.cotangents(B, T, H, dk, dv, seed=78, final_state=states)
    s0 = si.initial_state(B, H, dk, dv, seed=79) if states else None
    got, ref = check_backward(GLA, d, cot, s0=s0, want_ds0=states, label=f"long T={T} dv={dv}")
    # the error of the earliest tokens (the longest sums) is no worse than the bar either
    scale = np.abs(ref["dlog_decay"]).max()
    early = np.abs(got["dlog_decay"][:, :512] - ref["dlog_decay"][:, :512]).max() / scale
    assert early <= TOL["bf16"]


@pytest.mark.parametrize("variant", [RETNET, GLA])
@pytest.mark.parametrize("T,segments,states", [(700, 2, True), (1000, 3, False), (2048 + 37, 4, True), (512, 2, True)])
def test_segment_schedule(variant, T, segments, states):
    """Batch rows cut into segments that run as packed sequences: entry states from the forward's pre-pass, end
    cotangents from a dv-sweep pre-pass and a combine kernel.  Same answers as the single pass, to the same bar."""
    B, H, dk, dv = 2, 2, 128, 128
    d = si.custom(variant, "bf16", B=B, T=T, H=H, dk=dk, dv=dv, seed=990 + T + variant)
    cot = si.cotangents(B, T, H, dk, dv, seed=991 + T, final_state=states)
    s0 = si.initial_state(B, H, dk, dv, seed=992 + T) if states else None
    check_backward(variant, d, cot, s0=s0, want_ds0=True, label=f"T={T} in {segments} segments", segments=segments)


def test_segment_count_chosen_for_the_device():
    """segments = 0 in the binding asks sla_backward_segments: few sequences, so the rows are cut."""
    import torch
    import paper_2602_01744_amd as sla

    B, T, H, dk, dv = 1, 1500, 2, 64, 128
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert sla.sla_backward_segments(sla.SlaParams(GLA, sla.BF16, B, T, H, dk, dv, 0, 0, 1), cus) > 1
    d = si.custom(GLA, "bf16", B=B, T=T, H=H, dk=dk, dv=dv, seed=995)
    cot = si.cotangents(B, T, H, dk, dv, seed=996, final_state=True)
    check_backward(GLA, d, cot, s0=si.initial_state(B, H, dk, dv, seed=997), want_ds0=True,
                   label="segments chosen by the library", segments=0)


def test_segment_schedule_on_the_paper_shape():
    """gla_paper_h4 (B=8, T=4096, H=4, dk=128, dv=256: 32 sequences) in 4 segments; every batch row is compared."""
    w = si.workload("gla_paper_h4")
    d = si.generate(w)
    cot = si.cotangents(w.B, w.T, w.H, w.dk, w.dv, seed=w.seed + 50)
    check_backward(w.variant, d, cot, label="gla_paper_h4, 4 segments", segments=4, c_oracle=True)


@pytest.mark.parametrize("name", ["gla_train", "retnet_train"])
def test_full_size(name):
    """The bench workload, in the launch configuration bench.py times; every batch row against the C gradient oracle."""
    w = si.workload(name)
    d = si.generate(w)
    cot = si.cotangents(w.B, w.T, w.H, w.dk, w.dv, seed=w.seed + 50)
    got, _ = check_backward(w.variant, d, cot, label=name, c_oracle=True)
    # properties that hold for every batch row, whatever the size: all values finite, and the logit gradients of a
    # token sum to zero over the heads (Eq. 4's softmax)
    for n, x in got.items():
        assert x is None or np.all(np.isfinite(x)), n
    for n in ("dq_head_logits", "dk_head_logits"):
        scale = np.max(np.abs(got[n]))
        assert np.max(np.abs(got[n].sum(axis=-1))) <= 1e-5 * scale * w.H, n
