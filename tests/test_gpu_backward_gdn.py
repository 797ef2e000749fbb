"""GPU parity of the gated delta rule's backward pass (sla_backward_gdn through the C ABI) against the gradient
oracle on the same seeded inputs and cotangents.  Tolerance: the bf16 bar of the other parity tests,
max|x - x*| / max|x*| <= 2e-2 per gradient tensor.  bf16 tensors take the block form on the matrix cores (bf16
operands, fp32 accumulation; intermediates pass through the workspace in bf16): measured errors 2e-3 to 7e-3 for
every output.  fp32 tensors take the token-recurrent fp32 path, whose fp32 outputs are held to 1e-4."""
import numpy as np
import pytest

import sla_inputs as si
from gpu_util import GDN, TOL, rel_err, to_device
from oracle import sla_backward as ob

pytestmark = pytest.mark.gpu

NAMES = {"dq": "dq", "dk": "dk", "dv": "dv", "dq_head_logits": "dq_logits", "dk_head_logits": "dk_logits",
         "dlog_decay": "dlog_decay", "dbeta": "dbeta", "d_initial_state": "dinitial_state"}
# fp32 tensors: fp32 outputs of fp32 arithmetic, far below the bf16 bar
TIGHT = {"dq_head_logits": 1e-4, "dk_head_logits": 1e-4, "dlog_decay": 1e-4, "dbeta": 1e-4, "d_initial_state": 1e-4}


def run_backward_gdn(d, cot, s0=None, want_ds0=False, dtype="bf16"):
    import torch
    import paper_2602_01744_amd as sla

    g, tdt = to_device(d, dtype, GDN)
    dev = torch.device("cuda:0")
    up = lambda a, dt: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dt).to(dev)
    res = sla.backward_gdn(g["q"], g["k"], g["v"], g["q_logits"], g["k_logits"], g["log_decay"], g["beta"],
                           up(cot["d_out"], tdt), up(s0, torch.float32),
                           up(cot["d_final_state"], torch.float32), want_d_initial_state=want_ds0)
    torch.cuda.synchronize()
    return {n: None if t is None else t.to(torch.float32).cpu().numpy().astype(np.float64) for n, t in res.items()}


def check_backward_gdn(d, cot, s0=None, want_ds0=False, label="", batch_rows=None, dtype="bf16", c_oracle=False):
    """c_oracle: the reference is the C gradient oracle (whole workloads in seconds) instead of the numpy one."""
    import oracle

    got = run_backward_gdn(d, cot, s0, want_ds0, dtype)
    rows = slice(None) if batch_rows is None else batch_rows
    sub = lambda a: None if a is None else a[rows]
    fn = oracle.backward if c_oracle else ob.backward
    ref = fn(GDN, sub(d["q"]), sub(d["k"]), sub(d["v"]), sub(d["q_logits"]), sub(d["k_logits"]),
             sub(d["log_decay"]), sub(cot["d_out"]), sub(s0), sub(cot["d_final_state"]), beta=sub(d["beta"]))
    errs = {}
    for n, rn in NAMES.items():
        x, r = got[n], ref[rn]
        if n == "d_initial_state" and not want_ds0:
            continue
        if r is None:
            assert x is None, n
            continue
        x = x[rows]
        assert np.all(np.isfinite(x)), f"{label}: non-finite {n}"
        errs[n] = rel_err(x, r)
    print(f"[gdn backward parity] {label} " + " ".join(f"{n}={e:.2e}" for n, e in errs.items()), flush=True)
    for n, e in errs.items():
        assert e <= TOL[dtype], f"{label}: {n} error {e:.3e} > {TOL[dtype]}"
        if dtype == "f32" and n in TIGHT:
            assert e <= TIGHT[n], f"{label}: {n} error {e:.3e} > {TIGHT[n]} (fp32 output)"
    return got, ref


def make(B, T, H, dk, dv, seed, states=False, k_logits=True):
    d = si.custom(GDN, "bf16", B=B, T=T, H=H, dk=dk, dv=dv, seed=seed)
    if not k_logits:
        d["k_logits"] = None
    cot = si.cotangents(B, T, H, dk, dv, seed=seed + 1, final_state=states)
    s0 = si.initial_state(B, H, dk, dv, seed=seed + 2) if states else None
    return d, cot, s0


def test_small_block_aligned():
    d, cot, s0 = make(2, 64, 4, 64, 64, seed=1100)
    check_backward_gdn(d, cot, label="B2 T64 H4 d64")


@pytest.mark.parametrize("states", [False, True])
def test_ragged_multi_chunk(states):
    d, cot, s0 = make(2, 203, 3, 128, 128, seed=1110, states=states)
    check_backward_gdn(d, cot, s0=s0, want_ds0=states, label=f"B2 T203 H3 d128 states={states}")


@pytest.mark.parametrize("dk,dv", [(64, 64), (64, 128), (128, 64), (128, 256), (64, 256)])
def test_head_widths(dk, dv):
    d, cot, s0 = make(1, 77, 2, dk, dv, seed=1120 + dk + dv, states=True)
    check_backward_gdn(d, cot, s0=s0, want_ds0=True, label=f"dk={dk} dv={dv}")


@pytest.mark.parametrize("dk,dv,T", [(128, 256, 1100), (64, 64, 1300), (64, 128, 520), (128, 64, 1024 + 31)])
def test_head_widths_across_anchors(dk, dv, T):
    """Every width pair over sequences long enough for the loaders' register sets to go round several times, for the
    three-stage and the two-half step (value heads of width 256 take the latter) and for one or two anchors of the
    decay gradient; two batch rows, so a row's anchors sit next to another row's in the workspace."""
    d, cot, s0 = make(2, T, 2, dk, dv, seed=1125 + dk + dv, states=True)
    check_backward_gdn(d, cot, s0=s0, want_ds0=True, label=f"dk={dk} dv={dv} T={T}")


@pytest.mark.parametrize("T", [1, 2, 15, 16, 17, 33])
def test_short_sequences(T):
    d, cot, s0 = make(2, T, 2, 64, 64, seed=1130 + T, states=True)
    check_backward_gdn(d, cot, s0=s0, want_ds0=True, label=f"T={T}")


@pytest.mark.parametrize("H", [1, 7, 64])
def test_head_counts(H):
    d, cot, s0 = make(1, 40, H, 64, 64, seed=1140 + H)
    check_backward_gdn(d, cot, label=f"H={H}")


def test_read_gate_only():
    d, cot, s0 = make(2, 50, 4, 64, 128, seed=1150, k_logits=False)
    got, _ = check_backward_gdn(d, cot, label="no k logits")
    assert got["dk_head_logits"] is None


def test_beta_zero_tokens_write_nothing():
    # beta = 0: the token neither erases nor writes, so dk and dv vanish there (exactly) while dbeta does not
    d, cot, s0 = make(1, 48, 2, 64, 64, seed=1160)
    d["beta"][:, ::3] = 0.0
    got, ref = check_backward_gdn(d, cot, label="beta = 0 on every third token")
    assert np.all(got["dv"][:, ::3] == 0.0)
    assert np.max(np.abs(ref["dbeta"][:, ::3])) > 0.0


def test_strong_decay_domain():
    # log-decay down to -5 per token (and a few at -20): the sweeps keep their tiles divided by a running decay
    # product over 4 tokens, which must stay inside fp32's range
    B, T, H = 1, 100, 2
    d, cot, s0 = make(B, T, H, 64, 128, seed=1165, states=True)
    r = np.random.default_rng(1166)
    d["log_decay"] = (-5.0 * r.random(size=d["log_decay"].shape)).astype(np.float32)
    d["log_decay"][:, 40:48] = -20.0
    check_backward_gdn(d, cot, s0=s0, want_ds0=True, label="decay in [-5, 0], eight tokens at -20")


@pytest.mark.parametrize("dk,dv,T", [(128, 128, 203), (64, 256, 77), (128, 64, 16)])
def test_fp32_tensors(dk, dv, T):
    """fp32 q, k, v, d_out and gradients: every output to the fp32 bar (1e-4)."""
    B, H = 2, 3
    d = si.custom(GDN, "f32", B=B, T=T, H=H, dk=dk, dv=dv, seed=1180 + T)
    cot = si.cotangents(B, T, H, dk, dv, seed=1181 + T, dtype="f32", final_state=True)
    s0 = si.initial_state(B, H, dk, dv, seed=1182 + T)
    check_backward_gdn(d, cot, s0=s0, want_ds0=True, label=f"fp32 dk={dk} dv={dv} T={T}", dtype="f32")


@pytest.mark.parametrize("T", [4096 + 24, 8192 + 40])
def test_long_sequence(T):
    """dlog_decay is a suffix sum of per-token scalars made of bf16-operand products; the block form re-derives it
    exactly (as <X, S>) every 512 tokens, so its error does not grow with the length: held to half the bar here, on
    the earliest tokens (the longest sums) too."""
    d, cot, s0 = make(1, T, 2, 128, 128, seed=1170, states=True)
    got, ref = check_backward_gdn(d, cot, s0=s0, want_ds0=True, label=f"T={T}")
    scale = np.abs(ref["dlog_decay"]).max()
    assert np.abs(got["dlog_decay"] - ref["dlog_decay"]).max() / scale <= 0.5 * TOL["bf16"]
    assert np.abs(got["dlog_decay"][:, :512] - ref["dlog_decay"][:, :512]).max() / scale <= 0.5 * TOL["bf16"]


def test_full_size():
    """The bench workload (gdn: B=8, T=4096, H=16, d=128), as bench.py launches it; every batch row against the C
    gradient oracle."""
    w = si.workload("gdn")
    d = si.generate(w)
    cot = si.cotangents(w.B, w.T, w.H, w.dk, w.dv, seed=w.seed + 50)
    got, _ = check_backward_gdn(d, cot, label="gdn", c_oracle=True)
    for n, x in got.items():  # every batch row: finite, and logit gradients summing to zero over the heads
        assert x is None or np.all(np.isfinite(x)), n
    for n in ("dq_head_logits", "dk_head_logits"):
        assert np.max(np.abs(got[n].sum(axis=-1))) <= 1e-5 * np.max(np.abs(got[n])) * w.H, n
