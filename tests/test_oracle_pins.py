"""Pins for the CPU oracle: everything here runs without a GPU.

Each test checks the C oracle (``oracle.forward``) against something other than
itself: a hand-worked example, the quadratic form of Appendix A, closed forms,
textbook matmuls, invariants of the gates (Eq. 4, Thm 4.2, Thm 4.3) and
properties of the delta rule.
"""
import json
import math
import os

import numpy as np
import pytest

import oracle
from oracle import sla_numpy as ref
import sla_inputs as si

RETNET, GLA, GDN = 0, 1, 2
HERE = os.path.dirname(os.path.abspath(__file__))


def _rand(seed, variant, B=2, T=9, H=3, dk=4, dv=5, dual=True, strong=False):
    rng = np.random.default_rng(seed)
    f = lambda *s: rng.standard_normal(s).astype(np.float32)
    d = dict(q=f(B, T, H, dk), k=f(B, T, H, dk), v=f(B, T, H, dv), q_logits=f(B, T, H))
    d["k_logits"] = f(B, T, H) if dual else None
    scale = 2.0 if strong else 0.3
    if variant == RETNET:
        d["log_decay"] = (-np.abs(f(H)) * scale).astype(np.float32)
    elif variant == GLA:
        d["log_decay"] = (-np.abs(f(B, T, H, dk)) * scale).astype(np.float32)
    else:
        d["log_decay"] = (-np.abs(f(B, T, H)) * scale).astype(np.float32)
        d["k"] /= np.linalg.norm(d["k"], axis=-1, keepdims=True)
    d["beta"] = (1 / (1 + np.exp(-f(B, T, H)))).astype(np.float32) if variant == GDN else None
    return d


def _head_decay(variant, ld, h):
    """The log-decay of head h alone, in the layout of its variant."""
    return ld[h:h + 1] if variant == RETNET else ld[:, :, h:h + 1]


def _run(variant, d, initial_state=None):
    return oracle.forward(variant, d["q"], d["k"], d["v"], d["q_logits"], d["k_logits"], d["log_decay"],
                          d["beta"], initial_state)


# ---------------------------------------------------------------- hand-worked example
def test_hand_worked_example():
    """Sec. 5.1 updates + Eq. 4-6 on a 2-token, 2-head, 1x1-state case worked by hand."""
    g = json.load(open(os.path.join(HERE, "golden", "worked_example.json")))
    T, H = 2, 2
    q = np.array(g["q"], np.float32).reshape(1, T, 1, 1).repeat(H, 2)
    k = np.array(g["k"], np.float32).reshape(1, T, 1, 1).repeat(H, 2)
    v = np.array(g["v"], np.float32).reshape(1, T, 1, 1).repeat(H, 2)
    ql = np.tile(np.array([math.log(3.0), 0.0], np.float32), (1, T, 1))
    kl = np.tile(np.array([0.0, math.log(4.0)], np.float32), (1, T, 1))
    lg = math.log(g["decay_factor"])
    want = np.array(g["gla_retnet"]["out"]).reshape(1, T, H, 1)
    wantS = np.array(g["gla_retnet"]["final_state"]).reshape(1, H, 1, 1)
    out, S = oracle.forward(GLA, q, k, v, ql, kl, np.full((1, T, H, 1), lg, np.float32))
    np.testing.assert_allclose(out, want, rtol=1e-6)
    np.testing.assert_allclose(S, wantS, rtol=1e-6)
    out, S = oracle.forward(RETNET, q, k, v, ql, kl, np.full((H,), lg, np.float32))
    np.testing.assert_allclose(out, want, rtol=1e-6)
    np.testing.assert_allclose(S, wantS, rtol=1e-6)
    out, S = oracle.forward(GDN, q, k, v, ql, kl, np.full((1, T, H), lg, np.float32),
                            np.full((1, T, H), g["beta"], np.float32))
    np.testing.assert_allclose(out, np.array(g["gdn"]["out"]).reshape(1, T, H, 1), rtol=1e-6)
    np.testing.assert_allclose(S, np.array(g["gdn"]["final_state"]).reshape(1, H, 1, 1), rtol=1e-6)


# ---------------------------------------------------------------- brute force: Appendix A
@pytest.mark.parametrize("variant", [RETNET, GLA])
@pytest.mark.parametrize("dual", [True, False])
@pytest.mark.parametrize("strong", [False, True])
def test_recurrence_equals_quadratic_form(variant, dual, strong):
    d = _rand(11 + variant, variant, dual=dual, strong=strong)
    out, _ = _run(variant, d)
    want = ref.quadratic(variant, d["q"], d["k"], d["v"], d["q_logits"], d["k_logits"], d["log_decay"])
    np.testing.assert_allclose(out, want, rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("variant", [RETNET, GLA, GDN])
def test_c_oracle_equals_numpy_recurrence(variant):
    d = _rand(23 + variant, variant, B=2, T=33, H=4, dk=6, dv=3)
    s0 = si.initial_state(2, 4, 6, 3, seed=5)
    out, S = _run(variant, d, s0)
    o2, S2 = ref.recurrent(variant, d["q"], d["k"], d["v"], d["q_logits"], d["k_logits"], d["log_decay"],
                           d["beta"], s0)
    np.testing.assert_allclose(out, o2, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(S, S2, rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("chunk", [1, 2, 7, 16, 64])
def test_gdn_recurrence_equals_chunked_solve(chunk):
    d = _rand(31, GDN, B=1, T=40, H=2, dk=8, dv=5)
    s0 = si.initial_state(1, 2, 8, 5, seed=9)
    out, S = _run(GDN, d, s0)
    o2, S2 = ref.gdn_chunked(d["q"], d["k"], d["v"], d["q_logits"], d["k_logits"], d["log_decay"], d["beta"],
                             chunk, s0)
    np.testing.assert_allclose(out, o2, rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(S, S2, rtol=1e-10, atol=1e-11)


# ---------------------------------------------------------------- textbook special cases
def test_single_head_no_decay_is_causal_linear_attention():
    """H=1 makes the gate 1 (Eq. 4); without decay Eq. 2 is tril(QK^T)V and S = K^T V."""
    rng = np.random.default_rng(3)
    T, dk, dv = 12, 5, 7
    q, k, v = (rng.standard_normal((1, T, 1, n)).astype(np.float32) for n in (dk, dk, dv))
    lg = rng.standard_normal((1, T, 1)).astype(np.float32)
    Q, K, V = q[0, :, 0].astype(np.float64), k[0, :, 0].astype(np.float64), v[0, :, 0].astype(np.float64)
    for variant, ld in ((RETNET, np.zeros(1, np.float32)), (GLA, np.zeros((1, T, 1, dk), np.float32))):
        out, S = oracle.forward(variant, q, k, v, lg, lg, ld)
        np.testing.assert_allclose(out[0, :, 0], np.tril(Q @ K.T) @ V, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(S[0, 0], K.T @ V, rtol=1e-12, atol=1e-13)


def test_single_head_scalar_decay_matrix_and_geometric_closed_form():
    rng = np.random.default_rng(4)
    T, dk, dv = 10, 3, 4
    gamma = 0.8
    q, k, v = (rng.standard_normal((1, T, 1, n)).astype(np.float32) for n in (dk, dk, dv))
    lg = np.zeros((1, T, 1), np.float32)
    ld = np.array([math.log(gamma)], np.float32)
    g32 = math.exp(float(ld[0]))
    out, _ = oracle.forward(RETNET, q, k, v, lg, None, ld)
    Q, K, V = q[0, :, 0].astype(np.float64), k[0, :, 0].astype(np.float64), v[0, :, 0].astype(np.float64)
    idx = np.arange(T)
    Gam = np.where(idx[:, None] >= idx[None, :], g32 ** (idx[:, None] - idx[None, :]), 0.0)
    np.testing.assert_allclose(out[0, :, 0], ((Q @ K.T) * Gam) @ V, rtol=1e-12, atol=1e-13)
    # constant q,k,v: out_t = (q.k) v (1 - gamma^(t+1)) / (1 - gamma)
    qc = np.tile(q[:, :1], (1, T, 1, 1)); kc = np.tile(k[:, :1], (1, T, 1, 1)); vc = np.tile(v[:, :1], (1, T, 1, 1))
    out, _ = oracle.forward(RETNET, qc, kc, vc, lg, None, ld)
    qk = float(Q[0] @ K[0])
    want = qk * V[0][None, :] * ((1 - g32 ** (idx + 1)) / (1 - g32))[:, None]
    np.testing.assert_allclose(out[0, :, 0], want, rtol=1e-12)


def test_retnet_is_gla_with_broadcast_decay():
    d = _rand(41, RETNET, B=2, T=17, H=3, dk=4, dv=6)
    out, S = _run(RETNET, d)
    ld = np.broadcast_to(d["log_decay"][None, None, :, None], (2, 17, 3, 4)).copy()
    o2, S2 = oracle.forward(GLA, d["q"], d["k"], d["v"], d["q_logits"], d["k_logits"], ld)
    np.testing.assert_allclose(out, o2, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(S, S2, rtol=1e-12, atol=1e-13)


# ---------------------------------------------------------------- gate invariants
def test_gates_are_a_distribution_over_heads():
    rng = np.random.default_rng(6)
    x = (rng.standard_normal((3, 5, 16)) * 4).astype(np.float32)
    g = ref.head_softmax(x)
    assert np.all(g >= 0)
    np.testing.assert_allclose(g.sum(-1), 1.0, rtol=0, atol=1e-15)
    # read the gate back out of the C oracle: with dk=dv=1, q=k=v=1, no decay and no write gate, T=1,
    # the output of head h is exactly G^Q[h].
    B, T, H = 3, 1, 16
    one = np.ones((B, T, H, 1), np.float32)
    out, _ = oracle.forward(GLA, one, one, one, x[:, :1], None, np.zeros((B, T, H, 1), np.float32))
    np.testing.assert_allclose(out[..., 0], g[:, :1], rtol=1e-14)
    assert np.all(out >= 0)
    np.testing.assert_allclose(out.sum(axis=2), 1.0, atol=1e-15)


def test_gate_entropy_decreases_with_scale_and_saturates_to_one_hot():
    """Thm 4.2."""
    rng = np.random.default_rng(7)
    s = rng.standard_normal(8)
    ent = []
    for lam in (0.25, 0.5, 1, 2, 4, 8, 16):
        g = ref.head_softmax((lam * s)[None, None, :])[0, 0]
        ent.append(-np.sum(g * np.log(g + 1e-300)))
    assert all(a > b for a, b in zip(ent, ent[1:]))
    g = ref.head_softmax((1e4 * s)[None, None, :])[0, 0]
    want = np.zeros(8); want[np.argmax(s)] = 1.0
    np.testing.assert_array_equal(g, want)


@pytest.mark.parametrize("variant", [RETNET, GLA, GDN])
def test_uniform_logits_scale_output_and_state(variant):
    """All gates equal 1/H (Eq. 4 with equal scores): dual gating scales the output by 1/H^2 and the
    state by 1/H; read-only gating scales the output by 1/H and leaves the state alone."""
    H = 4
    d = _rand(51 + variant, variant, B=1, T=14, H=H, dk=4, dv=3)
    base_out, base_S = [], []
    for h in range(H):  # each head alone: H=1, gate 1
        ld = _head_decay(variant, d["log_decay"], h)
        bt = None if d["beta"] is None else d["beta"][:, :, h:h + 1]
        o, S = oracle.forward(variant, d["q"][:, :, h:h + 1], d["k"][:, :, h:h + 1], d["v"][:, :, h:h + 1],
                              np.zeros((1, 14, 1), np.float32), None, ld, bt)
        base_out.append(o); base_S.append(S)
    base_out = np.concatenate(base_out, axis=2); base_S = np.concatenate(base_S, axis=1)
    const = np.full((1, 14, H), 0.7, np.float32)
    o, S = oracle.forward(variant, d["q"], d["k"], d["v"], const, const, d["log_decay"], d["beta"])
    np.testing.assert_allclose(o, base_out / H**2, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(S, base_S / H, rtol=1e-12, atol=1e-14)
    o, S = oracle.forward(variant, d["q"], d["k"], d["v"], const, None, d["log_decay"], d["beta"])
    np.testing.assert_allclose(o, base_out / H, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(S, base_S, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("variant", [RETNET, GLA, GDN])
def test_saturated_logits_select_one_head_exactly(variant):
    H, T, sel = 4, 11, 2
    d = _rand(61 + variant, variant, B=1, T=T, H=H, dk=4, dv=3)
    sat = np.zeros((1, T, H), np.float32); sat[..., sel] = 1e4
    o, S = oracle.forward(variant, d["q"], d["k"], d["v"], sat, sat, d["log_decay"], d["beta"])
    ld = _head_decay(variant, d["log_decay"], sel)
    bt = None if d["beta"] is None else d["beta"][:, :, sel:sel + 1]
    ob, Sb = oracle.forward(variant, d["q"][:, :, sel:sel + 1], d["k"][:, :, sel:sel + 1], d["v"][:, :, sel:sel + 1],
                            np.zeros((1, T, 1), np.float32), None, ld, bt)
    np.testing.assert_array_equal(o[:, :, sel], ob[:, :, 0])
    np.testing.assert_array_equal(S[:, sel], Sb[:, 0])
    others = [h for h in range(H) if h != sel]
    assert np.all(o[:, :, others] == 0.0)
    if variant != GDN:
        assert np.all(S[:, others] == 0.0)


def test_winner_take_all_needs_consensus():
    """Thm 4.3: a token written under winner h_K is visible to a query with winner h_Q only if they agree."""
    H, T = 4, 6
    d = _rand(71, GLA, B=1, T=T, H=H, dk=4, dv=3)
    write = np.zeros((1, T, H), np.float32); write[..., 1] = 1e4
    read_same = write.copy()
    read_other = np.zeros((1, T, H), np.float32); read_other[..., 3] = 1e4
    o_same, _ = oracle.forward(GLA, d["q"], d["k"], d["v"], read_same, write, d["log_decay"])
    o_diff, _ = oracle.forward(GLA, d["q"], d["k"], d["v"], read_other, write, d["log_decay"])
    assert np.abs(o_same[:, :, 1]).max() > 1e-3
    assert np.all(o_diff == 0.0)
    # flow coefficient C = sum_h G^Q_h G^K_h tends to the Kronecker delta
    sq, sk = np.array([0.3, 1.0, -0.2, 0.1]), np.array([0.0, 0.9, 0.2, -1.0])
    C = lambda a, b, lam: float(np.sum(ref.head_softmax(lam * a[None, None])[0, 0] * ref.head_softmax(lam * b[None, None])[0, 0]))
    assert abs(C(sq, sk, 200.0) - 1.0) < 1e-12
    assert C(sq, np.roll(sk, 1), 200.0) < 1e-12


@pytest.mark.parametrize("variant", [RETNET, GLA, GDN])
def test_gates_can_be_absorbed_into_the_inputs(variant):
    """Appendix A: SLA on (q,k,v) equals the ungated recurrence on gated feature maps.  For the delta rule
    the write gate sits on v (Sec. 5.1), so it is absorbed there."""
    H, T = 3, 13
    d = _rand(81 + variant, variant, B=2, T=T, H=H, dk=4, dv=5)
    o, S = _run(variant, d)
    gq = ref.head_softmax(d["q_logits"]); gk = ref.head_softmax(d["k_logits"])
    # float32 inputs cannot hold the gated values exactly, so compare through the numpy recurrence in fp64
    zeros = np.zeros((2, T, H), np.float32)
    qg = d["q"].astype(np.float64) * gq[..., None]
    kg = d["k"].astype(np.float64) * (gk[..., None] if variant != GDN else 1.0)
    vg = d["v"].astype(np.float64) * (gk[..., None] if variant == GDN else 1.0)
    # ungated = every head computed alone with gate 1
    for h in range(H):
        ld = _head_decay(variant, d["log_decay"], h)
        bt = None if d["beta"] is None else d["beta"][:, :, h:h + 1]
        o1, S1 = ref.recurrent(variant, qg[:, :, h:h + 1], kg[:, :, h:h + 1], vg[:, :, h:h + 1],
                               zeros[:, :, :1], None, ld, bt)
        np.testing.assert_allclose(o[:, :, h], o1[:, :, 0], rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(S[:, h], S1[:, 0], rtol=1e-11, atol=1e-13)


# ---------------------------------------------------------------- delta rule properties
def test_delta_rule_associative_recall_and_overwrite():
    """beta=1, no decay, gates 1, orthonormal keys: after writing (k_j, v_j) the state returns v_j for k_j;
    writing a key again replaces its value."""
    rng = np.random.default_rng(8)
    dk, dv, n = 8, 5, 6
    Qm, _ = np.linalg.qr(rng.standard_normal((dk, dk)))
    keys = Qm[:n].astype(np.float64)
    vals = rng.standard_normal((n + 1, dv))
    k = np.concatenate([keys, keys[2:3]], 0)  # token n rewrites key 2
    T = n + 1
    kk = k.reshape(1, T, 1, dk).astype(np.float32)
    vv = vals.reshape(1, T, 1, dv).astype(np.float32)
    zero = np.zeros((1, T, 1), np.float32)
    out, S = oracle.forward(GDN, kk, kk, vv, zero, None, zero, np.ones((1, T, 1), np.float32))
    k32 = kk[0, :, 0].astype(np.float64); v32 = vv[0, :, 0].astype(np.float64)
    # reading with q_t = k_t right after the write returns v_t (keys are orthonormal up to float32 rounding)
    np.testing.assert_allclose(out[0, :, 0], v32, atol=2e-6)
    recall = k32[:n] @ S[0, 0]
    want = v32[:n].copy(); want[2] = v32[n]
    np.testing.assert_allclose(recall, want, atol=2e-6)


def test_delta_rule_beta_zero_is_a_noop_and_zero_state_stays_zero():
    d = _rand(91, GDN, B=1, T=9, H=2, dk=4, dv=3)
    d["beta"] = np.zeros_like(d["beta"])
    out, S = _run(GDN, d)
    assert np.all(out == 0.0) and np.all(S == 0.0)
    s0 = si.initial_state(1, 2, 4, 3, seed=1)
    d["log_decay"] = np.zeros_like(d["log_decay"])
    out, S = _run(GDN, d, s0)
    np.testing.assert_array_equal(S, s0.astype(np.float64))


def test_gdn_without_decay_is_the_printed_delta_rule():
    """log-decay 0 must give the equations exactly as printed in Sec. 5.1 (no decay term)."""
    d = _rand(95, GDN, B=1, T=7, H=2, dk=3, dv=2)
    d["log_decay"] = np.zeros_like(d["log_decay"])
    out, S = _run(GDN, d)
    gq = ref.head_softmax(d["q_logits"]); gk = ref.head_softmax(d["k_logits"])
    for h in range(2):
        St = np.zeros((3, 2))
        for t in range(7):
            kt = d["k"][0, t, h].astype(np.float64); vt = d["v"][0, t, h].astype(np.float64)
            vnew = float(d["beta"][0, t, h]) * (gk[0, t, h] * vt - kt @ St)
            St = St + np.outer(kt, vnew)
            np.testing.assert_allclose(out[0, t, h], gq[0, t, h] * (d["q"][0, t, h].astype(np.float64) @ St),
                                       rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(S[0, h], St, rtol=1e-11, atol=1e-13)


# ---------------------------------------------------------------- state carry
@pytest.mark.parametrize("variant", [RETNET, GLA, GDN])
@pytest.mark.parametrize("split", [1, 5, 16, 20])
def test_two_chained_calls_equal_one_call(variant, split):
    T = 21
    d = _rand(101 + variant, variant, B=2, T=T, H=2, dk=4, dv=3)
    out, S = _run(variant, d)

    def cut(a, lo, hi, per_token):
        return None if a is None else (a[:, lo:hi] if per_token else a)

    def part(lo, hi, s0):
        return oracle.forward(variant, d["q"][:, lo:hi], d["k"][:, lo:hi], d["v"][:, lo:hi],
                              d["q_logits"][:, lo:hi], d["k_logits"][:, lo:hi],
                              cut(d["log_decay"], lo, hi, variant != RETNET), cut(d["beta"], lo, hi, True), s0)

    o1, S1 = part(0, split, None)
    o2, S2 = part(split, T, S1)
    # initial_state is float32 at the oracle's boundary: allow that rounding
    np.testing.assert_allclose(np.concatenate([o1, o2], 1), out, rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(S2, S, rtol=1e-5, atol=1e-6)


def test_empty_and_single_token():
    d = _rand(111, GLA, B=1, T=1, H=2, dk=3, dv=2)
    out, S = _run(GLA, d)
    gq = ref.head_softmax(d["q_logits"]); gk = ref.head_softmax(d["k_logits"])
    for h in range(2):
        St = gk[0, 0, h] * np.outer(d["k"][0, 0, h].astype(np.float64), d["v"][0, 0, h].astype(np.float64))
        np.testing.assert_allclose(S[0, h], St, rtol=1e-13)
        np.testing.assert_allclose(out[0, 0, h], gq[0, 0, h] * (d["q"][0, 0, h].astype(np.float64) @ St), rtol=1e-12)
    s0 = si.initial_state(1, 2, 3, 2, seed=2)
    e = lambda *s: np.zeros(s, np.float32)
    out, S = oracle.forward(GLA, e(1, 0, 2, 3), e(1, 0, 2, 3), e(1, 0, 2, 2), e(1, 0, 2), None, e(1, 0, 2, 3), None, s0)
    assert out.shape == (1, 0, 2, 2)
    np.testing.assert_array_equal(S, s0.astype(np.float64))


# ---------------------------------------------------------------- input generator sanity (no method arithmetic)
def test_generators_are_seeded_and_bf16_exact():
    w = si.workload("gla_train")
    a = si.generate(w, T=32, B=1); b = si.generate(w, T=32, B=1)
    for key in a:
        if a[key] is not None:
            np.testing.assert_array_equal(a[key], b[key])
    for key in ("q", "k", "v", "log_decay"):
        si.bf16_bits(a[key])  # raises if a value is not bf16-representable
    assert np.all(a["log_decay"] <= 0)
    w = si.workload("gla_long")
    c = si.generate(w, T=1024)
    top = np.argmax(c["q_logits"][0], axis=-1)
    assert (top[:512] == np.bincount(top[:512]).argmax()).mean() > 0.9
    g = si.generate(si.workload("gdn"), T=16, B=1)
    assert np.all((g["beta"] > 0) & (g["beta"] < 1))
    np.testing.assert_allclose(np.linalg.norm(g["k"].astype(np.float64), axis=-1), 1.0, atol=1e-2)


# ------------------------------------------------------------------ gate logits (the projection in front of Eq. 4)
def test_gate_logits_brute_force_and_selection():
    r = np.random.default_rng(77)
    x = r.normal(size=(2, 5, 3, 4))
    w = r.normal(size=(3, 4))
    got = ref.gate_logits(x, w)
    for b in range(2):
        for t in range(5):
            for h in range(3):
                assert abs(got[b, t, h] - sum(x[b, t, h, d] * w[h, d] for d in range(4))) < 1e-12
    # a one-hot weight row reads out one coordinate of its own head and nothing of the others
    sel = np.zeros((3, 4))
    sel[0, 2] = sel[1, 0] = sel[2, 3] = 1.0
    got = ref.gate_logits(x, sel)
    assert np.array_equal(got[..., 0], x[:, :, 0, 2]) and np.array_equal(got[..., 1], x[:, :, 1, 0])
    assert np.array_equal(got[..., 2], x[:, :, 2, 3])
    # linear in x and in w
    np.testing.assert_allclose(ref.gate_logits(2 * x, w) + ref.gate_logits(x, 3 * w), 5 * ref.gate_logits(x, w),
                               rtol=1e-13, atol=1e-13)


# ------------------------------------------------------------------ short causal convolution + SiLU (Sec. 5.1, GDN blocks)
def test_short_conv_silu_against_library_filters():
    from scipy.signal import lfilter
    import torch

    r = np.random.default_rng(88)
    x = r.normal(size=(2, 37, 6))
    for K in (1, 2, 3, 4):
        w = r.normal(size=(6, K))
        got = ref.short_conv_silu(x, w)
        # an FIR filter per channel: coefficient of x[t - m] is w[c, K-1-m]
        pre = np.stack([np.stack([lfilter(w[c, ::-1], [1.0], x[b, :, c]) for c in range(6)], axis=-1) for b in range(2)])
        np.testing.assert_allclose(got, pre / (1.0 + np.exp(-pre)), rtol=1e-12, atol=1e-13)
        # torch's depthwise conv1d with left padding, then its own SiLU
        xt = torch.tensor(x).permute(0, 2, 1)
        yt = torch.nn.functional.conv1d(torch.nn.functional.pad(xt, (K - 1, 0)), torch.tensor(w)[:, None, :], groups=6)
        np.testing.assert_allclose(got, torch.nn.functional.silu(yt).permute(0, 2, 1).numpy(), rtol=1e-12, atol=1e-13)
    # one tap of weight 1 is SiLU itself; causality: changing a later input leaves earlier outputs alone
    one = np.ones((6, 1))
    np.testing.assert_allclose(ref.short_conv_silu(x, one), x / (1.0 + np.exp(-x)), rtol=1e-14)
    w = r.normal(size=(6, 4))
    x2 = x.copy()
    x2[:, 20:] += 1.0
    assert np.array_equal(ref.short_conv_silu(x, w)[:, :20], ref.short_conv_silu(x2, w)[:, :20])
