"""Pins of the gradient oracle (oracle/sla_backward.py) against things other than itself:

* central finite differences of the recurrence (Eq. 5-6, Sec. 5.1) for every element of every input,
  including the initial state and the final-state cotangent;
* torch's reverse-mode autograd through the masked parallel form of Appendix A (which never forms a
  state) with the decay weights of RetNet / GLA;
* for the gated delta rule, torch's autograd through the per-chunk triangular-solve form (no per-token state);
* the closed form for a single token;
* properties of Eq. 4's softmax: logit gradients sum to zero over heads, and vanish for one head.
"""
import numpy as np
import pytest
import torch

from oracle import sla_backward, sla_numpy

RETNET, GLA, GDN = sla_numpy.RETNET, sla_numpy.GLA, sla_numpy.GDN


def make(variant, B, T, H, dk, dv, seed, k_logits=True, states=True):
    r = np.random.default_rng(seed)
    d = {
        "q": r.normal(size=(B, T, H, dk)),
        "k": r.normal(size=(B, T, H, dk)),
        "v": r.normal(size=(B, T, H, dv)),
        "q_logits": r.normal(size=(B, T, H)),
        "k_logits": r.normal(size=(B, T, H)) if k_logits else None,
        "log_decay": -r.uniform(0.05, 1.0, size={RETNET: (H,), GLA: (B, T, H, dk), GDN: (B, T, H)}[variant]),
        "initial_state": r.normal(size=(B, H, dk, dv)) if states else None,
    }
    if variant == GDN:
        d["k"] /= np.linalg.norm(d["k"], axis=-1, keepdims=True)
        d["beta"] = r.uniform(0.1, 0.9, size=(B, T, H))
    cot = {
        "d_out": r.normal(size=(B, T, H, dv)),
        "d_final_state": r.normal(size=(B, H, dk, dv)) if states else None,
    }
    return d, cot


def objective(variant, d, cot):
    out, fin = sla_numpy.recurrent(variant, d["q"], d["k"], d["v"], d["q_logits"], d["k_logits"], d["log_decay"],
                                   d.get("beta"), d["initial_state"])
    val = np.sum(out * cot["d_out"])
    if cot["d_final_state"] is not None:
        val += np.sum(fin * cot["d_final_state"])
    return val


def oracle_grads(variant, d, cot, **kw):
    return sla_backward.backward(variant, d["q"], d["k"], d["v"], d["q_logits"], d["k_logits"], d["log_decay"],
                                 cot["d_out"], d["initial_state"], cot["d_final_state"], beta=d.get("beta"), **kw)


NAMES = {"q": "dq", "k": "dk", "v": "dv", "q_logits": "dq_logits", "k_logits": "dk_logits",
         "log_decay": "dlog_decay", "initial_state": "dinitial_state", "beta": "dbeta"}


@pytest.mark.parametrize("variant", [RETNET, GLA, GDN])
@pytest.mark.parametrize("k_logits,states", [(True, True), (False, False)])
def test_finite_differences(variant, k_logits, states):
    d, cot = make(variant, 2, 5, 3, 3, 4, seed=7 + variant, k_logits=k_logits, states=states)
    g = oracle_grads(variant, d, cot, checkpoint=2)
    h = 1e-6
    for name, gname in NAMES.items():
        if name not in d:
            assert g[gname] is None
            continue
        if d[name] is None:
            assert g[gname] is None or name == "initial_state"
            continue
        fd = np.zeros_like(d[name])
        it = np.nditer(d[name], flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            keep = d[name][i]
            d[name][i] = keep + h
            up = objective(variant, d, cot)
            d[name][i] = keep - h
            dn = objective(variant, d, cot)
            d[name][i] = keep
            fd[i] = (up - dn) / (2 * h)
        scale = max(1.0, np.max(np.abs(fd)))
        assert np.max(np.abs(fd - g[gname])) <= 1e-7 * scale, name


def torch_quadratic(variant, q, k, v, ql, kl, ld):
    """Appendix A's parallel form with decay weights, in torch fp64 (differentiable)."""
    B, T, H, dk = q.shape
    gq = torch.softmax(ql, dim=-1)
    gk = torch.softmax(kl, dim=-1) if kl is not None else torch.ones_like(ql)
    if variant == RETNET:
        steps = ld[None, None, :, None].expand(B, T, H, dk)
    else:
        steps = ld
    c = torch.cumsum(steps, dim=1)  # [B,T,H,dk]
    # w[b,t,j,h,d] = exp(c_t - c_j) for j <= t
    w = torch.exp(c[:, :, None] - c[:, None, :])
    score = torch.einsum("bthd,bjhd,btjhd->bhtj", q, k, w)
    mask = torch.tril(torch.ones(T, T, dtype=torch.bool))
    score = torch.where(mask[None, None], score, torch.zeros((), dtype=q.dtype))
    score = score * gk.permute(0, 2, 1)[:, :, None, :]
    return gq[..., None] * torch.einsum("bhtj,bjhn->bthn", score, v)


@pytest.mark.parametrize("variant", [RETNET, GLA])
@pytest.mark.parametrize("k_logits", [True, False])
def test_autograd_of_parallel_form(variant, k_logits):
    d, cot = make(variant, 2, 23, 4, 5, 6, seed=31 + variant, k_logits=k_logits, states=False)
    g = oracle_grads(variant, d, cot, checkpoint=7)
    names = ["q", "k", "v", "q_logits", "log_decay"] + (["k_logits"] if k_logits else [])
    t = {n: torch.tensor(d[n], dtype=torch.float64, requires_grad=True) for n in names}
    out = torch_quadratic(variant, t["q"], t["k"], t["v"], t["q_logits"], t.get("k_logits"), t["log_decay"])
    (out * torch.tensor(cot["d_out"])).sum().backward()
    for n in names:
        ref = t[n].grad.numpy()
        assert np.max(np.abs(ref - g[NAMES[n]])) <= 1e-10 * max(1.0, np.max(np.abs(ref))), n


def torch_gdn_chunked(q, k, v, ql, kl, ld, beta, chunk, S0=None):
    """The gated delta rule as one triangular solve per chunk (unrolled recurrence of Sec. 5.1), torch fp64."""
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    gq = torch.softmax(ql, dim=-1)
    gk = torch.softmax(kl, dim=-1) if kl is not None else torch.ones_like(ql)
    outs = []
    S = torch.zeros(B, H, dk, dv, dtype=q.dtype) if S0 is None else S0
    for s in range(0, T, chunk):
        e = min(T, s + chunk)
        n = e - s
        K, Q, V = (x[:, s:e].permute(0, 2, 1, 3) for x in (k, q, v))      # [B,H,n,d]
        bt, gK, gQ = (x[:, s:e].permute(0, 2, 1) for x in (beta, gk, gq))  # [B,H,n]
        c = torch.cumsum(ld[:, s:e].permute(0, 2, 1), dim=-1)
        D = torch.exp(c[..., :, None] - c[..., None, :])
        L = torch.tril(bt[..., :, None] * D * (K @ K.transpose(-1, -2)), -1)
        rhs = (bt * gK)[..., None] * V - (bt * torch.exp(c))[..., None] * (K @ S)
        U = torch.linalg.solve_triangular(torch.eye(n, dtype=q.dtype) + L, rhs, upper=False)
        A = torch.tril(D * (Q @ K.transpose(-1, -2)))
        outs.append((gQ[..., None] * (torch.exp(c)[..., None] * (Q @ S) + A @ U)).permute(0, 2, 1, 3))
        S = torch.exp(c[..., -1])[..., None, None] * S + (torch.exp(c[..., -1:] - c)[..., None] * K).transpose(-1, -2) @ U
    return torch.cat(outs, dim=1), S


@pytest.mark.parametrize("k_logits,states,chunk", [(True, True, 4), (False, False, 23), (True, False, 7)])
def test_gdn_autograd_of_chunked_solve_form(k_logits, states, chunk):
    d, cot = make(GDN, 2, 23, 3, 5, 6, seed=41, k_logits=k_logits, states=states)
    g = oracle_grads(GDN, d, cot, checkpoint=5)
    names = ["q", "k", "v", "q_logits", "log_decay", "beta"] + (["k_logits"] if k_logits else []) + \
            (["initial_state"] if states else [])
    t = {n: torch.tensor(d[n], dtype=torch.float64, requires_grad=True) for n in names}
    out, fin = torch_gdn_chunked(t["q"], t["k"], t["v"], t["q_logits"], t.get("k_logits"), t["log_decay"], t["beta"],
                                 chunk, t.get("initial_state"))
    loss = (out * torch.tensor(cot["d_out"])).sum()
    if states:
        loss = loss + (fin * torch.tensor(cot["d_final_state"])).sum()
    loss.backward()
    for n in names:
        ref = t[n].grad.numpy()
        assert np.max(np.abs(ref - g[NAMES[n]])) <= 1e-10 * max(1.0, np.max(np.abs(ref))), n


def test_gdn_single_token_closed_form():
    # T = 1, zero state: out = G^Q (q . k) beta G^K v; the decay only touches the zero state
    d, cot = make(GDN, 1, 1, 3, 4, 5, seed=6, states=False)
    g = oracle_grads(GDN, d, cot)
    gq = sla_numpy.head_softmax(d["q_logits"])[0, 0]
    gk = sla_numpy.head_softmax(d["k_logits"])[0, 0]
    q, k, v, do, bt = d["q"][0, 0], d["k"][0, 0], d["v"][0, 0], cot["d_out"][0, 0], d["beta"][0, 0]
    qk, dov = np.sum(q * k, axis=-1), np.sum(do * v, axis=-1)
    np.testing.assert_allclose(g["dbeta"][0, 0], gq * gk * qk * dov, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(g["dq"][0, 0], (gq * gk * bt * dov)[:, None] * k, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(g["dk"][0, 0], (gq * gk * bt * dov)[:, None] * q, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(g["dv"][0, 0], (gq * gk * bt * qk)[:, None] * do, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(g["dlog_decay"], 0.0, atol=1e-14)


def test_gdn_without_erasure_is_scalar_decay_linear_attention():
    # keys that the state never holds yet (zero state, mutually orthogonal keys): k_t Sb = 0, so the delta rule
    # writes beta G^K v like RetNet / GLA write G^K v; compare with GLA fed v * beta and a decay constant over dk
    B, T, H, dk, dv = 1, 4, 2, 4, 3
    d, cot = make(GDN, B, T, H, dk, dv, seed=9, states=False)
    d["k"] = np.broadcast_to(np.eye(dk)[None, :T, None, :], (B, T, H, dk)).copy()
    g = oracle_grads(GDN, d, cot)
    dg = {n: d[n] for n in ("q", "k", "q_logits", "k_logits", "initial_state")}
    dg["v"] = d["v"] * d["beta"][..., None]
    dg["log_decay"] = np.broadcast_to(d["log_decay"][..., None], (B, T, H, dk)).copy()
    gg = oracle_grads(GLA, dg, cot)
    for n in ("dq", "dq_logits", "dk_logits"):
        np.testing.assert_allclose(g[n], gg[n], rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(g["dv"], gg["dv"] * d["beta"][..., None], rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(g["dbeta"], np.sum(gg["dv"] * d["v"], axis=-1), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(g["dlog_decay"], np.sum(gg["dlog_decay"], axis=-1), rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("variant", [RETNET, GLA])
def test_single_token_closed_form(variant):
    # T = 1, zero initial state: out = G^Q G^K (q . k) v, so every gradient is a one-line expression
    d, cot = make(variant, 1, 1, 3, 4, 5, seed=5, states=False)
    g = oracle_grads(variant, d, cot)
    gq = sla_numpy.head_softmax(d["q_logits"])[0, 0]
    gk = sla_numpy.head_softmax(d["k_logits"])[0, 0]
    q, k, v, do = d["q"][0, 0], d["k"][0, 0], d["v"][0, 0], cot["d_out"][0, 0]
    qk = np.sum(q * k, axis=-1)
    dov = np.sum(do * v, axis=-1)
    np.testing.assert_allclose(g["dq"][0, 0], (gq * gk * dov)[:, None] * k, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(g["dk"][0, 0], (gq * gk * dov)[:, None] * q, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(g["dv"][0, 0], (gq * gk * qk)[:, None] * do, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(g["dlog_decay"], 0.0, atol=1e-14)  # the decay only touches the zero state
    dgq = gk * qk * dov
    np.testing.assert_allclose(g["dq_logits"][0, 0], gq * (dgq - np.sum(gq * dgq)), rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("variant", [RETNET, GLA])
def test_softmax_properties(variant):
    d, cot = make(variant, 2, 9, 4, 3, 3, seed=11)
    g = oracle_grads(variant, d, cot)
    assert np.max(np.abs(np.sum(g["dq_logits"], axis=-1))) < 1e-12
    assert np.max(np.abs(np.sum(g["dk_logits"], axis=-1))) < 1e-12
    d1, cot1 = make(variant, 2, 9, 1, 3, 3, seed=12)  # one head: the gate is identically 1
    g1 = oracle_grads(variant, d1, cot1)
    assert np.max(np.abs(g1["dq_logits"])) == 0.0 and np.max(np.abs(g1["dk_logits"])) == 0.0


def test_retnet_is_gla_with_constant_decay():
    d, cot = make(RETNET, 2, 11, 3, 4, 5, seed=3)
    g = oracle_grads(RETNET, d, cot)
    dg = dict(d)
    dg["log_decay"] = np.broadcast_to(d["log_decay"][None, None, :, None], (2, 11, 3, 4)).copy()
    gg = oracle_grads(GLA, dg, cot)
    for n in ("dq", "dk", "dv", "dq_logits", "dk_logits", "dinitial_state"):
        np.testing.assert_allclose(g[n], gg[n], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(g["dlog_decay"], gg["dlog_decay"].sum(axis=(0, 1, 3)), rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("variant", [0, 1, 2])
@pytest.mark.parametrize("with_kl,with_states", [(True, True), (False, False), (True, False)])
def test_c_gradient_oracle_equals_the_numpy_one(variant, with_kl, with_states):
    """oracle/sla_oracle_backward.c is a second implementation of oracle/sla_backward.py (itself pinned above by
    finite differences and autograd): every gradient agrees to fp64 rounding, for a length that spans several of
    its 64-token checkpoints and ends inside one."""
    import oracle
    import sla_inputs as si

    B, T, H, dk, dv = 2, 150, 3, 8, 5
    d = si.custom(variant, "f32", B=B, T=T, H=H, dk=dk, dv=dv, seed=700 + variant)
    cot = si.cotangents(B, T, H, dk, dv, seed=701, dtype="f32", final_state=with_states)
    s0 = si.initial_state(B, H, dk, dv, seed=702) if with_states else None
    kl = d["k_logits"] if with_kl else None
    ref = sla_backward.backward(variant, d["q"], d["k"], d["v"], d["q_logits"], kl, d["log_decay"], cot["d_out"], s0,
                                cot.get("d_final_state"), beta=d["beta"])
    got = oracle.backward(variant, d["q"], d["k"], d["v"], d["q_logits"], kl, d["log_decay"], cot["d_out"], s0,
                          cot.get("d_final_state"), beta=d["beta"], nthreads=2)
    assert set(got) == set(ref)
    for name in ref:
        if ref[name] is None:
            assert got[name] is None, name
            continue
        scale = max(float(np.max(np.abs(ref[name]))), 1e-30)
        assert float(np.max(np.abs(got[name] - ref[name]))) <= 1e-12 * scale, name
