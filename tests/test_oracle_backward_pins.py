"""Pins of the gradient oracle (oracle/sla_backward.py) against things other than itself:

* central finite differences of the recurrence (Eq. 5-6, Sec. 5.1) for every element of every input,
  including the initial state and the final-state cotangent;
* torch's reverse-mode autograd through the masked parallel form of Appendix A (which never forms a
  state) with the decay weights of RetNet / GLA;
* the closed form for a single token;
* properties of Eq. 4's softmax: logit gradients sum to zero over heads, and vanish for one head.
"""
import numpy as np
import pytest
import torch

from oracle import sla_backward, sla_numpy

RETNET, GLA = sla_numpy.RETNET, sla_numpy.GLA


def make(variant, B, T, H, dk, dv, seed, k_logits=True, states=True):
    r = np.random.default_rng(seed)
    d = {
        "q": r.normal(size=(B, T, H, dk)),
        "k": r.normal(size=(B, T, H, dk)),
        "v": r.normal(size=(B, T, H, dv)),
        "q_logits": r.normal(size=(B, T, H)),
        "k_logits": r.normal(size=(B, T, H)) if k_logits else None,
        "log_decay": -r.uniform(0.05, 1.0, size=(H,) if variant == RETNET else (B, T, H, dk)),
        "initial_state": r.normal(size=(B, H, dk, dv)) if states else None,
    }
    cot = {
        "d_out": r.normal(size=(B, T, H, dv)),
        "d_final_state": r.normal(size=(B, H, dk, dv)) if states else None,
    }
    return d, cot


def objective(variant, d, cot):
    out, fin = sla_numpy.recurrent(variant, d["q"], d["k"], d["v"], d["q_logits"], d["k_logits"], d["log_decay"],
                                   None, d["initial_state"])
    val = np.sum(out * cot["d_out"])
    if cot["d_final_state"] is not None:
        val += np.sum(fin * cot["d_final_state"])
    return val


def oracle_grads(variant, d, cot, **kw):
    return sla_backward.backward(variant, d["q"], d["k"], d["v"], d["q_logits"], d["k_logits"], d["log_decay"],
                                 cot["d_out"], d["initial_state"], cot["d_final_state"], **kw)


NAMES = {"q": "dq", "k": "dk", "v": "dv", "q_logits": "dq_logits", "k_logits": "dk_logits",
         "log_decay": "dlog_decay", "initial_state": "dinitial_state"}


@pytest.mark.parametrize("variant", [RETNET, GLA])
@pytest.mark.parametrize("k_logits,states", [(True, True), (False, False)])
def test_finite_differences(variant, k_logits, states):
    d, cot = make(variant, 2, 5, 3, 3, 4, seed=7 + variant, k_logits=k_logits, states=states)
    g = oracle_grads(variant, d, cot, checkpoint=2)
    h = 1e-6
    for name, gname in NAMES.items():
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
