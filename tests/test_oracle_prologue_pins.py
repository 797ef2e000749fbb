"""Pins of oracle/sla_prologue.py (no GPU): the backward statements against central finite differences of the
forward statements and against torch autograd through library operators (conv1d, silu, normalize, einsum); the L2
option against its defining properties."""
import numpy as np
import pytest
import torch

from oracle import sla_numpy as on
from oracle import sla_prologue as op


def _fd(f, x, eps=1e-6):
    """Central finite differences of the scalar function f at x (every element)."""
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = x[i]
        x[i] = old + eps
        fp = f()
        x[i] = old - eps
        fm = f()
        x[i] = old
        g[i] = (fp - fm) / (2 * eps)
    return g


def test_gate_logits_backward_finite_differences_and_autograd():
    rng = np.random.default_rng(1)
    B, T, H, d = 2, 3, 3, 4
    x, w, g = rng.normal(size=(B, T, H, d)), rng.normal(size=(H, d)), rng.normal(size=(B, T, H))
    dx, dw = op.gate_logits_backward(x, w, g)
    loss = lambda: float(np.sum(on.gate_logits(x, w) * g))
    np.testing.assert_allclose(dx, _fd(loss, x), rtol=1e-7, atol=1e-8)
    np.testing.assert_allclose(dw, _fd(loss, w), rtol=1e-7, atol=1e-8)
    xt, wt = torch.tensor(x, requires_grad=True), torch.tensor(w, requires_grad=True)
    (torch.einsum("bthd,hd->bth", xt, wt) * torch.tensor(g)).sum().backward()
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dw, wt.grad.numpy(), rtol=1e-12, atol=1e-12)
    # one head's weights touch only that head's slice
    g2 = np.zeros_like(g)
    g2[:, :, 1] = 1.0
    dx2, dw2 = op.gate_logits_backward(x, w, g2)
    assert np.all(dx2[:, :, [0, 2]] == 0) and np.all(dw2[[0, 2]] == 0)
    np.testing.assert_allclose(dw2[1], x[:, :, 1].sum(axis=(0, 1)))


def test_l2_option_properties():
    rng = np.random.default_rng(2)
    x, w = rng.normal(size=(2, 9, 8)), rng.normal(size=(8, 4))
    plain = op.short_conv_silu_l2(x, w)
    np.testing.assert_allclose(plain, on.short_conv_silu(x, w), rtol=1e-14)  # head_width = 0: the feature map alone
    y = op.short_conv_silu_l2(x, w, head_width=4, eps=0.0)
    np.testing.assert_allclose(np.sum(y.reshape(2, 9, 2, 4) ** 2, axis=-1), 1.0, rtol=1e-12)  # unit vectors per head
    # the direction is the feature map's; torch's normalize agrees
    want = torch.nn.functional.normalize(torch.tensor(plain).reshape(2, 9, 2, 4), dim=-1, eps=0.0).reshape(2, 9, 8)
    np.testing.assert_allclose(y, want.numpy(), rtol=1e-12)
    # eps enters under the root: a zero vector stays zero and finite
    z = op.short_conv_silu_l2(np.zeros((1, 3, 8)), w, head_width=4, eps=1e-6)
    assert np.all(z == 0)
    # with eps: y = a / sqrt(|a|^2 + eps)
    a = plain.reshape(2, 9, 2, 4)
    y6 = op.short_conv_silu_l2(x, w, head_width=4, eps=1e-2).reshape(2, 9, 2, 4)
    np.testing.assert_allclose(y6, a / np.sqrt((a * a).sum(-1, keepdims=True) + 1e-2), rtol=1e-12)


@pytest.mark.parametrize("head_width,eps", [(0, 0.0), (4, 1e-6), (8, 1e-2)])
@pytest.mark.parametrize("K", [1, 3, 4])
def test_short_conv_backward_finite_differences_and_autograd(head_width, eps, K):
    rng = np.random.default_rng(3 + K)
    B, T, C = 2, 7, 8
    x, w, g = rng.normal(size=(B, T, C)), rng.normal(size=(C, K)), rng.normal(size=(B, T, C))
    dx, dw = op.short_conv_silu_l2_backward(x, w, g, head_width, eps)
    loss = lambda: float(np.sum(op.short_conv_silu_l2(x, w, head_width, eps) * g))
    np.testing.assert_allclose(dx, _fd(loss, x), rtol=2e-6, atol=1e-8)
    np.testing.assert_allclose(dw, _fd(loss, w), rtol=2e-6, atol=1e-8)
    # autograd through library operators: left-padded depthwise conv1d, silu, normalisation written with torch ops
    xt, wt = torch.tensor(x, requires_grad=True), torch.tensor(w, requires_grad=True)
    s = torch.nn.functional.conv1d(torch.nn.functional.pad(xt.transpose(1, 2), (K - 1, 0)), wt[:, None, :], groups=C)
    a = torch.nn.functional.silu(s).transpose(1, 2)
    if head_width:
        ah = a.reshape(B, T, C // head_width, head_width)
        a = (ah * torch.rsqrt((ah * ah).sum(-1, keepdim=True) + eps)).reshape(B, T, C)
    (a * torch.tensor(g)).sum().backward()
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dw, wt.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_short_conv_backward_is_causal_and_per_channel():
    """A cotangent on one token and channel reaches only that channel, and only the K tokens up to it."""
    rng = np.random.default_rng(9)
    x, w = rng.normal(size=(1, 10, 4)), rng.normal(size=(4, 3))
    g = np.zeros((1, 10, 4))
    g[0, 6, 2] = 1.0
    dx, dw = op.short_conv_silu_l2_backward(x, w, g)
    mask = np.zeros_like(dx, dtype=bool)
    mask[0, 4:7, 2] = True
    assert np.all(dx[~mask] == 0) and np.all(dx[mask] != 0)
    assert np.all(dw[[0, 1, 3]] == 0)
