"""Oracle statements for what sits in front of the SLA mixer and for the gradients flowing back through it, fp64
numpy.  TEST INFRASTRUCTURE ONLY: the GPU library never imports this module and shares no code with it.

* the gate projections of Eq. 4 (``q W_GQ``, ``k W_GK`` under the per-head reading of the gate matrices that the
  parameter count of Sec. 3.2, Parameter Efficiency, implies) and their backward;
* the feature map of the Gated DeltaNet blocks (Sec. 5.1, Model Configuration: short convolution, then SiLU),
  optionally followed by an L2 normalisation of every head's vector (the benchmark's delta-rule workload feeds
  L2-normalised queries and keys; the paper does not spell the normalisation out, so it is an option here), and its
  backward.

Every function is the definition written out with loops over taps / heads; nothing is blocked or fused.
"""
from __future__ import annotations

from typing import Tuple

import numpy as np


def gate_logits_backward(x, w, dlogits) -> Tuple[np.ndarray, np.ndarray]:
    """Backward of ``logits[b,t,h] = sum_d x[b,t,h,d] w[h,d]`` (Eq. 4's scores): returns (dx, dw) with
    dx[b,t,h,:] = dlogits[b,t,h] w[h,:] and dw[h,:] = sum_{b,t} dlogits[b,t,h] x[b,t,h,:]."""
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    g = np.asarray(dlogits, dtype=np.float64)
    B, T, H, d = x.shape
    assert w.shape == (H, d) and g.shape == (B, T, H)
    dx = np.zeros_like(x)
    dw = np.zeros_like(w)
    for h in range(H):
        dx[:, :, h, :] = g[:, :, h, None] * w[h][None, None, :]
        dw[h] = np.einsum("bt,btd->d", g[:, :, h], x[:, :, h, :])
    return dx, dw


def _conv(x: np.ndarray, w: np.ndarray) -> np.ndarray:
    B, T, C = x.shape
    K = w.shape[1]
    s = np.zeros_like(x)
    for t in range(T):
        for i in range(K):
            src = t - (K - 1) + i
            if src >= 0:
                s[:, t, :] += w[:, i] * x[:, src, :]
    return s


def _sigmoid(s: np.ndarray) -> np.ndarray:
    return 1.0 / (1.0 + np.exp(-s))


def short_conv_silu_l2(x, w, head_width: int = 0, eps: float = 1e-6) -> np.ndarray:
    """y = silu(causal depthwise convolution of x with w) (x [B,T,C], w [C,K], tap K-1 on the current token, zeros
    before the sequence); with head_width > 0 every group of head_width adjacent channels of a token is then
    divided by sqrt(sum of its squares + eps)."""
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    s = _conv(x, w)
    a = s * _sigmoid(s)
    if head_width <= 0:
        return a
    B, T, C = a.shape
    assert C % head_width == 0
    ah = a.reshape(B, T, C // head_width, head_width)
    r = 1.0 / np.sqrt(np.sum(ah * ah, axis=-1, keepdims=True) + eps)
    return (ah * r).reshape(B, T, C)


def short_conv_silu_l2_backward(x, w, dy, head_width: int = 0, eps: float = 1e-6) -> Tuple[np.ndarray, np.ndarray]:
    """Backward of ``short_conv_silu_l2``: returns (dx [B,T,C], dw [C,K]) for the cotangent dy of y.

    Chain: y = a r with r = (sum_head a^2 + eps)^-1/2  =>  da = r dy - a r^3 sum_head(a dy);
           a = s sigmoid(s)                             =>  ds = da sigmoid(s) (1 + s (1 - sigmoid(s)));
           s[t] = sum_i w[i] x[t-(K-1)+i]               =>  dx[u] += w[i] ds[u+(K-1)-i],  dw[i] += ds[t] x[t-(K-1)+i]."""
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    dy = np.asarray(dy, dtype=np.float64)
    B, T, C = x.shape
    K = w.shape[1]
    s = _conv(x, w)
    sg = _sigmoid(s)
    a = s * sg
    if head_width > 0:
        nh = C // head_width
        ah = a.reshape(B, T, nh, head_width)
        gh = dy.reshape(B, T, nh, head_width)
        r = 1.0 / np.sqrt(np.sum(ah * ah, axis=-1, keepdims=True) + eps)
        da = (r * gh - ah * r ** 3 * np.sum(ah * gh, axis=-1, keepdims=True)).reshape(B, T, C)
    else:
        da = dy
    ds = da * sg * (1.0 + s * (1.0 - sg))
    dx = np.zeros_like(x)
    dw = np.zeros_like(w)
    for t in range(T):
        for i in range(K):
            src = t - (K - 1) + i
            if src >= 0:
                dx[:, src, :] += w[:, i] * ds[:, t, :]
                dw[:, i] += np.sum(ds[:, t, :] * x[:, src, :], axis=0)
    return dx, dw
