"""Plain numpy statements of the SLA forward pass (fp64).

TEST INFRASTRUCTURE ONLY: these functions define what the GPU library must
compute and are used to pin the C oracle (``sla_oracle.c``); the GPU library
never imports this package and shares no code with it.

``gate_logits`` states the projection in front of Eq. 4's softmax.  Three independent statements of the forward
mathematics live here:

* ``recurrent``     – the token-by-token recurrence (Eq. 5-6 and the three
                      instantiations of Sec. 5.1), vectorised over (batch, head)
                      only; the loop over tokens is the definition itself.
* ``quadratic``     – the masked parallel form of Appendix A (first equation),
                      extended with the decay weights of RetNet / GLA: every
                      output is an explicit sum over all earlier tokens.  It
                      never forms a state.
* ``gdn_chunked``   – the delta-rule update written per chunk with one
                      triangular solve (the "chunkwise parallel" paragraph of
                      Sec. 3.2 applied to the gated delta rule).  For chunk
                      size 1 it is the recurrence; agreement for every chunk
                      size is a pin of both.

Layouts: q,k [B,T,H,dk]; v [B,T,H,dv]; logits [B,T,H]; RetNet log_decay [H];
GLA log_decay [B,T,H,dk]; GDN log_decay, beta [B,T,H]; state [B,H,dk,dv].
"""
from __future__ import annotations

from typing import Optional, Tuple

import numpy as np

RETNET, GLA, GDN = 0, 1, 2


def head_softmax(logits: Optional[np.ndarray], shape=None) -> np.ndarray:
    """Eq. 4: softmax across the head axis (last axis of ``[B,T,H]``), fp64."""
    if logits is None:
        return np.ones(shape, dtype=np.float64)
    x = np.asarray(logits, dtype=np.float64)
    e = np.exp(x - np.max(x, axis=-1, keepdims=True))
    return e / np.sum(e, axis=-1, keepdims=True)


def gate_logits(x, w) -> np.ndarray:
    """The scores of Eq. 4 under the per-head reading of W in R^{d x H} (d = head width, Sec. 3.2 "Parameter
    Efficiency"): logits[b,t,h] = sum_d x[b,t,h,d] * W[d,h].  ``w`` is given as ``[H,d]`` (row h = column h of W)."""
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    B, T, H, d = x.shape
    assert w.shape == (H, d)
    out = np.zeros((B, T, H))
    for h in range(H):
        out[:, :, h] = x[:, :, h, :] @ w[h]
    return out


def short_conv_silu(x, w) -> np.ndarray:
    """The feature map of the Gated DeltaNet blocks (Sec. 5.1, "Model Configuration"): a short causal convolution
    along the tokens, per channel, followed by SiLU.  x [B,T,C], w [C,K]; tap K-1 multiplies the current token,
    inputs before the sequence are zero."""
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    B, T, C = x.shape
    K = w.shape[1]
    s = np.zeros_like(x)
    for t in range(T):
        for i in range(K):
            src = t - (K - 1) + i
            if src >= 0:
                s[:, t, :] += w[:, i] * x[:, src, :]
    return s / (1.0 + np.exp(-s))


def recurrent(
    variant: int,
    q,
    k,
    v,
    q_logits,
    k_logits,
    log_decay,
    beta=None,
    initial_state=None,
) -> Tuple[np.ndarray, np.ndarray]:
    """Token-by-token SLA recurrence.  Returns (out [B,T,H,dv], final_state [B,H,dk,dv])."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    gq = head_softmax(q_logits)
    gk = head_softmax(k_logits, (B, T, H))
    ld = np.asarray(log_decay, dtype=np.float64)
    S = np.zeros((B, H, dk, dv)) if initial_state is None else np.array(initial_state, dtype=np.float64)
    out = np.zeros((B, T, H, dv))
    for t in range(T):
        kt, vt, qt = k[:, t], v[:, t], q[:, t]  # [B,H,d]
        if variant == RETNET:
            S = np.exp(ld)[None, :, None, None] * S + (gk[:, t, :, None] * kt)[..., :, None] * vt[..., None, :]
        elif variant == GLA:
            S = np.exp(ld[:, t])[..., :, None] * S + (gk[:, t, :, None] * kt)[..., :, None] * vt[..., None, :]
        elif variant == GDN:
            Sb = np.exp(ld[:, t])[..., None, None] * S
            kS = np.einsum("bhd,bhdn->bhn", kt, Sb)
            u = np.asarray(beta, dtype=np.float64)[:, t, :, None] * (gk[:, t, :, None] * vt - kS)
            S = Sb + kt[..., :, None] * u[..., None, :]
        else:
            raise ValueError(variant)
        out[:, t] = gq[:, t, :, None] * np.einsum("bhd,bhdn->bhn", qt, S)
    return out, S


def quadratic(variant: int, q, k, v, q_logits, k_logits, log_decay) -> np.ndarray:
    """Appendix A, parallel form, with decay weights; RetNet and GLA only.

    out[b,t,h,:] = G^Q[t,h] * sum_{j<=t} G^K[j,h] * (sum_d q[t,d] k[j,d] w[t,j,d]) * v[j,:]
    with w[t,j,d] = prod_{i=j+1..t} alpha[i,d]  (alpha = gamma_h for RetNet).
    Written with explicit loops over (t, j); meant for tiny inputs.
    """
    if variant not in (RETNET, GLA):
        raise ValueError("the quadratic form exists for RetNet and GLA only")
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    gq = head_softmax(q_logits)
    gk = head_softmax(k_logits, (B, T, H))
    ld = np.asarray(log_decay, dtype=np.float64)
    out = np.zeros((B, T, H, dv))
    for b in range(B):
        for h in range(H):
            for t in range(T):
                acc = np.zeros(dv)
                for j in range(t + 1):
                    if variant == RETNET:
                        w = np.full(dk, np.exp(ld[h]) ** (t - j))
                    else:
                        w = np.exp(np.sum(ld[b, j + 1 : t + 1, h, :], axis=0))
                    score = np.sum(q[b, t, h] * k[b, j, h] * w)
                    acc += gk[b, j, h] * score * v[b, j, h]
                out[b, t, h] = gq[b, t, h] * acc
    return out


def gdn_chunked(q, k, v, q_logits, k_logits, log_decay, beta, chunk: int, initial_state=None):
    """Gated delta rule, one triangular solve per chunk of ``chunk`` tokens.

    Within a chunk entered with state S0, with c_t the running sum of the
    log-decay inside the chunk:
        (I + L) U = diag(beta G^K) V - diag(beta e^{c}) K S0,
        L[j,i] = beta_j e^{c_j - c_i} (k_j . k_i)   for i < j   (strictly lower)
        out_t  = G^Q_t ( e^{c_t} q_t S0 + sum_{j<=t} e^{c_t - c_j} (q_t . k_j) u_j )
        S_end  = e^{c_end} S0 + sum_j e^{c_end - c_j} k_j^T u_j
    which follows from unrolling the recurrence of Sec. 5.1 (Softmax-GatedDeltaNet).
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    beta = np.asarray(beta, dtype=np.float64)
    ld = np.asarray(log_decay, dtype=np.float64)
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    gq = head_softmax(q_logits)
    gk = head_softmax(k_logits, (B, T, H))
    S = np.zeros((B, H, dk, dv)) if initial_state is None else np.array(initial_state, dtype=np.float64)
    out = np.zeros((B, T, H, dv))
    for b in range(B):
        for h in range(H):
            S0 = S[b, h].copy()
            for s in range(0, T, chunk):
                e = min(T, s + chunk)
                n = e - s
                K, Q, V = k[b, s:e, h], q[b, s:e, h], v[b, s:e, h]
                bt, gK, gQ = beta[b, s:e, h], gk[b, s:e, h], gq[b, s:e, h]
                c = np.cumsum(ld[b, s:e, h])
                D = np.exp(c[:, None] - c[None, :])  # D[t,j] = e^{c_t - c_j}
                L = np.tril(bt[:, None] * D * (K @ K.T), -1)
                rhs = (bt * gK)[:, None] * V - (bt * np.exp(c))[:, None] * (K @ S0)
                U = np.linalg.solve(np.eye(n) + L, rhs)
                A = np.tril(D * (Q @ K.T))
                out[b, s:e, h] = gQ[:, None] * (np.exp(c)[:, None] * (Q @ S0) + A @ U)
                S0 = np.exp(c[-1]) * S0 + (np.exp(c[-1] - c)[:, None] * K).T @ U
            S[b, h] = S0
    return out, S
