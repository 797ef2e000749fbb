"""Gradients of the SLA forward pass (the three instantiations of Sec. 5.1), fp64 numpy.

TEST INFRASTRUCTURE ONLY: the GPU library never imports this module and shares no code with it.

The training objective reaches the mixer only through its outputs, so the backward pass of the
chunkwise form of Sec. 3.2 (Chunkwise Parallel Training) is, by definition, the derivative of the
recurrence of Eq. 5-6.  ``backward`` is that derivative taken the plain way: reverse-mode
differentiation of the token-by-token recurrence, one token at a time, in the order the recurrence
was run.  With the scalar objective

    L = sum(out * d_out) + sum(final_state * d_final_state)

and, per head, ``S_t = diag(alpha_t) S_{t-1} + G^K_t k_t^T v_t``, ``out_t = G^Q_t q_t S_t``
(alpha_t = gamma_h for RetNet, exp(log_decay_t) for GLA), walking t = T-1 .. 0 with ``dS`` the
gradient with respect to ``S_t``:

    dS      += G^Q_t q_t^T d_out_t
    dG^Q_t   = d_out_t . (q_t S_t)             dq_t = G^Q_t d_out_t S_t^T
    dk_t     = G^K_t dS v_t                    dv_t = G^K_t k_t dS          dG^K_t = k_t dS v_t
    dalpha_t = rowsum(dS * S_{t-1})            dlog_decay_t = alpha_t dalpha_t
    dS       = diag(alpha_t) dS                (now the gradient with respect to S_{t-1})

and the gate gradients go through the head softmax of Eq. 4:
``dlogits = G * (dG - sum_h G dG)``.

Gated delta rule (Softmax-GatedDeltaNet, Sec. 5.1), whose step is, with a scalar decay ``alpha_t`` and write
strength ``beta_t`` per head,

    Sb = alpha_t S_{t-1}       u = beta_t (G^K_t v_t - k_t Sb)       S_t = Sb + k_t^T u

the same walk undoes these three assignments in reverse order:

    du       = k_t dS                  dk_t  = dS u                  (from S_t = Sb + k_t^T u; dSb = dS)
    dbeta_t  = du . (G^K_t v_t - k_t Sb)
    dG^K_t   = beta_t du . v_t         dv_t  = beta_t G^K_t du       w = beta_t du
    dk_t    -= w Sb^T                  dSb  -= k_t^T w               (from the term -beta_t k_t Sb of u)
    dlog_decay_t = sum(dSb * Sb)       dS    = alpha_t dSb           (from Sb = alpha_t S_{t-1})

States are kept at every ``checkpoint``-th token and recomputed in between, so memory stays
bounded at full workload sizes; the arithmetic is the same for every choice of ``checkpoint``.

Layouts as in ``sla_numpy``: q,k [B,T,H,dk]; v, d_out [B,T,H,dv]; logits [B,T,H];
RetNet log_decay [H]; GLA log_decay [B,T,H,dk]; states [B,H,dk,dv].
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np

from .sla_numpy import GDN, GLA, RETNET, head_softmax


def _alpha(variant: int, ld: np.ndarray, t: int) -> np.ndarray:
    """Decay of token t, broadcastable against a state [B,H,dk,dv]."""
    if variant == RETNET:
        return np.exp(ld)[None, :, None, None]
    if variant == GDN:
        return np.exp(ld[:, t])[..., None, None]
    return np.exp(ld[:, t])[..., :, None]


def backward(
    variant: int,
    q,
    k,
    v,
    q_logits,
    k_logits,
    log_decay,
    d_out,
    initial_state=None,
    d_final_state=None,
    checkpoint: int = 64,
    beta=None,
) -> Dict[str, Optional[np.ndarray]]:
    """Gradients of L with respect to every differentiable input.

    Returns a dict with dq, dk, dv, dq_logits, dk_logits (None when ``k_logits`` is None),
    dlog_decay (RetNet: [H]; GLA: [B,T,H,dk]; GDN: [B,T,H]), dbeta (GDN: [B,T,H], else None)
    and dinitial_state.
    """
    if variant not in (RETNET, GLA, GDN):
        raise ValueError(variant)
    if variant == GDN:
        bt = np.asarray(beta, dtype=np.float64)
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    do = np.asarray(d_out, dtype=np.float64)
    ld = np.asarray(log_decay, dtype=np.float64)
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    gq = head_softmax(q_logits)
    gk = head_softmax(k_logits, (B, T, H))

    def step(S, t):
        if variant == GDN:
            Sb = _alpha(variant, ld, t) * S
            u = bt[:, t, :, None] * (gk[:, t, :, None] * v[:, t] - np.einsum("bhd,bhdn->bhn", k[:, t], Sb))
            return Sb + k[:, t][..., :, None] * u[..., None, :]
        return _alpha(variant, ld, t) * S + (gk[:, t, :, None] * k[:, t])[..., :, None] * v[:, t][..., None, :]

    # forward sweep: keep the state entering every checkpoint-th token
    S = np.zeros((B, H, dk, dv)) if initial_state is None else np.array(initial_state, dtype=np.float64)
    kept = {}
    for t in range(T):
        if t % checkpoint == 0:
            kept[t] = S
        S = step(S, t)

    dq = np.zeros_like(q)
    dkk = np.zeros_like(k)
    dvv = np.zeros_like(v)
    dgq = np.zeros((B, T, H))
    dgk = np.zeros((B, T, H))
    dld = np.zeros(H) if variant == RETNET else np.zeros((B, T, H) if variant == GDN else (B, T, H, dk))
    dbt = np.zeros((B, T, H)) if variant == GDN else None
    dS = np.zeros((B, H, dk, dv)) if d_final_state is None else np.array(d_final_state, dtype=np.float64)

    for seg in sorted(kept.keys(), reverse=True):
        end = min(T, seg + checkpoint)
        before = [kept[seg]]  # before[i] = state entering token seg + i
        for t in range(seg, end):
            before.append(step(before[-1], t))
        for t in range(end - 1, seg - 1, -1):
            S_prev, S_t = before[t - seg], before[t - seg + 1]
            y = np.einsum("bhd,bhdn->bhn", q[:, t], S_t)
            dgq[:, t] = np.sum(do[:, t] * y, axis=-1)
            dy = gq[:, t, :, None] * do[:, t]
            dq[:, t] = np.einsum("bhn,bhdn->bhd", dy, S_t)
            dS = dS + q[:, t][..., :, None] * dy[..., None, :]
            if variant == GDN:
                a = _alpha(variant, ld, t)
                Sb = a * S_prev
                resid = gk[:, t, :, None] * v[:, t] - np.einsum("bhd,bhdn->bhn", k[:, t], Sb)
                u = bt[:, t, :, None] * resid
                du = np.einsum("bhd,bhdn->bhn", k[:, t], dS)
                dbt[:, t] = np.sum(du * resid, axis=-1)
                dgk[:, t] = bt[:, t] * np.sum(du * v[:, t], axis=-1)
                dvv[:, t] = (bt[:, t] * gk[:, t])[..., None] * du
                w = bt[:, t, :, None] * du
                dkk[:, t] = np.einsum("bhdn,bhn->bhd", dS, u) - np.einsum("bhn,bhdn->bhd", w, Sb)
                dSb = dS - k[:, t][..., :, None] * w[..., None, :]
                dld[:, t] = np.sum(dSb * Sb, axis=(-1, -2))
                dS = a * dSb
                continue
            dSv = np.einsum("bhdn,bhn->bhd", dS, v[:, t])
            dkk[:, t] = gk[:, t, :, None] * dSv
            dvv[:, t] = gk[:, t, :, None] * np.einsum("bhd,bhdn->bhn", k[:, t], dS)
            dgk[:, t] = np.sum(k[:, t] * dSv, axis=-1)
            a = _alpha(variant, ld, t)
            dalpha = np.sum(dS * S_prev, axis=-1)  # [B,H,dk]
            if variant == RETNET:
                dld += np.exp(ld) * np.sum(dalpha, axis=(0, 2))
            else:
                dld[:, t] = a[..., 0] * dalpha
            dS = a * dS

    def softmax_backward(g, dg):
        return g * (dg - np.sum(g * dg, axis=-1, keepdims=True))

    return {
        "dq": dq,
        "dk": dkk,
        "dv": dvv,
        "dq_logits": softmax_backward(gq, dgq),
        "dk_logits": None if k_logits is None else softmax_backward(gk, dgk),
        "dlog_decay": dld,
        "dbeta": dbt,
        "dinitial_state": dS,
    }
