"""Seeded synthetic inputs for the SLA chunked-forward path.

This module only *draws* numbers.  It holds none of the method's arithmetic
(no softmax over heads, no recurrence, no decay products): both the CPU
oracle's tests and the GPU tests/benchmark import it so that the two sides
see bit-identical arrays, and neither side imports the other.

The shapes and distributions stand in for the paper's workloads (language
modelling at sequence length 2K-4K, Sec. 5.2 "Model Configuration" /
"Training Details", and long-context retrieval, Sec. 5.3): no item of any
dataset is used anywhere.

Conventions
-----------
* Layouts: q, k ``[B,T,H,dk]``; v ``[B,T,H,dv]``; head-gate logits ``[B,T,H]``;
  RetNet log-decay ``[H]``; GLA log-decay ``[B,T,H,dk]``; GDN log-decay and
  beta ``[B,T,H]``.
* Every array is returned as float32.  When ``dtype == "bf16"`` the arrays the
  kernel consumes in bf16 (q, k, v and the GLA log-decay) are already rounded
  to bf16 (round-to-nearest-even), so widening them is exact and the oracle and
  the kernel consume identical values.
* Draw order is fixed: q, k, v, q_logits, k_logits, log_decay, beta.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, Optional

import numpy as np

RETNET, GLA, GDN = 0, 1, 2
VARIANT_NAMES = {RETNET: "retnet", GLA: "gla", GDN: "gdn"}

SEED_BASE = 20260200


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); return float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits of float32 values that are already bf16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    if np.any(bits & np.uint32(0xFFFF)):
        raise ValueError("array holds values that are not bf16-representable")
    return (bits >> np.uint32(16)).astype(np.uint16)


def _logsigmoid(x: np.ndarray) -> np.ndarray:
    # log(sigmoid(x)) = -log1p(exp(-x)), written to stay finite for large |x|.
    x = x.astype(np.float64)
    return -(np.maximum(-x, 0.0) + np.log1p(np.exp(-np.abs(x))))


@dataclasses.dataclass
class Workload:
    """One named configuration of the benchmark/test matrix."""

    name: str
    variant: int
    dtype: str  # "f32" | "bf16"
    B: int
    T: int
    H: int
    dk: int
    dv: int
    seed: int
    qk_prep: str = "scale"  # "scale": multiply q,k by dk**-0.5 ; "l2": L2-normalise q,k
    logit_std: float = 1.0
    decay_div: float = 16.0
    decay_shift: float = 0.0
    peaked_segment: int = 0  # >0: one random head per segment of this many tokens gets +6
    dual_gates: bool = True

    def tokens(self) -> int:
        return self.B * self.T


# The five configurations of the benchmark definition, in its order.
def workload(name: str) -> Workload:
    table = {
        "gla_tiny": Workload("gla_tiny", GLA, "f32", 1, 256, 4, 64, 64, SEED_BASE + 0),
        "retnet": Workload("retnet", RETNET, "bf16", 4, 2048, 8, 128, 128, SEED_BASE + 1, logit_std=2.0),
        "gla_train": Workload("gla_train", GLA, "bf16", 8, 2048, 16, 128, 128, SEED_BASE + 2),
        "gdn": Workload("gdn", GDN, "bf16", 8, 4096, 16, 128, 128, SEED_BASE + 3, qk_prep="l2", decay_div=8.0),
        "gla_long": Workload(
            "gla_long", GLA, "bf16", 1, 65536, 32, 128, 128, SEED_BASE + 4, decay_shift=2.0, peaked_segment=512
        ),
        # Same shape as the headline configuration for the two other variants.
        "retnet_train": Workload("retnet_train", RETNET, "bf16", 8, 2048, 16, 128, 128, SEED_BASE + 5),
        "gdn_train": Workload(
            "gdn_train", GDN, "bf16", 8, 2048, 16, 128, 128, SEED_BASE + 6, qk_prep="l2", decay_div=8.0
        ),
        # The paper's 340M-class model shapes (Sec. 5.2 "Model Configuration": hidden 1024, few wide heads; GLA keys
        # at half width) at its training length, and the H = 8 point of its head ablation at the same width.
        "gla_paper_h4": Workload("gla_paper_h4", GLA, "bf16", 8, 4096, 4, 128, 256, SEED_BASE + 10),
        "gla_paper_h8": Workload("gla_paper_h8", GLA, "bf16", 8, 4096, 8, 64, 128, SEED_BASE + 11),
        # ... and its H = 16 point (Sec. 5.6: the gain of the head competition grows with the head count): keys of
        # width 32, values of width 64.
        "gla_paper_h16": Workload("gla_paper_h16", GLA, "bf16", 8, 4096, 16, 32, 64, SEED_BASE + 12),
        # The same 4-head, 4K-token, batch-8 regime for the two other variants (32 sequences: the few-sequence case).
        # Their reference models use key heads of width 256, which the kernels do not tile; keys are taken at width
        # 128 as for GLA, values at 256.
        "retnet_paper_h4": Workload("retnet_paper_h4", RETNET, "bf16", 8, 4096, 4, 128, 256, SEED_BASE + 13),
        "gdn_paper_h4": Workload(
            "gdn_paper_h4", GDN, "bf16", 8, 4096, 4, 128, 256, SEED_BASE + 14, qk_prep="l2", decay_div=8.0
        ),
        # One decode step (T = 1) over a serving-sized batch: the recurrent form, one token per sequence.
        "decode_gla": Workload("decode_gla", GLA, "bf16", 64, 1, 16, 128, 128, SEED_BASE + 7),
        "decode_retnet": Workload("decode_retnet", RETNET, "bf16", 64, 1, 16, 128, 128, SEED_BASE + 8),
        "decode_gdn": Workload(
            "decode_gdn", GDN, "bf16", 64, 1, 16, 128, 128, SEED_BASE + 9, qk_prep="l2", decay_div=8.0
        ),
    }
    return dataclasses.replace(table[name])


WORKLOAD_NAMES = ("gla_tiny", "retnet", "gla_train", "gdn", "gla_long", "retnet_train", "gdn_train", "gla_paper_h4",
                  "gla_paper_h8", "gla_paper_h16", "retnet_paper_h4", "gdn_paper_h4")
DECODE_WORKLOAD_NAMES = ("decode_gla", "decode_retnet", "decode_gdn")


def _normal(rng: np.random.Generator, shape) -> np.ndarray:
    return rng.standard_normal(size=shape, dtype=np.float32)


def generate(w: Workload, *, T: Optional[int] = None, B: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Draw the arrays of workload ``w``.

    ``T``/``B`` override the sizes (used to cut a bounded sample of a large
    workload); the stream of random numbers then differs from the full-size
    draw, which is fine because both sides always consume the same call.
    """
    B = w.B if B is None else B
    T = w.T if T is None else T
    H, dk, dv = w.H, w.dk, w.dv
    rng = np.random.default_rng(w.seed)
    narrow = w.dtype == "bf16"

    q = _normal(rng, (B, T, H, dk))
    k = _normal(rng, (B, T, H, dk))
    v = _normal(rng, (B, T, H, dv))
    if w.qk_prep == "scale":
        s = np.float32(dk ** -0.5)
        q *= s
        k *= s
    elif w.qk_prep == "l2":
        q /= np.sqrt(np.sum(q.astype(np.float64) ** 2, axis=-1, keepdims=True)).astype(np.float32)
        k /= np.sqrt(np.sum(k.astype(np.float64) ** 2, axis=-1, keepdims=True)).astype(np.float32)
    else:
        raise ValueError(w.qk_prep)

    q_logits = _normal(rng, (B, T, H)) * np.float32(w.logit_std)
    k_logits = _normal(rng, (B, T, H)) * np.float32(w.logit_std)
    if w.peaked_segment > 0:
        nseg = (T + w.peaked_segment - 1) // w.peaked_segment
        winners = rng.integers(0, H, size=(B, nseg))
        tok_seg = np.arange(T) // w.peaked_segment
        bump = np.zeros((B, T, H), dtype=np.float32)
        bump[np.arange(B)[:, None], np.arange(T)[None, :], winners[:, tok_seg]] = 6.0
        q_logits += bump
        k_logits += bump

    beta = None
    if w.variant == RETNET:
        gamma = 1.0 - 2.0 ** (-5.0 - np.arange(H, dtype=np.float64))
        log_decay = np.log(gamma).astype(np.float32)
    elif w.variant == GLA:
        x = _normal(rng, (B, T, H, dk)) + np.float32(w.decay_shift)
        log_decay = (_logsigmoid(x) / w.decay_div).astype(np.float32)
    elif w.variant == GDN:
        x = _normal(rng, (B, T, H)) + np.float32(w.decay_shift)
        log_decay = (_logsigmoid(x) / w.decay_div).astype(np.float32)
        xb = _normal(rng, (B, T, H)).astype(np.float64)
        beta = (1.0 / (1.0 + np.exp(-xb))).astype(np.float32)
    else:
        raise ValueError(w.variant)

    if narrow:
        q, k, v = round_to_bf16(q), round_to_bf16(k), round_to_bf16(v)
        if w.variant == GLA:
            log_decay = round_to_bf16(log_decay)

    out = {
        "q": q,
        "k": k,
        "v": v,
        "q_logits": np.ascontiguousarray(q_logits, dtype=np.float32),
        "k_logits": np.ascontiguousarray(k_logits, dtype=np.float32) if w.dual_gates else None,
        "log_decay": np.ascontiguousarray(log_decay, dtype=np.float32),
        "beta": beta,
    }
    return out


def custom(
    variant: int,
    dtype: str,
    B: int,
    T: int,
    H: int,
    dk: int,
    dv: int,
    seed: int,
    **kw,
) -> Dict[str, np.ndarray]:
    """Draw a free-form case (edge shapes in the parity tests)."""
    qk_prep = kw.pop("qk_prep", "l2" if variant == GDN else "scale")
    decay_div = kw.pop("decay_div", 8.0 if variant == GDN else 16.0)
    w = Workload("custom", variant, dtype, B, T, H, dk, dv, seed, qk_prep=qk_prep, decay_div=decay_div, **kw)
    return generate(w)


def initial_state(B: int, H: int, dk: int, dv: int, seed: int, scale: float = 0.5) -> np.ndarray:
    """A random fp32 entry state ``[B,H,dk,dv]`` for the chaining tests."""
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(size=(B, H, dk, dv), dtype=np.float32) * np.float32(scale)).astype(np.float32)


def cotangents(B: int, T: int, H: int, dk: int, dv: int, seed: int, dtype: str = "bf16",
               final_state: bool = False) -> Dict[str, Optional[np.ndarray]]:
    """Seeded cotangents for the backward pass: ``d_out [B,T,H,dv]`` ~ N(0,1) (rounded to bf16 when the
    workload is bf16) and, when asked for, ``d_final_state [B,H,dk,dv]`` ~ N(0, 0.25) in fp32."""
    rng = np.random.default_rng(seed)
    d_out = rng.standard_normal(size=(B, T, H, dv), dtype=np.float32)
    if dtype == "bf16":
        d_out = round_to_bf16(d_out)
    dsf = None
    if final_state:
        dsf = (rng.standard_normal(size=(B, H, dk, dv), dtype=np.float32) * np.float32(0.5)).astype(np.float32)
    return {"d_out": np.ascontiguousarray(d_out, dtype=np.float32), "d_final_state": dsf}


def gate_weights(H: int, dk: int, seed: int) -> Dict[str, np.ndarray]:
    """Seeded gate matrices of Sec. 3.2 as ``[H,dk]`` fp32 (row h = column h of W_GQ / W_GK), N(0,1): with q, k
    of variance 1/dk per element the logits come out with unit variance, as the workloads' logits have."""
    rng = np.random.default_rng(seed)
    return {"w_gq": rng.standard_normal(size=(H, dk), dtype=np.float32),
            "w_gk": rng.standard_normal(size=(H, dk), dtype=np.float32)}


def packed_lengths(total: int, seed: int, longest: int = 4096, shortest: int = 64) -> np.ndarray:
    """A seeded mix of sequence lengths that sums to ``total``: powers of two between ``shortest`` and
    ``longest`` drawn with probability proportional to 1/length until the budget is used, the remainder as one last
    sequence; sorted longest first.  Stands in for packing documents of mixed length into a 2K-8K token budget
    (Sec. 5.2 trains on 4K contexts, Sec. 5.3 evaluates 1K-8K)."""
    rng = np.random.default_rng(seed)
    sizes = []
    s = shortest
    while s <= longest:
        sizes.append(s)
        s *= 2
    sizes = np.array(sizes)
    prob = (1.0 / sizes) / np.sum(1.0 / sizes)
    out, left = [], int(total)
    while left > 0:
        n = int(rng.choice(sizes, p=prob))
        n = min(n, left)
        out.append(n)
        left -= n
    return np.array(sorted(out, reverse=True), dtype=np.int32)


def to_device(d: Dict[str, np.ndarray], dtype: str, variant: int):
    """The generated arrays as torch tensors on cuda:0 (marshalling only: bf16 workloads hold bf16-representable
    values, which is asserted, so narrowing them changes nothing).  Returns (dict of tensors, torch dtype)."""
    import torch

    dev = torch.device("cuda:0")
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32

    def t(a, narrow):
        if a is None:
            return None
        x = torch.from_numpy(np.ascontiguousarray(a))
        if narrow and dtype == "bf16":
            y = x.to(torch.bfloat16)
            assert torch.equal(y.to(torch.float32), x), "inputs must be bf16-representable"
            x = y
        return x.to(dev).contiguous()

    return dict(
        q=t(d["q"], True), k=t(d["k"], True), v=t(d["v"], True),
        q_logits=t(d["q_logits"], False), k_logits=t(d["k_logits"], False),
        log_decay=t(d["log_decay"], variant == GLA), beta=t(d["beta"], False),
    ), tdt
