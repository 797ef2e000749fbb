"""CPU oracle for the SLA forward pass — test infrastructure, not product code.

``forward``      – the plain-C fp64 token-by-token recurrence (``sla_oracle.c``),
                   loaded through ctypes; the function the GPU library is
                   compared against and the one timed as the CPU baseline.
``sla_numpy``    – independent numpy statements used to pin it.
``sla_backward`` – gradients of the recurrence (RetNet, GLA) by reverse-mode
                   differentiation token by token, fp64 numpy; pinned by finite
                   differences and by autograd through the parallel form.

``backward``     – the same gradients in plain C (``sla_oracle_backward.c``, OpenMP over (batch, head)), pinned
                   against ``sla_backward``; fast enough for whole workloads.
``sla_prologue`` – gate projections, short convolution + SiLU (+ L2 normalisation) and their
                   backward, fp64 numpy; pinned by finite differences and library autograd.

Nothing under the GPU package imports this package; only ``tests/``, the smoke
check and the benchmark's cpu_baseline leg do.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

from . import sla_backward, sla_numpy, sla_prologue  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sla_oracle.c")
_SRC_BWD = os.path.join(_HERE, "sla_oracle_backward.c")
_LIB = os.path.join(_HERE, "libsla_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile ``sla_oracle.c`` and ``sla_oracle_backward.c`` with gcc (-O2, OpenMP) into this directory."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_BWD))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, _SRC_BWD, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        fp = ctypes.POINTER(ctypes.c_float)
        dp = ctypes.POINTER(ctypes.c_double)
        lib.sla_oracle_forward.restype = ctypes.c_int
        lib.sla_oracle_forward.argtypes = [ctypes.c_int] * 6 + [fp] * 8 + [dp, dp, ctypes.c_int]
        lib.sla_oracle_backward.restype = ctypes.c_int
        lib.sla_oracle_backward.argtypes = [ctypes.c_int] * 6 + [fp] * 10 + [dp] * 8 + [ctypes.c_int]
        lib.sla_oracle_threads.restype = ctypes.c_int
        lib.sla_oracle_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def threads(requested: int = 0) -> int:
    """Threads the C oracle's (batch, head) loop will use."""
    return int(_load().sla_oracle_threads(int(requested)))


def _f32(a) -> Optional[np.ndarray]:
    if a is None:
        return None
    return np.ascontiguousarray(a, dtype=np.float32)


def _ptr(a, ty):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ty))


def forward(
    variant: int,
    q,
    k,
    v,
    q_logits,
    k_logits,
    log_decay,
    beta=None,
    initial_state=None,
    nthreads: int = 0,
) -> Tuple[np.ndarray, np.ndarray]:
    """Run the C oracle.  Inputs are float32 arrays; returns fp64 (out, final_state)."""
    lib = _load()
    q, k, v = _f32(q), _f32(k), _f32(v)
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    assert k.shape == (B, T, H, dk) and v.shape == (B, T, H, dv)
    ql, kl = _f32(q_logits), _f32(k_logits)
    assert ql.shape == (B, T, H) and (kl is None or kl.shape == (B, T, H))
    ld, bt, s0 = _f32(log_decay), _f32(beta), _f32(initial_state)
    want = {0: (H,), 1: (B, T, H, dk), 2: (B, T, H)}[variant]
    assert ld.shape == want, (ld.shape, want)
    assert bt is None or bt.shape == (B, T, H)
    assert s0 is None or s0.shape == (B, H, dk, dv)
    out = np.empty((B, T, H, dv), dtype=np.float64)
    fin = np.empty((B, H, dk, dv), dtype=np.float64)
    rc = lib.sla_oracle_forward(
        variant, B, T, H, dk, dv,
        _ptr(q, ctypes.c_float), _ptr(k, ctypes.c_float), _ptr(v, ctypes.c_float),
        _ptr(ql, ctypes.c_float), _ptr(kl, ctypes.c_float), _ptr(ld, ctypes.c_float),
        _ptr(bt, ctypes.c_float), _ptr(s0, ctypes.c_float),
        _ptr(out, ctypes.c_double), _ptr(fin, ctypes.c_double), int(nthreads),
    )
    if rc != 0:
        raise RuntimeError(f"sla_oracle_forward failed with code {rc}")
    return out, fin


def backward(variant: int, q, k, v, q_logits, k_logits, log_decay, d_out, initial_state=None, d_final_state=None,
             beta=None, nthreads: int = 0):
    """Gradients of the forward by the C oracle (``sla_oracle_backward.c``).  Same conventions and the same dict of
    fp64 results as ``sla_backward.backward``."""
    lib = _load()
    q, k, v, do = _f32(q), _f32(k), _f32(v), _f32(d_out)
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    ql, kl, ld, bt = _f32(q_logits), _f32(k_logits), _f32(log_decay), _f32(beta)
    s0, dsf = _f32(initial_state), _f32(d_final_state)
    want = {0: (H,), 1: (B, T, H, dk), 2: (B, T, H)}[variant]
    assert ld.shape == want and do.shape == v.shape
    z = lambda *shape: np.zeros(shape, dtype=np.float64)
    res = {
        "dq": z(B, T, H, dk), "dk": z(B, T, H, dk), "dv": z(B, T, H, dv), "dq_logits": z(B, T, H),
        "dk_logits": None if kl is None else z(B, T, H), "dlog_decay": z(*want),
        "dbeta": z(B, T, H) if variant == 2 else None, "dinitial_state": z(B, H, dk, dv),
    }
    f, d = ctypes.c_float, ctypes.c_double
    rc = lib.sla_oracle_backward(
        variant, B, T, H, dk, dv, _ptr(q, f), _ptr(k, f), _ptr(v, f), _ptr(ql, f), _ptr(kl, f), _ptr(ld, f), _ptr(bt, f),
        _ptr(s0, f), _ptr(do, f), _ptr(dsf, f), _ptr(res["dq"], d), _ptr(res["dk"], d), _ptr(res["dv"], d),
        _ptr(res["dq_logits"], d), _ptr(res["dk_logits"], d), _ptr(res["dlog_decay"], d), _ptr(res["dbeta"], d),
        _ptr(res["dinitial_state"], d), int(nthreads))
    if rc != 0:
        raise RuntimeError(f"sla_oracle_backward failed with code {rc}")
    return res
