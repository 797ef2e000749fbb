"""ctypes binding for libsla.so: argument marshalling only.

The functions ``sla_*`` mirror the C ABI one to one (raw integer addresses in,
status code out).  ``forward`` is the convenience wrapper the tests and the
benchmark use: it takes torch CUDA tensors, allocates the outputs with torch and
passes ``data_ptr()``s and the current stream to ``sla_forward``.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

RETNET, GLA, GDN = 0, 1, 2
FLAG_HEAD_MAJOR = 1
F32, BF16 = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsla.so")
_lib = None


class SlaError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"libsla: {text} (status {status})")
        self.status = status


class SlaParams(ctypes.Structure):
    _fields_ = [
        ("variant", ctypes.c_int32),
        ("dtype", ctypes.c_int32),
        ("B", ctypes.c_int32),
        ("T", ctypes.c_int32),
        ("H", ctypes.c_int32),
        ("dk", ctypes.c_int32),
        ("dv", ctypes.c_int32),
        ("dv_split", ctypes.c_int32),
        ("flags", ctypes.c_int32),
        ("segments", ctypes.c_int32),
    ]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libsla.so; raises if it has not been built (there is no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2602_01744_amd.build` "
            "(or __graft_entry__.build()); there is no CPU fallback"
        )
    lib = ctypes.CDLL(_LIB_PATH)
    vp = ctypes.c_void_p
    pp = ctypes.POINTER(SlaParams)
    lib.sla_forward.restype = ctypes.c_int
    lib.sla_forward.argtypes = [pp] + [vp] * 11
    lib.sla_forward_ws.restype = ctypes.c_int
    lib.sla_forward_ws.argtypes = [pp] + [vp] * 11 + [ctypes.c_size_t, vp]
    lib.sla_forward_static.restype = ctypes.c_int
    lib.sla_forward_static.argtypes = [pp] + [vp] * 11
    lib.sla_device_status.restype = ctypes.c_int
    lib.sla_device_status.argtypes = [ctypes.POINTER(ctypes.c_uint32), ctypes.c_int, vp]
    lib.sla_init.restype = ctypes.c_int
    lib.sla_init.argtypes = []
    lib.sla_static_scratch_bytes.restype = ctypes.c_size_t
    lib.sla_static_scratch_bytes.argtypes = []
    lib.sla_decode_step.restype = ctypes.c_int
    lib.sla_decode_step.argtypes = [pp] + [vp] * 10
    lib.sla_decode_step_fused.restype = ctypes.c_int
    lib.sla_decode_step_fused.argtypes = [pp] + [vp] * 10
    lib.sla_forward_varlen.restype = ctypes.c_int
    lib.sla_forward_varlen.argtypes = [pp] + [vp] * 12
    lib.sla_backward_varlen.restype = ctypes.c_int
    lib.sla_backward_varlen.argtypes = [pp] + [vp] * 18 + [ctypes.c_size_t, vp]
    lib.sla_backward_varlen_workspace_bytes.restype = ctypes.c_size_t
    lib.sla_backward_varlen_workspace_bytes.argtypes = [pp]
    lib.sla_short_conv_silu.restype = ctypes.c_int
    lib.sla_short_conv_silu.argtypes = [ctypes.c_int] * 5 + [vp] * 4
    lib.sla_short_conv_silu_l2.restype = ctypes.c_int
    lib.sla_short_conv_silu_l2.argtypes = [ctypes.c_int] * 6 + [ctypes.c_float] + [vp] * 4
    lib.sla_short_conv_silu_l2_backward.restype = ctypes.c_int
    lib.sla_short_conv_silu_l2_backward.argtypes = [ctypes.c_int] * 6 + [ctypes.c_float] + [vp] * 6 + [ctypes.c_size_t, vp]
    lib.sla_short_conv_silu_l2_backward_workspace_bytes.restype = ctypes.c_size_t
    lib.sla_short_conv_silu_l2_backward_workspace_bytes.argtypes = [ctypes.c_int] * 4
    lib.sla_gate_logits_backward.restype = ctypes.c_int
    lib.sla_gate_logits_backward.argtypes = [pp] + [vp] * 6 + [ctypes.c_size_t, vp]
    lib.sla_gate_logits_backward_workspace_bytes.restype = ctypes.c_size_t
    lib.sla_gate_logits_backward_workspace_bytes.argtypes = [pp]
    lib.sla_gate_logits.restype = ctypes.c_int
    lib.sla_gate_logits.argtypes = [pp] + [vp] * 7
    lib.sla_backward.restype = ctypes.c_int
    lib.sla_backward.argtypes = [pp] + [vp] * 17 + [ctypes.c_size_t, vp]
    lib.sla_backward_gdn.restype = ctypes.c_int
    lib.sla_backward_gdn.argtypes = [pp] + [vp] * 19 + [ctypes.c_size_t, vp]
    lib.sla_backward_gdn_workspace_bytes.restype = ctypes.c_size_t
    lib.sla_backward_gdn_workspace_bytes.argtypes = [pp]
    lib.sla_backward_gdn_varlen.restype = ctypes.c_int
    lib.sla_backward_gdn_varlen.argtypes = [pp] + [vp] * 20 + [ctypes.c_size_t, vp]
    lib.sla_backward_gdn_varlen_workspace_bytes.restype = ctypes.c_size_t
    lib.sla_backward_gdn_varlen_workspace_bytes.argtypes = [pp]
    lib.sla_backward_workspace_bytes.restype = ctypes.c_size_t
    lib.sla_backward_workspace_bytes.argtypes = [pp]
    lib.sla_workspace_bytes.restype = ctypes.c_size_t
    lib.sla_workspace_bytes.argtypes = [pp, ctypes.c_int]
    lib.sla_segments.restype = ctypes.c_int
    lib.sla_segments.argtypes = [pp, ctypes.c_int]
    lib.sla_backward_segments.restype = ctypes.c_int
    lib.sla_backward_segments.argtypes = [pp, ctypes.c_int]
    lib.sla_check_args.restype = ctypes.c_int
    lib.sla_check_args.argtypes = [pp] + [vp] * 10
    lib.sla_default_dv_split.restype = ctypes.c_int
    lib.sla_default_dv_split.argtypes = [pp, ctypes.c_int]
    lib.sla_kernel_name.restype = ctypes.c_char_p
    lib.sla_kernel_name.argtypes = [pp]
    lib.sla_status_string.restype = ctypes.c_char_p
    lib.sla_status_string.argtypes = [ctypes.c_int]
    lib.sla_version.restype = ctypes.c_int
    lib.sla_version.argtypes = []
    _lib = lib
    return lib


def _p(x) -> Optional[int]:
    return None if not x else int(x)


def sla_status_string(status: int) -> str:
    return load_library().sla_status_string(int(status)).decode()


def sla_version() -> int:
    return int(load_library().sla_version())


def sla_default_dv_split(params: SlaParams, compute_units: int) -> int:
    return int(load_library().sla_default_dv_split(ctypes.byref(params), int(compute_units)))


def sla_workspace_bytes(params: SlaParams, compute_units: int) -> int:
    return int(load_library().sla_workspace_bytes(ctypes.byref(params), int(compute_units)))


def sla_segments(params: SlaParams, compute_units: int) -> int:
    return int(load_library().sla_segments(ctypes.byref(params), int(compute_units)))


def sla_backward_segments(params: SlaParams, compute_units: int) -> int:
    pr = ctypes.byref(params) if params is not None else None
    return int(load_library().sla_backward_segments(pr, int(compute_units)))


def sla_kernel_name(params: SlaParams) -> Optional[str]:
    s = load_library().sla_kernel_name(ctypes.byref(params))
    return None if s is None else s.decode()


def sla_check_args(params, q, k, v, q_head_logits, k_head_logits, log_decay, beta, initial_state, out, final_state) -> int:
    """Raw call: integer addresses (0/None = NULL).  Returns the status code."""
    pr = ctypes.byref(params) if params is not None else None
    return int(
        load_library().sla_check_args(
            pr, _p(q), _p(k), _p(v), _p(q_head_logits), _p(k_head_logits), _p(log_decay), _p(beta),
            _p(initial_state), _p(out), _p(final_state),
        )
    )


def sla_forward(params, q, k, v, q_head_logits, k_head_logits, log_decay, beta, initial_state, out, final_state,
                stream) -> int:
    """Raw call: integer device addresses (0/None = NULL) and a hipStream_t handle.  Returns the status code."""
    pr = ctypes.byref(params) if params is not None else None
    return int(
        load_library().sla_forward(
            pr, _p(q), _p(k), _p(v), _p(q_head_logits), _p(k_head_logits), _p(log_decay), _p(beta),
            _p(initial_state), _p(out), _p(final_state), _p(stream),
        )
    )


def sla_forward_ws(params, q, k, v, q_head_logits, k_head_logits, log_decay, beta, initial_state, out, final_state,
                   workspace, workspace_bytes, stream) -> int:
    """Raw call of the workspace-taking entry point (same conventions as sla_forward)."""
    pr = ctypes.byref(params) if params is not None else None
    return int(
        load_library().sla_forward_ws(
            pr, _p(q), _p(k), _p(v), _p(q_head_logits), _p(k_head_logits), _p(log_decay), _p(beta),
            _p(initial_state), _p(out), _p(final_state), _p(workspace), int(workspace_bytes), _p(stream),
        )
    )


def sla_init() -> int:
    return int(load_library().sla_init())


DEVICE_WAIT_EXPIRED, DEVICE_DECAY_RANGE = 1, 2


def sla_device_status(reset: bool = False, stream=None):
    """Returns (status code, device status word) of the current device; waits for ``stream`` first."""
    word = ctypes.c_uint32(0)
    rc = int(load_library().sla_device_status(ctypes.byref(word), int(bool(reset)), _p(stream)))
    return rc, int(word.value)


def sla_static_scratch_bytes() -> int:
    return int(load_library().sla_static_scratch_bytes())


def sla_forward_static(params, q, k, v, q_head_logits, k_head_logits, log_decay, beta, initial_state, out,
                       final_state, stream) -> int:
    """Raw call of the entry point that allocates nothing (same conventions as sla_forward)."""
    pr = ctypes.byref(params) if params is not None else None
    return int(
        load_library().sla_forward_static(
            pr, _p(q), _p(k), _p(v), _p(q_head_logits), _p(k_head_logits), _p(log_decay), _p(beta),
            _p(initial_state), _p(out), _p(final_state), _p(stream),
        )
    )


def sla_decode_step(params, q, k, v, q_head_logits, k_head_logits, log_decay, beta, state, out, stream) -> int:
    """Raw call of the decode entry point (same conventions as sla_forward)."""
    pr = ctypes.byref(params) if params is not None else None
    return int(
        load_library().sla_decode_step(
            pr, _p(q), _p(k), _p(v), _p(q_head_logits), _p(k_head_logits), _p(log_decay), _p(beta), _p(state),
            _p(out), _p(stream),
        )
    )


def sla_decode_step_fused(params, q, k, v, w_gq, w_gk, log_decay, beta, state, out, stream) -> int:
    """Raw call of the decode entry point that forms the gate logits itself."""
    pr = ctypes.byref(params) if params is not None else None
    return int(
        load_library().sla_decode_step_fused(
            pr, _p(q), _p(k), _p(v), _p(w_gq), _p(w_gk), _p(log_decay), _p(beta), _p(state), _p(out), _p(stream),
        )
    )


def sla_forward_varlen(params, q, k, v, q_head_logits, k_head_logits, log_decay, beta, cu_seqlens, initial_state, out,
                       final_state, stream) -> int:
    """Raw call of the packed variable-length forward (same conventions as sla_forward)."""
    pr = ctypes.byref(params) if params is not None else None
    return int(load_library().sla_forward_varlen(
        pr, _p(q), _p(k), _p(v), _p(q_head_logits), _p(k_head_logits), _p(log_decay), _p(beta), _p(cu_seqlens),
        _p(initial_state), _p(out), _p(final_state), _p(stream)))


def sla_backward_varlen_workspace_bytes(params: SlaParams) -> int:
    return int(load_library().sla_backward_varlen_workspace_bytes(ctypes.byref(params)))


def sla_backward_varlen(params, q, k, v, q_head_logits, k_head_logits, log_decay, cu_seqlens, initial_state, d_out,
                        d_final_state, dq, dk, dv, dq_head_logits, dk_head_logits, dlog_decay, d_initial_state,
                        workspace, workspace_bytes, stream) -> int:
    """Raw call of the packed variable-length backward (same conventions as sla_backward)."""
    pr = ctypes.byref(params) if params is not None else None
    return int(load_library().sla_backward_varlen(
        pr, _p(q), _p(k), _p(v), _p(q_head_logits), _p(k_head_logits), _p(log_decay), _p(cu_seqlens),
        _p(initial_state), _p(d_out), _p(d_final_state), _p(dq), _p(dk), _p(dv), _p(dq_head_logits),
        _p(dk_head_logits), _p(dlog_decay), _p(d_initial_state), _p(workspace), int(workspace_bytes), _p(stream)))


def forward_varlen(variant: int, q, k, v, q_head_logits, k_head_logits, log_decay, beta, cu_seqlens,
                   initial_state=None, *, want_final_state: bool = True):
    """Packed sequences: q, k [T,H,dk], v [T,H,dv], logits (beta, GDN decay) [T,H], cu_seqlens int32 [B+1] on the
    device, initial_state [B,H,dk,dv] or None.  Returns (out [T,H,dv], final_state [B,H,dk,dv] or None)."""
    import torch

    assert q.is_cuda and q.is_contiguous() and k.is_contiguous() and v.is_contiguous()
    T, H, dk = q.shape
    dv = v.shape[-1]
    assert cu_seqlens.is_cuda and cu_seqlens.dtype == torch.int32 and cu_seqlens.dim() == 1 and cu_seqlens.is_contiguous()
    B = cu_seqlens.numel() - 1
    dtype = {torch.float32: F32, torch.bfloat16: BF16}[q.dtype]
    out = torch.empty((T, H, dv), dtype=q.dtype, device=q.device)
    fin = torch.empty((B, H, dk, dv), dtype=torch.float32, device=q.device) if want_final_state else None
    params = SlaParams(variant, dtype, B, T, H, dk, dv, 0, 0, 1)
    ptr = lambda t: None if t is None else t.data_ptr()
    rc = sla_forward_varlen(params, ptr(q), ptr(k), ptr(v), ptr(q_head_logits), ptr(k_head_logits), ptr(log_decay),
                            ptr(beta), ptr(cu_seqlens), ptr(initial_state), ptr(out), ptr(fin),
                            torch.cuda.current_stream(q.device).cuda_stream)
    if rc != 0:
        raise SlaError(rc, sla_status_string(rc))
    return out, fin


def backward_varlen(variant: int, q, k, v, q_head_logits, k_head_logits, log_decay, d_out, cu_seqlens,
                    initial_state=None, d_final_state=None, *, want_d_initial_state: bool = False):
    """Gradients of ``forward_varlen`` (RetNet, GLA; bfloat16 or float32); tensors packed as there.  Returns a dict
    as ``backward`` does, with d_initial_state [B,H,dk,dv]."""
    import torch

    assert q.is_cuda and q.dtype in (torch.bfloat16, torch.float32)
    T, H, dk = q.shape
    dv = v.shape[-1]
    B = cu_seqlens.numel() - 1
    dev = q.device
    g = {
        "dq": torch.empty_like(q),
        "dk": torch.empty_like(k),
        "dv": torch.empty_like(v),
        "dq_head_logits": torch.empty_like(q_head_logits),
        "dk_head_logits": None if k_head_logits is None else torch.empty_like(k_head_logits),
        "dlog_decay": torch.empty_like(log_decay) if variant == GLA else None,
        "d_initial_state": torch.empty((B, H, dk, dv), dtype=torch.float32, device=dev) if want_d_initial_state else None,
    }
    params = SlaParams(variant, BF16 if q.dtype == torch.bfloat16 else F32, B, T, H, dk, dv, 0, 0, 1)
    need = sla_backward_varlen_workspace_bytes(params)
    workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    ptr = lambda t: None if t is None else t.data_ptr()
    rc = sla_backward_varlen(
        params, ptr(q), ptr(k), ptr(v), ptr(q_head_logits), ptr(k_head_logits), ptr(log_decay), ptr(cu_seqlens),
        ptr(initial_state), ptr(d_out), ptr(d_final_state), ptr(g["dq"]), ptr(g["dk"]), ptr(g["dv"]),
        ptr(g["dq_head_logits"]), ptr(g["dk_head_logits"]), ptr(g["dlog_decay"]), ptr(g["d_initial_state"]),
        ptr(workspace), workspace.numel(), torch.cuda.current_stream(dev).cuda_stream,
    )
    if rc != 0:
        raise SlaError(rc, sla_status_string(rc))
    return g


def sla_short_conv_silu(dtype: int, B: int, T: int, channels: int, taps: int, x, w, y, stream) -> int:
    """Raw call of the short-convolution + SiLU entry point (integer device addresses or None)."""
    return int(load_library().sla_short_conv_silu(int(dtype), int(B), int(T), int(channels), int(taps), _p(x), _p(w),
                                                   _p(y), _p(stream)))


def short_conv_silu(x, w):
    """x [B,T,C] (float32 or bfloat16), w [C,taps] float32 -> silu(causal depthwise convolution) [B,T,C]."""
    import torch

    assert x.is_cuda and x.is_contiguous() and x.dim() == 3
    B, T, C = x.shape
    assert w.dtype == torch.float32 and w.is_contiguous() and w.shape[0] == C
    y = torch.empty_like(x)
    dtype = {torch.float32: F32, torch.bfloat16: BF16}[x.dtype]
    rc = sla_short_conv_silu(dtype, B, T, C, w.shape[1], x.data_ptr(), w.data_ptr(), y.data_ptr(),
                             torch.cuda.current_stream(x.device).cuda_stream)
    if rc != 0:
        raise SlaError(rc, sla_status_string(rc))
    return y


def sla_short_conv_silu_l2(dtype, B, T, channels, taps, head_width, eps, x, w, y, stream) -> int:
    """Raw call of the feature map with the L2 option (integer device addresses or None)."""
    return int(load_library().sla_short_conv_silu_l2(int(dtype), int(B), int(T), int(channels), int(taps),
                                                      int(head_width), float(eps), _p(x), _p(w), _p(y), _p(stream)))


def sla_short_conv_silu_l2_backward_workspace_bytes(B, T, channels, taps) -> int:
    return int(load_library().sla_short_conv_silu_l2_backward_workspace_bytes(int(B), int(T), int(channels), int(taps)))


def sla_short_conv_silu_l2_backward(dtype, B, T, channels, taps, head_width, eps, x, w, dy, dx, dw, workspace,
                                    workspace_bytes, stream) -> int:
    """Raw call of the feature map's backward (integer device addresses or None)."""
    return int(load_library().sla_short_conv_silu_l2_backward(
        int(dtype), int(B), int(T), int(channels), int(taps), int(head_width), float(eps), _p(x), _p(w), _p(dy), _p(dx),
        _p(dw), _p(workspace), int(workspace_bytes), _p(stream)))


def sla_gate_logits_backward_workspace_bytes(params: SlaParams) -> int:
    return int(load_library().sla_gate_logits_backward_workspace_bytes(ctypes.byref(params)))


def sla_gate_logits_backward(params, x, w, d_head_logits, dx, dw, workspace, workspace_bytes, stream) -> int:
    """Raw call of one gate projection's backward (integer device addresses or None); dx is updated in place."""
    pr = ctypes.byref(params) if params is not None else None
    return int(load_library().sla_gate_logits_backward(pr, _p(x), _p(w), _p(d_head_logits), _p(dx), _p(dw),
                                                        _p(workspace), int(workspace_bytes), _p(stream)))


def short_conv_silu_l2(x, w, head_width: int = 0, eps: float = 1e-6):
    """x [B,T,C], w [C,taps] float32 -> silu(conv) with every head of head_width channels L2-normalised."""
    import torch

    assert x.is_cuda and x.is_contiguous() and x.dim() == 3
    B, T, C = x.shape
    y = torch.empty_like(x)
    dtype = {torch.float32: F32, torch.bfloat16: BF16}[x.dtype]
    rc = sla_short_conv_silu_l2(dtype, B, T, C, w.shape[1], head_width, eps, x.data_ptr(), w.data_ptr(), y.data_ptr(),
                                torch.cuda.current_stream(x.device).cuda_stream)
    if rc != 0:
        raise SlaError(rc, sla_status_string(rc))
    return y


def short_conv_silu_l2_backward(x, w, dy, head_width: int = 0, eps: float = 1e-6):
    """Gradients (dx like x, dw [C,taps] float32) of ``short_conv_silu_l2`` for the cotangent dy."""
    import torch

    B, T, C = x.shape
    K = w.shape[1]
    dx = torch.empty_like(x)
    dw = torch.empty((C, K), dtype=torch.float32, device=x.device)
    need = sla_short_conv_silu_l2_backward_workspace_bytes(B, T, C, K)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
    dtype = {torch.float32: F32, torch.bfloat16: BF16}[x.dtype]
    rc = sla_short_conv_silu_l2_backward(dtype, B, T, C, K, head_width, eps, x.data_ptr(), w.data_ptr(), dy.data_ptr(),
                                         dx.data_ptr(), dw.data_ptr(), ws.data_ptr(), ws.numel(),
                                         torch.cuda.current_stream(x.device).cuda_stream)
    if rc != 0:
        raise SlaError(rc, sla_status_string(rc))
    return dx, dw


def gate_logits_backward(x, w, d_head_logits, dx):
    """dx [B,T,H,dk] += d_head_logits[..., None] * w (in place); returns dw [H,dk] float32."""
    import torch

    B, T, H, dk = x.shape
    dtype = {torch.float32: F32, torch.bfloat16: BF16}[x.dtype]
    params = SlaParams(GLA, dtype, B, T, H, dk, 64, 0, 0, 1)
    dw = torch.empty((H, dk), dtype=torch.float32, device=x.device)
    need = sla_gate_logits_backward_workspace_bytes(params)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
    rc = sla_gate_logits_backward(params, x.data_ptr(), w.data_ptr(), d_head_logits.data_ptr(), dx.data_ptr(),
                                  dw.data_ptr(), ws.data_ptr(), ws.numel(), torch.cuda.current_stream(x.device).cuda_stream)
    if rc != 0:
        raise SlaError(rc, sla_status_string(rc))
    return dw


def sla_gate_logits(params, q, k, w_gq, w_gk, q_head_logits, k_head_logits, stream) -> int:
    """Raw call of the gate-logit entry point: every pointer argument is an integer device address or None."""
    pr = ctypes.byref(params) if params is not None else None
    return int(load_library().sla_gate_logits(pr, _p(q), _p(k), _p(w_gq), _p(w_gk), _p(q_head_logits),
                                               _p(k_head_logits), _p(stream)))


def gate_logits(q, k, w_gq, w_gk, *, dv: int = 0):
    """q, k [B,T,H,dk] (float32 or bfloat16; k may be None), w_gq, w_gk [H,dk] float32 -> (q_head_logits,
    k_head_logits) [B,T,H] float32 on the current CUDA(HIP) device and stream."""
    import torch

    assert q.is_cuda and q.is_contiguous()
    B, T, H, dk = q.shape
    dtype = {torch.float32: F32, torch.bfloat16: BF16}[q.dtype]
    assert w_gq.dtype == torch.float32 and tuple(w_gq.shape) == (H, dk) and w_gq.is_contiguous()
    ql = torch.empty((B, T, H), dtype=torch.float32, device=q.device)
    kl = None
    if k is not None:
        assert k.shape == q.shape and k.dtype == q.dtype and k.is_contiguous()
        assert w_gk.dtype == torch.float32 and tuple(w_gk.shape) == (H, dk) and w_gk.is_contiguous()
        kl = torch.empty_like(ql)
    params = SlaParams(GLA, dtype, B, T, H, dk, dv or dk, 0, 0, 1)
    ptr = lambda t: None if t is None else t.data_ptr()
    rc = sla_gate_logits(params, ptr(q), ptr(k), ptr(w_gq), ptr(w_gk), ptr(ql), ptr(kl),
                         torch.cuda.current_stream(q.device).cuda_stream)
    if rc != 0:
        raise SlaError(rc, sla_status_string(rc))
    return ql, kl


def sla_backward_workspace_bytes(params: SlaParams) -> int:
    return int(load_library().sla_backward_workspace_bytes(ctypes.byref(params)))


def sla_backward(params, q, k, v, q_head_logits, k_head_logits, log_decay, initial_state, d_out, d_final_state,
                 dq, dk, dv, dq_head_logits, dk_head_logits, dlog_decay, d_initial_state, workspace, workspace_bytes,
                 stream) -> int:
    """Raw call of the backward entry point: every pointer argument is an integer device address or None."""
    pr = ctypes.byref(params) if params is not None else None
    return int(
        load_library().sla_backward(
            pr, _p(q), _p(k), _p(v), _p(q_head_logits), _p(k_head_logits), _p(log_decay), _p(initial_state),
            _p(d_out), _p(d_final_state), _p(dq), _p(dk), _p(dv), _p(dq_head_logits), _p(dk_head_logits),
            _p(dlog_decay), _p(d_initial_state), _p(workspace), int(workspace_bytes), _p(stream),
        )
    )


def backward(variant: int, q, k, v, q_head_logits, k_head_logits, log_decay, d_out, initial_state=None,
             d_final_state=None, *, want_d_initial_state: bool = False, workspace=None, head_major: bool = False,
             segments: int = 1):
    """Gradients of ``forward`` (RetNet, GLA; bfloat16, or float32 in the single pass) on the current CUDA(HIP) device
    and stream.  Returns a dict
    of new tensors: dq, dk, dv, dq_head_logits, dk_head_logits (None without k_head_logits), dlog_decay (GLA only,
    else None) and d_initial_state (None unless asked for).  ``segments`` >= 2 cuts every batch row into that many
    segments that run in parallel (for batches with few sequences); 0 asks ``sla_backward_segments`` for the count
    that fills this device."""
    import torch

    assert q.is_cuda and q.dtype in (torch.bfloat16, torch.float32)
    if head_major:  # q, k, v, d_out, the GLA decay and their gradients are [B,H,T,d]
        B, H, T, dk = q.shape
    else:
        B, T, H, dk = q.shape
    dv = v.shape[-1]
    wide = (lambda d: (B, H, T, d)) if head_major else (lambda d: (B, T, H, d))
    for t, shape, dt in ((q, wide(dk), q.dtype), (k, wide(dk), q.dtype), (v, wide(dv), q.dtype),
                         (d_out, wide(dv), q.dtype), (q_head_logits, (B, T, H), torch.float32),
                         (k_head_logits, (B, T, H), torch.float32), (initial_state, (B, H, dk, dv), torch.float32),
                         (d_final_state, (B, H, dk, dv), torch.float32)):
        assert t is None or (tuple(t.shape) == shape and t.dtype == dt and t.is_contiguous() and t.is_cuda)
    want = {RETNET: ((H,), torch.float32), GLA: (tuple(q.shape), q.dtype)}[variant]
    assert tuple(log_decay.shape) == want[0] and log_decay.dtype == want[1] and log_decay.is_contiguous()
    dev = q.device
    g = {
        "dq": torch.empty_like(q),
        "dk": torch.empty_like(k),
        "dv": torch.empty_like(v),
        "dq_head_logits": torch.empty_like(q_head_logits),
        "dk_head_logits": None if k_head_logits is None else torch.empty_like(k_head_logits),
        "dlog_decay": torch.empty_like(log_decay) if variant == GLA else None,
        "d_initial_state": torch.empty((B, H, dk, dv), dtype=torch.float32, device=dev) if want_d_initial_state else None,
    }
    params = SlaParams(variant, BF16 if q.dtype == torch.bfloat16 else F32, B, T, H, dk, dv, 0,
                       FLAG_HEAD_MAJOR if head_major else 0, max(int(segments), 1))
    if int(segments) == 0:
        cus = torch.cuda.get_device_properties(q.device).multi_processor_count
        params.segments = max(sla_backward_segments(params, cus), 1)
    need = sla_backward_workspace_bytes(params)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    ptr = lambda t: None if t is None else t.data_ptr()
    rc = sla_backward(
        params, ptr(q), ptr(k), ptr(v), ptr(q_head_logits), ptr(k_head_logits), ptr(log_decay), ptr(initial_state),
        ptr(d_out), ptr(d_final_state), ptr(g["dq"]), ptr(g["dk"]), ptr(g["dv"]), ptr(g["dq_head_logits"]),
        ptr(g["dk_head_logits"]), ptr(g["dlog_decay"]), ptr(g["d_initial_state"]), ptr(workspace),
        workspace.numel() * workspace.element_size(), torch.cuda.current_stream(dev).cuda_stream,
    )
    if rc != 0:
        raise SlaError(rc, sla_status_string(rc))
    return g


def sla_backward_gdn_workspace_bytes(params: SlaParams) -> int:
    return int(load_library().sla_backward_gdn_workspace_bytes(ctypes.byref(params)))


def sla_backward_gdn(params, q, k, v, q_head_logits, k_head_logits, log_decay, beta, initial_state, d_out,
                     d_final_state, dq, dk, dv, dq_head_logits, dk_head_logits, dlog_decay, dbeta, d_initial_state,
                     workspace, workspace_bytes, stream) -> int:
    """Raw call of the gated delta rule's backward: every pointer argument is an integer device address or None."""
    pr = ctypes.byref(params) if params is not None else None
    return int(
        load_library().sla_backward_gdn(
            pr, _p(q), _p(k), _p(v), _p(q_head_logits), _p(k_head_logits), _p(log_decay), _p(beta),
            _p(initial_state), _p(d_out), _p(d_final_state), _p(dq), _p(dk), _p(dv), _p(dq_head_logits),
            _p(dk_head_logits), _p(dlog_decay), _p(dbeta), _p(d_initial_state), _p(workspace),
            ctypes.c_size_t(int(workspace_bytes)), _p(stream),
        )
    )


def sla_backward_gdn_varlen_workspace_bytes(params: SlaParams) -> int:
    return int(load_library().sla_backward_gdn_varlen_workspace_bytes(ctypes.byref(params)))


def sla_backward_gdn_varlen(params, q, k, v, q_head_logits, k_head_logits, log_decay, beta, cu_seqlens, initial_state,
                            d_out, d_final_state, dq, dk, dv, dq_head_logits, dk_head_logits, dlog_decay, dbeta,
                            d_initial_state, workspace, workspace_bytes, stream) -> int:
    """Raw call of the packed variable-length backward of the gated delta rule."""
    pr = ctypes.byref(params) if params is not None else None
    return int(
        load_library().sla_backward_gdn_varlen(
            pr, _p(q), _p(k), _p(v), _p(q_head_logits), _p(k_head_logits), _p(log_decay), _p(beta), _p(cu_seqlens),
            _p(initial_state), _p(d_out), _p(d_final_state), _p(dq), _p(dk), _p(dv), _p(dq_head_logits),
            _p(dk_head_logits), _p(dlog_decay), _p(dbeta), _p(d_initial_state), _p(workspace),
            ctypes.c_size_t(int(workspace_bytes)), _p(stream),
        )
    )


def backward_gdn_varlen(q, k, v, q_head_logits, k_head_logits, log_decay, beta, d_out, cu_seqlens, initial_state=None,
                        d_final_state=None, *, want_d_initial_state: bool = False):
    """Gradients of ``forward_varlen(GDN, ...)``: q, k [T,H,dk], v, d_out [T,H,dv] bfloat16; logits, log_decay, beta
    [T,H] float32; cu_seqlens [B+1] int32 on the device; states [B,H,dk,dv].  Returns a dict as ``backward_gdn``."""
    import torch

    assert q.is_cuda and q.dtype in (torch.bfloat16, torch.float32) and q.dim() == 3
    T, H, dk = q.shape
    dv = v.shape[-1]
    B = cu_seqlens.numel() - 1
    assert cu_seqlens.dtype == torch.int32 and cu_seqlens.is_cuda
    dev = q.device
    g = {
        "dq": torch.empty_like(q),
        "dk": torch.empty_like(k),
        "dv": torch.empty_like(v),
        "dq_head_logits": torch.empty_like(q_head_logits),
        "dk_head_logits": None if k_head_logits is None else torch.empty_like(k_head_logits),
        "dlog_decay": torch.empty_like(log_decay),
        "dbeta": torch.empty_like(beta),
        "d_initial_state": torch.empty((B, H, dk, dv), dtype=torch.float32, device=dev) if want_d_initial_state else None,
    }
    params = SlaParams(GDN, BF16 if q.dtype == torch.bfloat16 else F32, B, T, H, dk, dv, 0, 0, 1)
    need = sla_backward_gdn_varlen_workspace_bytes(params)
    workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    ptr = lambda t: None if t is None else t.data_ptr()
    rc = sla_backward_gdn_varlen(
        params, ptr(q), ptr(k), ptr(v), ptr(q_head_logits), ptr(k_head_logits), ptr(log_decay), ptr(beta),
        ptr(cu_seqlens), ptr(initial_state), ptr(d_out), ptr(d_final_state), ptr(g["dq"]), ptr(g["dk"]), ptr(g["dv"]),
        ptr(g["dq_head_logits"]), ptr(g["dk_head_logits"]), ptr(g["dlog_decay"]), ptr(g["dbeta"]),
        ptr(g["d_initial_state"]), ptr(workspace), workspace.numel(), torch.cuda.current_stream(dev).cuda_stream,
    )
    if rc != 0:
        raise SlaError(rc, sla_status_string(rc))
    return g


def backward_gdn(q, k, v, q_head_logits, k_head_logits, log_decay, beta, d_out, initial_state=None,
                 d_final_state=None, *, want_d_initial_state: bool = False, workspace=None):
    """Gradients of ``forward(GDN, ...)`` (bfloat16 or float32 q, k, v, d_out [B,T,H,d]; float32 logits, log_decay and beta
    [B,T,H]) on the current CUDA(HIP) device and stream.  Returns a dict of new tensors: dq, dk, dv,
    dq_head_logits, dk_head_logits (None without k_head_logits), dlog_decay, dbeta and d_initial_state (None unless
    asked for)."""
    import torch

    assert q.is_cuda and q.dtype in (torch.bfloat16, torch.float32)
    B, T, H, dk = q.shape
    dv = v.shape[-1]
    for t, shape, dt in ((q, (B, T, H, dk), q.dtype), (k, (B, T, H, dk), q.dtype), (v, (B, T, H, dv), q.dtype),
                         (d_out, (B, T, H, dv), q.dtype), (q_head_logits, (B, T, H), torch.float32),
                         (k_head_logits, (B, T, H), torch.float32), (log_decay, (B, T, H), torch.float32),
                         (beta, (B, T, H), torch.float32), (initial_state, (B, H, dk, dv), torch.float32),
                         (d_final_state, (B, H, dk, dv), torch.float32)):
        assert t is None or (tuple(t.shape) == shape and t.dtype == dt and t.is_contiguous() and t.is_cuda)
    dev = q.device
    g = {
        "dq": torch.empty_like(q),
        "dk": torch.empty_like(k),
        "dv": torch.empty_like(v),
        "dq_head_logits": torch.empty_like(q_head_logits),
        "dk_head_logits": None if k_head_logits is None else torch.empty_like(k_head_logits),
        "dlog_decay": torch.empty_like(log_decay),
        "dbeta": torch.empty_like(beta),
        "d_initial_state": torch.empty((B, H, dk, dv), dtype=torch.float32, device=dev) if want_d_initial_state else None,
    }
    params = SlaParams(GDN, BF16 if q.dtype == torch.bfloat16 else F32, B, T, H, dk, dv, 0, 0, 1)
    need = sla_backward_gdn_workspace_bytes(params)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    ptr = lambda t: None if t is None else t.data_ptr()
    rc = sla_backward_gdn(
        params, ptr(q), ptr(k), ptr(v), ptr(q_head_logits), ptr(k_head_logits), ptr(log_decay), ptr(beta),
        ptr(initial_state), ptr(d_out), ptr(d_final_state), ptr(g["dq"]), ptr(g["dk"]), ptr(g["dv"]),
        ptr(g["dq_head_logits"]), ptr(g["dk_head_logits"]), ptr(g["dlog_decay"]), ptr(g["dbeta"]),
        ptr(g["d_initial_state"]), ptr(workspace), workspace.numel() * workspace.element_size(),
        torch.cuda.current_stream(dev).cuda_stream,
    )
    if rc != 0:
        raise SlaError(rc, sla_status_string(rc))
    return g


def decode_step(variant: int, q, k, v, q_head_logits, k_head_logits, log_decay, beta, state, *, out=None,
                w_gq=None, w_gk=None):
    """One recurrent step on the current CUDA(HIP) device and stream: q, k [B,H,dk], v [B,H,dv], logits / beta
    [B,H] float32, state [B,H,dk,dv] float32 (updated in place).  Returns out [B,H,dv].  With w_gq (and
    optionally w_gk) [H,dk] float32 the kernel forms the logits itself (sla_decode_step_fused) and the two logits
    arguments must be None."""
    import torch

    if w_gq is not None:
        assert q_head_logits is None and k_head_logits is None
        B, H, dk = q.shape
        dv = v.shape[-1]
        for w in (w_gq, w_gk):
            assert w is None or (w.dtype == torch.float32 and tuple(w.shape) == (H, dk) and w.is_contiguous())
        assert state.dtype == torch.float32 and state.shape == (B, H, dk, dv) and state.is_contiguous()
        dtype = {torch.float32: F32, torch.bfloat16: BF16}[q.dtype]
        if out is None:
            out = torch.empty((B, H, dv), dtype=q.dtype, device=q.device)
        params = SlaParams(variant, dtype, B, 1, H, dk, dv, 0, 0, 1)
        ptr = lambda t: None if t is None else t.data_ptr()
        rc = sla_decode_step_fused(params, ptr(q), ptr(k), ptr(v), ptr(w_gq), ptr(w_gk), ptr(log_decay), ptr(beta),
                                   ptr(state), ptr(out), torch.cuda.current_stream(q.device).cuda_stream)
        if rc != 0:
            raise SlaError(rc, sla_status_string(rc))
        return out

    assert q.is_cuda and q.is_contiguous() and k.is_contiguous() and v.is_contiguous()
    B, H, dk = q.shape
    dv = v.shape[-1]
    assert k.shape == (B, H, dk) and v.shape == (B, H, dv) and k.dtype == q.dtype and v.dtype == q.dtype
    dtype = {torch.float32: F32, torch.bfloat16: BF16}[q.dtype]
    assert q_head_logits.dtype == torch.float32 and q_head_logits.shape == (B, H) and q_head_logits.is_contiguous()
    if k_head_logits is not None:
        assert k_head_logits.dtype == torch.float32 and k_head_logits.shape == (B, H) and k_head_logits.is_contiguous()
    want = {RETNET: ((H,), torch.float32), GLA: ((B, H, dk), q.dtype), GDN: ((B, H), torch.float32)}[variant]
    assert tuple(log_decay.shape) == want[0] and log_decay.dtype == want[1] and log_decay.is_contiguous()
    if beta is not None:
        assert beta.dtype == torch.float32 and beta.shape == (B, H) and beta.is_contiguous()
    assert state.dtype == torch.float32 and state.shape == (B, H, dk, dv) and state.is_contiguous()
    if out is None:
        out = torch.empty((B, H, dv), dtype=q.dtype, device=q.device)
    params = SlaParams(variant, dtype, B, 1, H, dk, dv, 0, 0, 1)
    ptr = lambda t: None if t is None else t.data_ptr()
    rc = sla_decode_step(
        params, ptr(q), ptr(k), ptr(v), ptr(q_head_logits), ptr(k_head_logits), ptr(log_decay), ptr(beta), ptr(state),
        ptr(out), torch.cuda.current_stream(q.device).cuda_stream,
    )
    if rc != 0:
        raise SlaError(rc, sla_status_string(rc))
    return out


_cus = {}


def _compute_units(device) -> int:
    import torch

    i = torch.device(device).index
    i = torch.cuda.current_device() if i is None else i
    if i not in _cus:
        _cus[i] = torch.cuda.get_device_properties(i).multi_processor_count
    return _cus[i]


def forward(
    variant: int,
    q,
    k,
    v,
    q_head_logits,
    k_head_logits,
    log_decay,
    beta=None,
    initial_state=None,
    *,
    dv_split: int = 0,
    out=None,
    final_state=None,
    want_final_state: bool = True,
    segments: int = 1,
    workspace=None,
    head_major: bool = False,
) -> Tuple["torch.Tensor", Optional["torch.Tensor"]]:
    """SLA forward on the current CUDA(HIP) device and stream.  Tensors must be contiguous CUDA tensors:
    q,k [B,T,H,dk], v [B,T,H,dv] in float32 or bfloat16; logits/beta/initial_state float32.

    segments = 1 runs one fused pass (sla_forward).  segments = 0 lets the library choose the
    segment-parallel schedule, segments > 1 asks for that many segments (sla_forward_ws); the workspace
    is then taken from ``workspace`` (a CUDA tensor of at least sla_workspace_bytes bytes) or allocated here.

    head_major = True: q, k, v (and the GLA log_decay, and the returned out) are [B,H,T,d] (SLA_FLAG_HEAD_MAJOR)."""
    import torch

    assert q.is_cuda and q.is_contiguous() and k.is_contiguous() and v.is_contiguous()
    if head_major:
        B, H, T, dk = q.shape
    else:
        B, T, H, dk = q.shape
    dv = v.shape[-1]
    assert k.shape == q.shape and v.shape == q.shape[:3] + (dv,) and k.dtype == q.dtype and v.dtype == q.dtype
    dtype = {torch.float32: F32, torch.bfloat16: BF16}[q.dtype]
    assert q_head_logits.dtype == torch.float32 and q_head_logits.shape == (B, T, H) and q_head_logits.is_contiguous()
    if k_head_logits is not None:
        assert k_head_logits.dtype == torch.float32 and k_head_logits.shape == (B, T, H) and k_head_logits.is_contiguous()
    want = {RETNET: ((H,), torch.float32), GLA: (tuple(q.shape), q.dtype), GDN: ((B, T, H), torch.float32)}[variant]
    assert tuple(log_decay.shape) == want[0] and log_decay.dtype == want[1] and log_decay.is_contiguous()
    if beta is not None:
        assert beta.dtype == torch.float32 and beta.shape == (B, T, H) and beta.is_contiguous()
    if initial_state is not None:
        assert initial_state.dtype == torch.float32 and initial_state.shape == (B, H, dk, dv) and initial_state.is_contiguous()
    if out is None:
        out = torch.empty(tuple(v.shape), dtype=q.dtype, device=q.device)
    if final_state is None and want_final_state:
        final_state = torch.empty((B, H, dk, dv), dtype=torch.float32, device=q.device)
    params = SlaParams(variant, dtype, B, T, H, dk, dv, dv_split, FLAG_HEAD_MAJOR if head_major else 0, segments)
    ptr = lambda t: None if t is None else t.data_ptr()
    stream = torch.cuda.current_stream(q.device).cuda_stream
    if segments == 1:
        rc = sla_forward(
            params, ptr(q), ptr(k), ptr(v), ptr(q_head_logits), ptr(k_head_logits), ptr(log_decay), ptr(beta),
            ptr(initial_state), ptr(out), ptr(final_state), stream,
        )
    else:
        need = sla_workspace_bytes(params, _compute_units(q.device))
        if workspace is None and need > 0:
            workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
        ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
        rc = sla_forward_ws(
            params, ptr(q), ptr(k), ptr(v), ptr(q_head_logits), ptr(k_head_logits), ptr(log_decay), ptr(beta),
            ptr(initial_state), ptr(out), ptr(final_state), ptr(workspace), ws_bytes, stream,
        )
    if rc != 0:
        raise SlaError(rc, sla_status_string(rc))
    return out, final_state
