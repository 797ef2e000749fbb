"""MI355X-native Softmax Linear Attention (SLA) chunkwise-parallel forward.

A thin ctypes binding over ``libsla.so`` (C ABI declared in ``include/sla.h``).
PyTorch is used for device memory and streams only; every step of the path
runs in the library's HIP kernels.  There is no CPU fallback: without the
built library the calls raise.
"""
from .binding import (  # noqa: F401
    RETNET,
    GLA,
    GDN,
    F32,
    BF16,
    FLAG_HEAD_MAJOR,
    SlaError,
    SlaParams,
    library_path,
    load_library,
    sla_backward,
    sla_backward_workspace_bytes,
    sla_backward_gdn,
    sla_backward_gdn_workspace_bytes,
    sla_backward_gdn_varlen,
    sla_backward_gdn_varlen_workspace_bytes,
    sla_check_args,
    sla_gate_logits,
    sla_short_conv_silu,
    sla_short_conv_silu_l2,
    sla_short_conv_silu_l2_backward,
    sla_short_conv_silu_l2_backward_workspace_bytes,
    sla_gate_logits_backward,
    sla_gate_logits_backward_workspace_bytes,
    short_conv_silu_l2,
    short_conv_silu_l2_backward,
    gate_logits_backward,
    sla_decode_step,
    sla_decode_step_fused,
    sla_default_dv_split,
    sla_forward,
    sla_forward_ws,
    sla_forward_static,
    sla_init,
    sla_device_status,
    DEVICE_WAIT_EXPIRED,
    DEVICE_DECAY_RANGE,
    sla_static_scratch_bytes,
    sla_forward_varlen,
    sla_backward_varlen,
    sla_backward_varlen_workspace_bytes,
    sla_segments,
    sla_backward_segments,
    sla_workspace_bytes,
    sla_kernel_name,
    sla_status_string,
    sla_version,
    forward,
    forward_varlen,
    backward,
    backward_gdn,
    backward_gdn_varlen,
    backward_varlen,
    gate_logits,
    short_conv_silu,
    decode_step,
)

# Variants with kernels in this build (sla_forward returns SLA_ERR_UNSUPPORTED for the others).
SUPPORTED_VARIANTS = (RETNET, GLA, GDN)

