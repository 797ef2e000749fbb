"""The C-ABI library without a GPU: it loads, exports every symbol the header declares, and rejects bad
calls before any device work (validation runs first)."""
import ctypes
import os
import re

import pytest

import paper_2602_01744_amd as sla
from paper_2602_01744_amd import SlaParams

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
A = 1 << 20  # a 16-byte aligned fake address; validation never dereferences it


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(sla.library_path()):
        from paper_2602_01744_amd import build

        build.build()
    return sla.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "sla.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = re.findall(r"\b(sla_[a-z0-9_]+)\s*\(", header)
    assert set(names) >= {"sla_forward", "sla_forward_ws", "sla_forward_static", "sla_init", "sla_device_status", "sla_static_scratch_bytes", "sla_backward", "sla_backward_workspace_bytes", "sla_backward_gdn", "sla_backward_gdn_workspace_bytes", "sla_backward_gdn_varlen", "sla_backward_gdn_varlen_workspace_bytes", "sla_gate_logits", "sla_short_conv_silu", "sla_short_conv_silu_l2", "sla_short_conv_silu_l2_backward", "sla_short_conv_silu_l2_backward_workspace_bytes", "sla_gate_logits_backward", "sla_gate_logits_backward_workspace_bytes", "sla_forward_varlen", "sla_backward_varlen", "sla_backward_varlen_workspace_bytes", "sla_decode_step", "sla_decode_step_fused", "sla_workspace_bytes", "sla_segments", "sla_backward_segments", "sla_check_args", "sla_default_dv_split", "sla_kernel_name",
                          "sla_status_string", "sla_version"}
    for n in set(names):
        assert hasattr(lib, n), n


def test_version_and_status_strings(lib):
    assert sla.sla_version() >= 100
    for code in (0, -1, -2, -3, -4, -5, -6, -7):
        assert sla.sla_status_string(code)
    assert "unknown" in sla.sla_status_string(-99)


def _ok_params(**kw):
    d = dict(variant=sla.GLA, dtype=sla.BF16, B=2, T=128, H=4, dk=128, dv=128, dv_split=0, flags=0)
    d.update(kw)
    return SlaParams(**d)


def _call(p, **kw):
    a = dict(q=A, k=A, v=A, ql=A, kl=A, ld=A, beta=0, s0=0, out=A, fin=A)
    a.update(kw)
    return sla.sla_check_args(p, a["q"], a["k"], a["v"], a["ql"], a["kl"], a["ld"], a["beta"], a["s0"], a["out"], a["fin"])


def test_valid_calls_pass_validation(lib):
    assert _call(_ok_params()) == 0
    assert _call(_ok_params(), kl=0, fin=0) == 0
    assert _call(_ok_params(variant=sla.GDN), beta=A) == 0
    assert _call(_ok_params(variant=sla.RETNET, dtype=sla.F32, dk=64, dv=64, dv_split=16)) == 0
    assert _call(_ok_params(B=0), q=0, k=0, v=0, ql=0, ld=0, out=0) == 0
    assert _call(_ok_params(T=0), q=0, k=0, v=0, ql=0, ld=0, out=0) == 0


def test_null_and_misplaced_pointers(lib):
    for name in ("q", "k", "v", "ql", "ld", "out"):
        assert _call(_ok_params(), **{name: 0}) == -1, name
    assert sla.sla_check_args(None, A, A, A, A, A, A, 0, 0, A, A) == -1
    assert _call(_ok_params(variant=sla.GDN)) == -1           # GDN needs beta
    assert _call(_ok_params(), beta=A) == -1                   # beta only for GDN


def test_shapes_and_unsupported(lib):
    assert _call(_ok_params(B=-1)) == -2
    assert _call(_ok_params(T=-5)) == -2
    assert _call(_ok_params(H=0)) == -2
    assert _call(_ok_params(H=65)) == -2
    assert _call(_ok_params(dk=0)) == -2
    assert _call(_ok_params(dk=96)) == -3
    assert _call(_ok_params(dv=512)) == -3
    assert _call(_ok_params(dv=256)) == 0
    assert _call(_ok_params(variant=7)) == -3
    assert _call(_ok_params(dtype=2)) == -3
    assert _call(_ok_params(flags=4)) == -3
    assert _call(_ok_params(dv_split=48)) == -2
    assert _call(_ok_params(dv=64, dv_split=128)) == -2
    assert _call(_ok_params(dv_split=128)) == -3
    assert _call(_ok_params(B=1 << 20, T=1 << 20)) == -2


def test_alignment(lib):
    for name in ("q", "k", "v", "ql", "kl", "ld", "out", "fin", "s0"):
        assert _call(_ok_params(), **{name: A + 8}) == -4, name


def test_forward_rejects_before_touching_the_device(lib):
    # sla_forward runs the same checks first: a bad call returns its status even with no GPU present.
    p = _ok_params(dk=96)
    assert sla.sla_forward(p, A, A, A, A, A, A, 0, 0, A, A, 0) == -3
    assert sla.sla_forward(_ok_params(), 0, A, A, A, A, A, 0, 0, A, A, 0) == -1
    assert sla.sla_forward(_ok_params(B=0), 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0) == 0


def test_default_slice_width_fills_the_device(lib):
    # 128 sequences on 256 CUs: two slices of 64 columns each
    assert sla.sla_default_dv_split(_ok_params(B=8, H=16), 256) == 64
    # 32 sequences: 8 slices of 16 columns
    assert sla.sla_default_dv_split(_ok_params(B=4, H=8), 256) == 16
    assert sla.sla_default_dv_split(_ok_params(B=1, H=32), 256) == 16
    assert sla.sla_default_dv_split(_ok_params(B=64, H=16), 256) == 64
    assert sla.sla_default_dv_split(_ok_params(), 0) == -2
    name = sla.sla_kernel_name(_ok_params(B=8, H=16))
    assert name.startswith("sla_fwd_kernel<") and "128, 64" in name


def test_segment_schedule_choice_and_workspace_size(lib):
    # enough rows to fill the device: one pass, no workspace
    assert sla.sla_segments(_ok_params(B=8, T=2048, H=16), 256) == 1
    assert sla.sla_workspace_bytes(_ok_params(B=8, T=2048, H=16), 256) == 0
    # 32 (batch, head) pairs x 2 slices of 64 columns on 256 CUs: 4 segments of 512 tokens
    p = _ok_params(B=4, T=2048, H=8)
    assert sla.sla_segments(p, 256) == 4
    heads = 4 * 8
    # entry states of the 4 segments + up to 8 partial decay products for each of the first 3
    assert sla.sla_workspace_bytes(p, 256) == 4 * (heads * 4 * 128 * 128 + heads * 3 * 8 * 128)
    # segments are at least 256 tokens and a multiple of 64; short sequences stay in one pass
    assert sla.sla_segments(_ok_params(B=1, T=300, H=1), 256) == 2
    assert sla.sla_segments(_ok_params(B=1, T=256, H=1), 256) == 1
    assert sla.sla_segments(_ok_params(B=1, T=16384, H=4), 256) == 32
    # an explicit request is honoured down to the minimum segment length
    assert sla.sla_segments(_ok_params(B=8, T=2048, H=16, segments=3), 256) == 3
    assert sla.sla_segments(_ok_params(B=8, T=2048, H=16, segments=64), 256) == 8
    assert sla.sla_segments(_ok_params(B=8, T=2048, H=16, segments=1), 256) == 1
    # the delta rule has no segment schedule
    assert sla.sla_segments(_ok_params(variant=sla.GDN, B=1, T=4096, H=4), 256) == 1
    assert sla.sla_segments(_ok_params(variant=sla.GDN, segments=2), 256) == -3
    assert sla.sla_segments(_ok_params(segments=-1), 256) == -2
    assert sla.sla_workspace_bytes(_ok_params(segments=-1), 256) == 0


def test_segments_need_a_workspace(lib):
    p = _ok_params(B=1, T=1024, H=2, segments=2)
    assert sla.sla_forward(p, A, A, A, A, A, A, 0, 0, A, A, 0) == -6
    assert _call(_ok_params(variant=sla.GDN, segments=2), beta=A) == -3
    assert sla.sla_forward_ws(_ok_params(dk=96), A, A, A, A, A, A, 0, 0, A, A, A, 1 << 30, 0) == -3
    assert sla.sla_forward_ws(_ok_params(), A, A, A, A, A, A, 0, 0, A, A, A + 4, 1 << 30, 0) == -4
    assert sla.sla_forward_ws(_ok_params(B=0), 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0) == 0


def test_decode_step_validation(lib):
    one = _ok_params(T=1)
    args = (A, A, A, A, A, A, 0)
    assert sla.sla_decode_step(_ok_params(T=2), *args, A, A, 0) == -2          # one token per call
    assert sla.sla_decode_step(_ok_params(T=1, dk=96), *args, A, A, 0) == -3
    assert sla.sla_decode_step(one, 0, A, A, A, A, A, 0, A, A, 0) == -1        # q missing
    assert sla.sla_decode_step(one, *args, 0, A, 0) == -1                      # the state is required
    assert sla.sla_decode_step(one, *args, A + 4, A, 0) == -4
    assert sla.sla_decode_step(_ok_params(T=1, variant=sla.GDN), *args, A, A, 0) == -1   # GDN needs beta
    assert sla.sla_decode_step(_ok_params(T=1, B=0), 0, 0, 0, 0, 0, 0, 0, 0, 0, 0) == 0
    # the fused form: the gate matrices take the place of the logits, with the same rules
    assert sla.sla_decode_step_fused(_ok_params(T=2), *args, A, A, 0) == -2
    assert sla.sla_decode_step_fused(one, A, A, A, 0, A, A, 0, A, A, 0) == -1  # w_gq missing
    assert sla.sla_decode_step_fused(one, A, A, A, A + 4, A, A, 0, A, A, 0) == -4
    assert sla.sla_decode_step_fused(one, *args, 0, A, 0) == -1
    assert sla.sla_decode_step_fused(_ok_params(T=1, dk=32, dv=64), *args, A, A, 0) in (0, -5)  # valid: reaches the launch
    assert sla.sla_decode_step_fused(_ok_params(T=1, B=0), 0, 0, 0, 0, 0, 0, 0, 0, 0, 0) == 0


def test_missing_library_fails_loudly(monkeypatch):
    import paper_2602_01744_amd.binding as b

    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "_LIB_PATH", "/nonexistent/libsla.so")
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        b.load_library()


# ------------------------------------------------------------------ sla_backward: validation before any device work
def _bwd(p, **kw):
    a = dict(q=A, k=A, v=A, ql=A, kl=A, ld=A, s0=0, dout=A, dsf=0, dq=A, dk=A, dv=A, dql=A, dkl=A, dld=A, ds0=0,
             ws=A, ws_bytes=1 << 40)
    a.update(kw)
    return sla.sla_backward(p, a["q"], a["k"], a["v"], a["ql"], a["kl"], a["ld"], a["s0"], a["dout"], a["dsf"],
                            a["dq"], a["dk"], a["dv"], a["dql"], a["dkl"], a["dld"], a["ds0"], a["ws"], a["ws_bytes"], 0)


def test_backward_rejects_bad_calls(lib):
    ok = _ok_params()
    assert _bwd(_ok_params(variant=sla.GDN)) == -3           # the delta rule's backward is sla_backward_gdn
    assert _bwd(_ok_params(dtype=sla.F32, segments=2, T=1024)) == -3   # fp32 tensors: the single pass only
    assert _bwd(_ok_params(dk=96)) == -3
    assert _bwd(ok, dout=0) == -1
    assert _bwd(ok, dq=0) == -1
    assert _bwd(ok, dld=0) == -1                             # GLA needs the decay gradient buffer
    assert _bwd(_ok_params(variant=sla.RETNET), dld=A) == -1  # RetNet's decay is a constant
    assert _bwd(ok, kl=0) == -1 and _bwd(ok, dkl=0) == -1    # write-gate logits and their gradient go together
    assert _bwd(ok, dv=A + 4) == -4
    assert _bwd(ok, ws=0) == -6
    assert _bwd(ok, ws_bytes=1024) == -6
    assert _bwd(None) == -1
    # empty problems are accepted without touching the device
    assert _bwd(_ok_params(B=0)) == 0
    assert _bwd(_ok_params(T=0)) == 0


def test_backward_workspace_size(lib):
    B, T, H, dk, dv = 2, 128, 4, 128, 64
    n = B * T * H
    gla = sla.sla_backward_workspace_bytes(_ok_params(B=B, T=T, H=H, dk=dk, dv=dv))
    ret = sla.sla_backward_workspace_bytes(_ok_params(variant=sla.RETNET, B=B, T=T, H=H, dk=dk, dv=dv))
    # gates (2 planes), partial gate gradients (dk/16 planes each); GLA adds the q*dq block sums
    # [B*T/16 + B + 1][H,dk], [B,H,dk] and the bf16 states kept every 512 tokens [B*T/512 + 1][H,dk,dv]
    assert ret == 4 * n * (2 + 2 * (dk // 16))
    assert gla == ret + 4 * ((B * T // 16 + B + 1) * H * dk + B * H * dk + (B * T // 512 + 1) * H * dk * dv // 2)
    big = sla.sla_backward_workspace_bytes(_ok_params(B=8, T=2048, H=16, dk=128, dv=128))
    assert big == 4 * (8 * 2048 * 16 * 18 + (1024 + 9) * 2048 + 8 * 2048 + 33 * 16 * 128 * 128 // 2)
    assert sla.sla_backward_workspace_bytes(_ok_params(variant=sla.GDN)) == 0
    # fp32 tensors: gates, dk/8 + dv/8 partial planes, GLA the final-state term of the decay gradient [B,H,dk]
    f32 = sla.sla_backward_workspace_bytes(_ok_params(dtype=sla.F32, B=B, T=T, H=H, dk=dk, dv=dv))
    assert f32 == 4 * (n * (2 + dk // 8 + dv // 8) + B * H * dk)
    f32r = sla.sla_backward_workspace_bytes(_ok_params(variant=sla.RETNET, dtype=sla.F32, B=B, T=T, H=H, dk=dk, dv=dv))
    assert f32r == 4 * n * (2 + dk // 8 + dv // 8)
    assert sla.sla_backward_workspace_bytes(_ok_params(dtype=sla.F32, B=B, T=1024, H=H, dk=dk, dv=dv, segments=2)) == 0


def test_gate_logits_rejects_bad_calls(lib):
    ok = _ok_params()
    call = lambda p, q=A, k=A, wq=A, wk=A, ql=A, kl=A: sla.sla_gate_logits(p, q, k, wq, wk, ql, kl, 0)
    assert call(ok, q=0) == -1 and call(ok, wq=0) == -1 and call(ok, ql=0) == -1
    assert call(ok, k=0) == -1 and call(ok, wk=0) == -1 and call(ok, kl=0) == -1  # k, w_gk, k logits go together
    assert call(ok, wq=A + 8) == -4
    assert call(_ok_params(dk=48)) == -3
    assert call(None) == -1
    assert call(_ok_params(B=0)) == 0 and call(_ok_params(T=0)) == 0


def test_varlen_rejects_bad_calls(lib):
    ok = _ok_params()
    fwd = lambda p, cu=A, q=A: sla.sla_forward_varlen(p, q, A, A, A, A, A, 0, cu, 0, A, A, 0)
    assert fwd(ok, cu=0) == -1                       # the offsets are required
    assert fwd(ok, cu=A + 2) == -4
    assert fwd(ok, q=0) == -1
    assert fwd(_ok_params(segments=3)) == -3         # packed batches run one pass per sequence
    assert fwd(_ok_params(B=0), cu=0) == 0
    bwd = lambda p, cu=A: sla.sla_backward_varlen(p, A, A, A, A, A, A, cu, 0, A, 0, A, A, A, A, A, A, 0, A, 1 << 40, 0)
    assert bwd(ok, cu=0) == -1
    assert bwd(_ok_params(variant=sla.GDN)) == -3
    # the packed workspace is sized by the total token count p->T, not B * T
    p = _ok_params(B=5, T=1000)
    one = _ok_params(B=1, T=1000)
    extra = 4 * (5 - 1) * p.H * p.dk * 2  # per sequence: one [H,dk] row of final-state terms, one more block of sums
    assert sla.sla_backward_varlen_workspace_bytes(p) == sla.sla_backward_workspace_bytes(one) + extra


def test_layout_flag_is_for_rectangular_forward_and_backward(lib):
    hm = _ok_params(flags=1)
    assert _call(hm) == 0                                    # sla_forward accepts SLA_FLAG_HEAD_MAJOR
    assert _call(_ok_params(flags=2)) == -3                  # unknown flag bits
    assert _bwd(hm, ws_bytes=16) == -6                       # sla_backward too: validation gets as far as the workspace
    assert sla.sla_forward_varlen(hm, A, A, A, A, A, A, 0, A, 0, A, A, 0) == -3
    assert sla.sla_gate_logits(hm, A, A, A, A, A, A, 0) == -3


def test_short_conv_rejects_bad_calls(lib):
    call = lambda dtype=sla.BF16, B=2, T=64, C=256, taps=4, x=A, w=A, y=A: sla.sla_short_conv_silu(dtype, B, T, C, taps, x, w, y, 0)
    assert call(dtype=5) == -3 and call(taps=0) == -3 and call(taps=5) == -3
    assert call(C=12) == -2 and call(C=0) == -2 and call(B=-1) == -2
    assert call(x=0) == -1 and call(w=0) == -1 and call(y=0) == -1
    assert call(y=A + 4) == -4
    assert call(B=0) == 0 and call(T=0) == 0


def test_backward_gdn_rejects_bad_calls(lib):
    ok = _ok_params(variant=sla.GDN)
    big = 1 << 40

    def call(p, q=A, ld=A, beta=A, kl=A, dkl=A, dld=A, dbeta=A, ws=A, ws_bytes=big):
        return sla.sla_backward_gdn(p, q, A, A, A, kl, ld, beta, 0, A, 0, A, A, A, A, dkl, dld, dbeta, 0, ws,
                                    ws_bytes, 0)

    assert call(None) == -1
    assert call(_ok_params(variant=sla.GLA)) == -3 and call(_ok_params(variant=sla.RETNET)) == -3
    assert call(_ok_params(variant=sla.GDN, dtype=sla.F32), ws_bytes=16) == -6    # fp32 tensors are covered too
    assert call(_ok_params(variant=sla.GDN, flags=1)) == -3
    assert call(ok, q=0) == -1 and call(ok, ld=0) == -1 and call(ok, beta=0) == -1
    assert call(ok, dld=0) == -1 and call(ok, dbeta=0) == -1
    assert call(ok, kl=0) == -1 and call(ok, dkl=0) == -1 and call(ok, kl=0, dkl=0) != -1
    assert call(ok, beta=A + 4) == -4
    assert call(ok, ws=0) == -6 and call(ok, ws_bytes=16) == -6
    assert call(_ok_params(variant=sla.GDN, B=0)) == 0
    assert call(_ok_params(variant=sla.GDN, T=0), ws=0) == 0    # no tokens, no initial-state gradient asked for


def test_backward_gdn_workspace_size(lib):
    B, T, H, dk, dv = 2, 100, 4, 128, 64
    n = B * T * H
    # fp32 tensors (token-recurrent sweeps): gates and the decay scalar (3 planes), dk/8 partial planes of dG^Q and
    # dv/8 each of dG^K and dbeta, <d_final, S_T> partials, two fp32 tensors like v and one like k
    f32 = sla.sla_backward_gdn_workspace_bytes(_ok_params(variant=sla.GDN, dtype=sla.F32, B=B, T=T, H=H, dk=dk, dv=dv))
    pv, pk = dv // 8, dk // 8
    assert f32 == 4 * (n * (3 + 2 * pv + pk) + pk * B * H + 2 * n * dv + n * dk)
    # bf16 tensors (block form): a plane per 16 columns; per 32-token block and head 8 x 32 scalars, one 32 x 32
    # bf16 matrix, two bf16 [dv][32] tiles and one bf16 [dk][32] tile
    bf16 = sla.sla_backward_gdn_workspace_bytes(_ok_params(variant=sla.GDN, dtype=sla.BF16, B=B, T=T, H=H, dk=dk, dv=dv))
    pv, pk = dv // 16, dk // 16
    bh = B * ((T + 31) // 32) * H
    na = B * T // 512 + 1  # anchors of the decay gradient: partial <X, S> [na][H][dk/16] and X [na][H][dk][dv]
    assert bf16 == 4 * (n * (3 + 2 * pv + pk) + pk * B * H + na * H * pk + na * H * dk * dv +
                        bh * 256 + bh * 1024 // 2 + 2 * (bh * dv * 32 // 2) + bh * dk * 32 // 2)
    assert sla.sla_backward_gdn_workspace_bytes(_ok_params(variant=sla.GLA)) == 0
    # packed batches: floor(T / 32) + B + 1 blocks whatever the sequence lengths are
    packed = sla.sla_backward_gdn_varlen_workspace_bytes(_ok_params(variant=sla.GDN, dtype=sla.BF16, B=3, T=200, H=H, dk=dk, dv=dv))
    n, bh = 200 * H, (200 // 32 + 3 + 1) * H
    assert packed == 4 * (n * (3 + 2 * pv + pk) + pk * 3 * H + H * pk + H * dk * dv +
                          bh * 256 + bh * 1024 // 2 + 2 * (bh * dv * 32 // 2) + bh * dk * 32 // 2)


def test_backward_segment_schedule_workspace_and_validation(lib):
    # p->segments >= 2 cuts every batch row: the packed workspace of B * nseg sequences plus the pre-passes' own
    B, T, H, dk, dv, nseg = 2, 1024, 4, 128, 64, 4
    one = sla.sla_backward_workspace_bytes(_ok_params(B=B, T=T, H=H, dk=dk, dv=dv))
    seg = sla.sla_backward_workspace_bytes(_ok_params(B=B, T=T, H=H, dk=dk, dv=dv, segments=nseg))
    packed = sla.sla_backward_varlen_workspace_bytes(_ok_params(B=B * nseg, T=B * T, H=H, dk=dk, dv=dv))
    state = H * dk * dv
    forward_ws = B * H * (nseg * dk * dv + (nseg - 1) * 8 * dk)      # entry states, partial decay products
    extra = forward_ws + B * (nseg - 1) * H * dk + 2 * B * nseg * state + (B * nseg + 1 + 3) // 4 * 4
    assert seg == packed + 4 * extra and seg > one
    # a request that yields a single segment is the plain pass
    assert sla.sla_backward_workspace_bytes(_ok_params(B=B, T=200, H=H, dk=dk, dv=dv, segments=4)) == \
        sla.sla_backward_workspace_bytes(_ok_params(B=B, T=200, H=H, dk=dk, dv=dv))
    hm = _ok_params(flags=1, segments=2, T=1024)
    assert _bwd(hm, ws_bytes=1 << 40) == -3                   # segments run as a packed batch: [B,T,H,d] only
    assert _bwd(_ok_params(segments=2, T=1024), ws_bytes=sla.sla_backward_workspace_bytes(_ok_params(T=1024))) == -6


def test_backward_gdn_varlen_validation_and_workspace(lib):
    ok = _ok_params(variant=sla.GDN)
    call = lambda p, cu=A: sla.sla_backward_gdn_varlen(p, A, A, A, A, A, A, A, cu, 0, A, 0, A, A, A, A, A, A, A, 0, A,
                                                       1 << 40, 0)
    assert call(ok, cu=0) == -1 and call(ok, cu=A + 2) == -4
    assert call(_ok_params(variant=sla.GLA)) == -3
    assert call(_ok_params(variant=sla.GDN, B=0), cu=0) == 0
    # sized by the total token count p->T, not B * T
    p, one = (_ok_params(variant=sla.GDN, dtype=sla.F32, B=5, T=1000),
              _ok_params(variant=sla.GDN, dtype=sla.F32, B=1, T=1000))
    planes = p.dk // 8
    assert sla.sla_backward_gdn_varlen_workspace_bytes(p) == \
        sla.sla_backward_gdn_workspace_bytes(one) + 4 * ((planes * 5 * p.H + 3) // 4 * 4 - (planes * p.H + 3) // 4 * 4)
    # (the bf16 sizes are spelled out in test_backward_gdn_workspace_size)


def test_backward_segment_recommendation(lib):
    # the narrowest sweep runs B * H * min(dk, dv) / 64 workgroups per segment
    assert sla.sla_backward_segments(_ok_params(B=8, T=2048, H=16, dk=128, dv=128), 256) == 1     # 256 workgroups
    assert sla.sla_backward_segments(_ok_params(B=8, T=4096, H=4, dk=128, dv=256), 256) == 4      # 64
    assert sla.sla_backward_segments(_ok_params(B=8, T=4096, H=8, dk=64, dv=128), 256) == 4       # 64
    assert sla.sla_backward_segments(_ok_params(B=1, T=512, H=2, dk=64, dv=64), 256) == 2         # segments >= 256 tokens
    assert sla.sla_backward_segments(_ok_params(variant=sla.GDN, B=1, T=4096, H=2), 256) == 1
    assert sla.sla_backward_segments(_ok_params(), 0) == -2 and sla.sla_backward_segments(None, 256) == -1


def test_static_entry_point_validates_before_any_device_work(lib):
    """sla_forward_static: the same host-side checks as sla_forward, and a segment request whose workspace would
    exceed the static buffer is refused before the device is touched."""
    assert sla.sla_static_scratch_bytes() == 16 << 20
    assert sla.sla_forward_static(None, A, A, A, A, A, A, 0, 0, A, A, 0) == -1
    assert sla.sla_forward_static(_ok_params(dk=96), A, A, A, A, A, A, 0, 0, A, A, 0) == -3
    assert sla.sla_forward_static(_ok_params(), A, A + 4, A, A, A, A, 0, 0, A, A, 0) == -4
    assert sla.sla_forward_static(_ok_params(B=0), 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0) == 0
    # 8 segments of a 64-head batch: 8 * 64 * 128 * 128 floats of entry states alone = 32 MiB > 16 MiB
    big = _ok_params(B=4, T=8192, H=16, segments=8)
    assert sla.sla_forward_static(big, A, A, A, A, A, A, 0, 0, A, A, 0) == -7


def test_narrow_keys(lib):
    """dk = 32 passes the forward's validation; the backward passes run it zero-padded to 64 (single pass only) with
    the padded copies in the workspace; the decode step takes it."""
    p = _ok_params(dk=32, dv=64)
    assert _call(p) == 0
    assert _bwd(p) in (0, -5)                                # valid: reaches the launch (no device here)
    assert _bwd(_ok_params(dk=32, dv=64, segments=2, T=1024)) == -3
    B, T, H, dv = 2, 128, 4, 64
    n = B * T * H
    for dt, es in ((sla.BF16, 2), (sla.F32, 4)):
        wide, state = n * 64 * es // 4, B * H * 64 * dv      # floats of a padded [rows,H,64] tensor and of a padded state
        for variant in (sla.GLA, sla.RETNET):
            narrow = sla.sla_backward_workspace_bytes(_ok_params(variant=variant, dtype=dt, B=B, T=T, H=H, dk=32, dv=dv))
            inner = sla.sla_backward_workspace_bytes(_ok_params(variant=variant, dtype=dt, B=B, T=T, H=H, dk=64, dv=dv))
            assert narrow == inner + 4 * (6 * wide + 3 * state)
        narrow = sla.sla_backward_gdn_workspace_bytes(_ok_params(variant=sla.GDN, dtype=dt, B=B, T=T, H=H, dk=32, dv=dv))
        inner = sla.sla_backward_gdn_workspace_bytes(_ok_params(variant=sla.GDN, dtype=dt, B=B, T=T, H=H, dk=64, dv=dv))
        assert narrow == inner + 4 * (4 * wide + 3 * state)
    assert sla.sla_backward_workspace_bytes(_ok_params(dk=32, dv=64, segments=2, T=1024)) == 0
    assert sla.sla_backward_segments(_ok_params(B=1, T=4096, H=2, dk=32, dv=64), 256) == 1
    args = (A, A, A, A, A, A, 0)
    assert sla.sla_decode_step(_ok_params(T=1, dk=32, dv=64), *args, A, A, 0) in (0, -5)  # valid: reaches the launch


def test_prologue_gradient_entry_points_validate(lib):
    fm = sla.sla_short_conv_silu_l2
    assert fm(sla.BF16, 2, 64, 256, 4, 64, 1e-6, A, A, A, 0) in (0, -5)  # valid: reaches the launch (no device here)
    assert fm(sla.BF16, 2, 64, 256, 4, 48, 1e-6, A, A, A, 0) == -3         # head width not built
    assert fm(sla.BF16, 2, 64, 200, 4, 64, 1e-6, A, A, A, 0) == -2         # channels not whole rows of 128
    assert fm(sla.BF16, 2, 64, 256, 5, 64, 1e-6, A, A, A, 0) == -3
    assert fm(sla.BF16, 2, 64, 256, 4, 64, -1.0, A, A, A, 0) == -2
    assert fm(sla.BF16, 2, 64, 256, 4, 0, 0.0, 0, A, A, 0) == -1
    assert fm(sla.BF16, 0, 64, 256, 4, 64, 1e-6, 0, 0, 0, 0) == 0
    bw = sla.sla_short_conv_silu_l2_backward
    need = sla.sla_short_conv_silu_l2_backward_workspace_bytes(2, 100, 256, 4)
    assert need == 2 * 2 * 256 * 4 * 4
    assert bw(sla.BF16, 2, 100, 256, 4, 64, 1e-6, A, A, A, A, A, A, need - 1, 0) == -6
    assert bw(sla.BF16, 2, 100, 256, 4, 64, 1e-6, A, A, A, A, 0, A, need, 0) == -1
    assert bw(sla.BF16, 2, 100, 256, 4, 64, 1e-6, A, A, A + 2, A, A, A, need, 0) == -4
    gl = sla.sla_gate_logits_backward
    p = _ok_params()
    n = sla.sla_gate_logits_backward_workspace_bytes(p)
    assert n > 0 and n % (4 * 128 * 4) == 0
    assert gl(p, A, A, A, A, A, A, n - 1, 0) == -6
    assert gl(p, A, A, 0, A, A, A, n, 0) == -1
    assert gl(_ok_params(dk=48), A, A, A, A, A, A, n, 0) == -3
    assert gl(_ok_params(B=0), 0, 0, 0, 0, 0, 0, 0, 0) == 0
