// Backward passes for key heads of width 32 (the H = 16 point of the head-count ablation, Sec. 5.6, at fixed model
// width).  The backward sweeps slice the key dimension 64 columns to a workgroup, so a 32-wide head runs as a 64-wide
// one whose upper 32 key dimensions are zero: q, k, the GLA log-decay and the states are copied into zero-padded
// buffers in the workspace, the 64-wide pass runs on them, and dq, dk, the decay gradient and the state gradient are
// copied back.  Padded dimensions contribute nothing (q . k over them is zero, their decay factor is exp(0) = 1, their
// state rows stay zero), so the results are those of the 32-wide problem; the price is twice the key-side work and
// the copies.  Value heads are untouched.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sla.h"

namespace sla {

size_t backward_workspace_floats(const sla_params& p, bool packed);
int launch_backward(const sla_params& p, const void* q, const void* k, const void* v, const float* ql, const float* kl,
                    const void* ld, const float* s0, const void* dout, const float* dsf, void* dq, void* dk, void* dv,
                    float* dql, float* dkl, void* dld, float* ds0, float* ws, const int* cu, hipStream_t stream);
size_t backward_gdn_workspace_floats(const sla_params& p, bool packed);
int launch_backward_gdn(const sla_params& p, const void* q, const void* k, const void* v, const float* ql,
                        const float* kl, const float* ld, const float* beta, const float* s0, const void* dout,
                        const float* dsf, void* dq, void* dk, void* dv, float* dql, float* dkl, float* dld,
                        float* dbeta, float* ds0, float* ws, const int* cu, hipStream_t stream);

namespace {

constexpr int kNarrow = 32, kWide = 64, kEw = 256;

// A tensor seen as `count` pieces of `per` 16-byte units: dst gets each piece followed by as many zero units.
__global__ __launch_bounds__(kEw) void pad_halves_kernel(const uint4* src, uint4* dst, size_t count, unsigned per) {
    const size_t i = (size_t)blockIdx.x * kEw + threadIdx.x;
    if (i >= count * 2 * per) return;
    const size_t piece = i / (2 * per);
    const unsigned c = (unsigned)(i - piece * 2 * per);
    dst[i] = c < per ? src[piece * per + c] : uint4{0u, 0u, 0u, 0u};
}
// ... and back: the first half of every padded piece.
__global__ __launch_bounds__(kEw) void unpad_halves_kernel(const uint4* src, uint4* dst, size_t count, unsigned per) {
    const size_t i = (size_t)blockIdx.x * kEw + threadIdx.x;
    if (i >= count * per) return;
    const size_t piece = i / per;
    dst[i] = src[piece * 2 * per + (i - piece * per)];
}

int pad(const void* src, void* dst, size_t count, unsigned per, hipStream_t stream) {
    const size_t n = count * 2 * per;
    if (n == 0) return SLA_OK;
    hipLaunchKernelGGL(pad_halves_kernel, dim3((unsigned)((n + kEw - 1) / kEw)), dim3(kEw), 0, stream, (const uint4*)src,
                       (uint4*)dst, count, per);
    return hipGetLastError() == hipSuccess ? SLA_OK : SLA_ERR_HIP;
}
int unpad(const void* src, void* dst, size_t count, unsigned per, hipStream_t stream) {
    const size_t n = count * per;
    if (n == 0) return SLA_OK;
    hipLaunchKernelGGL(unpad_halves_kernel, dim3((unsigned)((n + kEw - 1) / kEw)), dim3(kEw), 0, stream,
                       (const uint4*)src, (uint4*)dst, count, per);
    return hipGetLastError() == hipSuccess ? SLA_OK : SLA_ERR_HIP;
}

struct Padded {  // what the wrappers carve out of the workspace behind the 64-wide pass's own part
    size_t rows_h;       // (token, head) rows
    size_t wide;         // floats of one padded wide tensor [rows, H, 64]
    size_t state;        // floats of one padded state [B, H, 64, dv]
    unsigned per_row;    // 16-byte units of a 32-element row
    unsigned per_state;  // 16-byte units of a [32, dv] fp32 state
};
Padded padded_sizes(const sla_params& p, bool packed) {
    Padded s;
    const size_t rows = packed ? (size_t)p.T : (size_t)p.B * p.T, es = p.dtype == SLA_BF16 ? 2 : 4;
    s.rows_h = rows * p.H;
    s.wide = s.rows_h * kWide * es / 4;
    s.state = (size_t)p.B * p.H * kWide * p.dv;
    s.per_row = (unsigned)(kNarrow * es / 16);
    s.per_state = (unsigned)(kNarrow * p.dv * 4 / 16);
    return s;
}
sla_params widened(const sla_params& p) {
    sla_params w = p;
    w.dk = kWide;
    return w;
}

}  // namespace

// Workspace of sla_backward / sla_backward_varlen in floats, any supported key width (no segment schedule).
size_t backward_any_workspace_floats(const sla_params& p, bool packed) {
    if (p.dk != kNarrow) return backward_workspace_floats(p, packed);
    const Padded s = padded_sizes(p, packed);
    return backward_workspace_floats(widened(p), packed) + 6 * s.wide + 3 * s.state;
}

int launch_backward_any(const sla_params& p, const void* q, const void* k, const void* v, const float* ql,
                        const float* kl, const void* ld, const float* s0, const void* dout, const float* dsf, void* dq,
                        void* dk, void* dv, float* dql, float* dkl, void* dld, float* ds0, float* ws, const int* cu,
                        bool packed, hipStream_t stream) {
    if (p.dk != kNarrow)
        return launch_backward(p, q, k, v, ql, kl, ld, s0, dout, dsf, dq, dk, dv, dql, dkl, dld, ds0, ws, cu, stream);
    const sla_params w = widened(p);
    const Padded s = padded_sizes(p, packed);
    const bool gla = p.variant == SLA_GLA;
    float* x = ws + backward_workspace_floats(w, packed);
    float* qp = x; x += s.wide;
    float* kp = x; x += s.wide;
    float* lp = x; x += s.wide;
    float* dqp = x; x += s.wide;
    float* dkp = x; x += s.wide;
    float* dlp = x; x += s.wide;
    float* s0p = x; x += s.state;
    float* dsfp = x; x += s.state;
    float* ds0p = x;
    const size_t heads = (size_t)p.B * p.H;
    int rc = pad(q, qp, s.rows_h, s.per_row, stream);
    if (rc == SLA_OK) rc = pad(k, kp, s.rows_h, s.per_row, stream);
    if (rc == SLA_OK && gla) rc = pad(ld, lp, s.rows_h, s.per_row, stream);
    if (rc == SLA_OK && s0) rc = pad(s0, s0p, heads, s.per_state, stream);
    if (rc == SLA_OK && dsf) rc = pad(dsf, dsfp, heads, s.per_state, stream);
    if (rc != SLA_OK) return rc;
    rc = launch_backward(w, qp, kp, v, ql, kl, gla ? (const void*)lp : ld, s0 ? s0p : nullptr, dout,
                         dsf ? dsfp : nullptr, dqp, dkp, dv, dql, dkl, gla ? (void*)dlp : nullptr, ds0 ? ds0p : nullptr,
                         ws, cu, stream);
    if (rc != SLA_OK) return rc;
    rc = unpad(dqp, dq, s.rows_h, s.per_row, stream);
    if (rc == SLA_OK) rc = unpad(dkp, dk, s.rows_h, s.per_row, stream);
    if (rc == SLA_OK && gla) rc = unpad(dlp, dld, s.rows_h, s.per_row, stream);
    if (rc == SLA_OK && ds0) rc = unpad(ds0p, ds0, heads, s.per_state, stream);
    return rc;
}

// The same for the gated delta rule (sla_backward_gdn, sla_backward_gdn_varlen).
size_t backward_gdn_any_workspace_floats(const sla_params& p, bool packed) {
    if (p.dk != kNarrow) return backward_gdn_workspace_floats(p, packed);
    const Padded s = padded_sizes(p, packed);
    return backward_gdn_workspace_floats(widened(p), packed) + 4 * s.wide + 3 * s.state;
}

int launch_backward_gdn_any(const sla_params& p, const void* q, const void* k, const void* v, const float* ql,
                            const float* kl, const float* ld, const float* beta, const float* s0, const void* dout,
                            const float* dsf, void* dq, void* dk, void* dv, float* dql, float* dkl, float* dld,
                            float* dbeta, float* ds0, float* ws, const int* cu, bool packed, hipStream_t stream) {
    if (p.dk != kNarrow)
        return launch_backward_gdn(p, q, k, v, ql, kl, ld, beta, s0, dout, dsf, dq, dk, dv, dql, dkl, dld, dbeta, ds0, ws,
                                   cu, stream);
    const sla_params w = widened(p);
    const Padded s = padded_sizes(p, packed);
    float* x = ws + backward_gdn_workspace_floats(w, packed);
    float* qp = x; x += s.wide;
    float* kp = x; x += s.wide;
    float* dqp = x; x += s.wide;
    float* dkp = x; x += s.wide;
    float* s0p = x; x += s.state;
    float* dsfp = x; x += s.state;
    float* ds0p = x;
    const size_t heads = (size_t)p.B * p.H;
    int rc = pad(q, qp, s.rows_h, s.per_row, stream);
    if (rc == SLA_OK) rc = pad(k, kp, s.rows_h, s.per_row, stream);
    if (rc == SLA_OK && s0) rc = pad(s0, s0p, heads, s.per_state, stream);
    if (rc == SLA_OK && dsf) rc = pad(dsf, dsfp, heads, s.per_state, stream);
    if (rc != SLA_OK) return rc;
    rc = launch_backward_gdn(w, qp, kp, v, ql, kl, ld, beta, s0 ? s0p : nullptr, dout, dsf ? dsfp : nullptr, dqp, dkp, dv,
                             dql, dkl, dld, dbeta, ds0 ? ds0p : nullptr, ws, cu, stream);
    if (rc != SLA_OK) return rc;
    rc = unpad(dqp, dq, s.rows_h, s.per_row, stream);
    if (rc == SLA_OK) rc = unpad(dkp, dk, s.rows_h, s.per_row, stream);
    if (rc == SLA_OK && ds0) rc = unpad(ds0p, ds0, heads, s.per_state, stream);
    return rc;
}

}  // namespace sla
