// SLA chunkwise-parallel forward for gfx950 (MI355X): host-side launch of the kernels in sla_fwd_kernels.h
// (argument block, workspace layout of the segment-parallel schedule, dispatch by element type).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sla.h"
#include "sla_fwd_args.h"

namespace sla {

int dispatch_forward_bf16(const KArgs& a, int variant, int dk, int dvw, hipStream_t stream);
int dispatch_forward_f32(const KArgs& a, int variant, int dk, int dvw, hipStream_t stream);
unsigned int* device_status_word();  // sla_api.hip

// T == 0: the state passes through unchanged.
__global__ void sla_state_passthrough_kernel(const float* s0, float* sT, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) sT[i] = s0 ? s0[i] : 0.f;
}

// Floats of workspace the segment-parallel schedule needs for nseg segments.
size_t segment_workspace_floats(const sla_params& p, int nseg) {
    if (nseg <= 1) return 0;
    const size_t heads = (size_t)p.B * p.H;
    return heads * nseg * p.dk * p.dv + heads * (nseg - 1) * kMaxSlots * p.dk;  // entry states, decay products
}

int launch_forward(const sla_params& p, int dvw, int nseg, int seg_len, const void* q, const void* k, const void* v,
                   const float* ql, const float* kl, const void* ld, const float* beta, const float* s0, void* out,
                   float* sT, float* workspace, const int* cu, hipStream_t stream) {
    KArgs a;
    a.head_major = (p.flags & SLA_FLAG_HEAD_MAJOR) != 0;
    a.q = q; a.k = k; a.v = v; a.ql = ql; a.kl = kl; a.ld = ld; a.beta = beta; a.s0 = s0; a.out = out; a.sT = sT;
    a.B = p.B; a.T = p.T; a.H = p.H; a.dv = p.dv; a.nslice = p.dv / dvw;
    a.nseg = nseg; a.nseg_grid = nseg; a.nparts = 0; a.Ls = nseg > 1 ? seg_len : p.T;
    a.ws_state = workspace;
    a.ws_decay = workspace ? workspace + (size_t)p.B * nseg * p.H * p.dk * p.dv : nullptr;
    a.ws_total = nullptr;
    a.states_only = false;
    a.cu = cu;
    a.status = device_status_word();
    if (!a.status) return SLA_ERR_HIP;
    if (p.T == 0) {
        if (!sT) return SLA_OK;
        const size_t n = (size_t)p.B * p.H * p.dk * p.dv;
        hipLaunchKernelGGL(sla_state_passthrough_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, s0, sT, n);
        return hipGetLastError() == hipSuccess ? SLA_OK : SLA_ERR_HIP;
    }
    if (p.dtype == SLA_BF16) return dispatch_forward_bf16(a, p.variant, p.dk, dvw, stream);
    return dispatch_forward_f32(a, p.variant, p.dk, dvw, stream);
}

// The first two steps of the segment-parallel schedule alone (RetNet, GLA; nseg >= 2; rectangular batch): on return
// (in stream order) workspace holds the state entering every segment, [B * nseg][H][dk][dv], followed by scratch of
// the pre-pass, and totals the decay of every segment but the last, [B][nseg - 1][H][dk].  workspace needs
// segment_workspace_floats(p, nseg) floats.
int launch_segment_states(const sla_params& p, int dvw, int nseg, int seg_len, const void* q, const void* k,
                          const void* v, const float* ql, const float* kl, const void* ld, const float* s0,
                          float* workspace, float* totals, hipStream_t stream) {
    if (nseg < 2 || p.variant == SLA_GDN || p.T == 0) return SLA_ERR_UNSUPPORTED;
    KArgs a;
    a.head_major = false;
    a.q = q; a.k = k; a.v = v; a.ql = ql; a.kl = kl; a.ld = ld; a.beta = nullptr; a.s0 = s0; a.out = nullptr;
    a.sT = nullptr;
    a.B = p.B; a.T = p.T; a.H = p.H; a.dv = p.dv; a.nslice = p.dv / dvw;
    a.nseg = nseg; a.nseg_grid = nseg; a.nparts = 0; a.Ls = seg_len;
    a.ws_state = workspace;
    a.ws_decay = workspace + (size_t)p.B * nseg * p.H * p.dk * p.dv;
    a.ws_total = totals;
    a.states_only = true;
    a.cu = nullptr;
    a.status = device_status_word();
    if (!a.status) return SLA_ERR_HIP;
    if (p.dtype == SLA_BF16) return dispatch_forward_bf16(a, p.variant, p.dk, dvw, stream);
    return dispatch_forward_f32(a, p.variant, p.dk, dvw, stream);
}

}  // namespace sla
