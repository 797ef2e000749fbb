// Gate logits for gfx950 (MI355X): the scores that Eq. 4 takes the head softmax of,
//     q_head_logits[b,t,h] = q[b,t,h,:] . W_GQ[:,h],      k_head_logits[b,t,h] = k[b,t,h,:] . W_GK[:,h],
// with W in R^{d x H} and d the head width (the reading under which the two matrices add the 0.05 M parameters
// the "Parameter Efficiency" paragraph of Sec. 3.2 counts for the 24-layer, hidden-1024 model).
//
// One pass over q and k: 2 flops per byte, so the kernel is a streaming read.  A wave owns a fixed group of
// heads and walks the tokens: lane l holds eight adjacent elements (16 bytes) of head (l / (dk/8)) of the group,
// its eight weights stay in registers for the whole walk, the 64 lanes of a load cover 1 KB of one token's row,
// and the dk/8 partial sums of a head meet by DPP adds inside a 16-lane row.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sla.h"

namespace sla {

namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t pu4;
typedef __attribute__((ext_vector_type(4))) float pf4;

constexpr int kPThreads = 256;
constexpr int kPUnroll = 4;  // tokens in flight per wave and tensor

template <int CTRL>
__device__ __forceinline__ float pdpp(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}

template <bool BF16, int DK>
__device__ __forceinline__ float dot8(const void* row, int off, const float* w) {
    float s = 0.f;
    if constexpr (BF16) {
        const pu4 x = *(const pu4*)((const uint16_t*)row + off);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            s += __uint_as_float(x[i] << 16) * w[2 * i];
            s += __uint_as_float(x[i] & 0xffff0000u) * w[2 * i + 1];
        }
    } else {
        const pf4 x0 = *(const pf4*)((const float*)row + off), x1 = *(const pf4*)((const float*)row + off + 4);
#pragma unroll
        for (int i = 0; i < 4; ++i) s += x0[i] * w[i] + x1[i] * w[4 + i];
    }
    return s;
}

// sum over the LPH adjacent lanes of one head (LPH = 8 or 16, aligned inside a 16-lane row); valid in the last lane
template <int LPH>
__device__ __forceinline__ float head_sum(float s) {
    s += pdpp<0x111>(s);
    s += pdpp<0x112>(s);
    s += pdpp<0x114>(s);
    if constexpr (LPH == 16) s += pdpp<0x118>(s);
    return s;
}

template <bool BF16, int DK>
__global__ __launch_bounds__(kPThreads) void sla_gate_logits_kernel(const void* q, const void* k, const float* wq,
                                                                     const float* wk, float* ql, float* kl,
                                                                     size_t rows, int H, int groups) {
    constexpr int LPH = DK / 8;    // lanes per head
    constexpr int HPW = 64 / LPH;  // heads per wave
    const int lane = threadIdx.x & 63;
    const size_t wave = ((size_t)blockIdx.x * kPThreads + threadIdx.x) >> 6;
    const size_t nwaves = ((size_t)gridDim.x * kPThreads) >> 6;
    // wave -> (head group, token stripe): all waves of a stripe walk the same tokens, one group each
    const int grp = (int)(wave % groups);
    const size_t stripe = wave / groups, nstripes = nwaves / groups;
    if (stripe >= nstripes) return;
    const int h = grp * HPW + lane / LPH, e = lane % LPH;
    const bool live = h < H;
    const int hc = live ? h : H - 1;  // lanes past the last head repeat it and store nothing
    float wqr[8], wkr[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        wqr[i] = wq[(size_t)hc * DK + 8 * e + i];
        wkr[i] = k ? wk[(size_t)hc * DK + 8 * e + i] : 0.f;
    }
    const size_t es = BF16 ? 2 : 4, row_bytes = (size_t)H * DK * es;
    const int off = hc * DK + 8 * e;
    const bool writer = live && e == LPH - 1;
    for (size_t r0 = stripe * kPUnroll; r0 < rows; r0 += nstripes * kPUnroll) {
        float sq[kPUnroll], sk[kPUnroll];
#pragma unroll
        for (int u = 0; u < kPUnroll; ++u) {
            const size_t r = r0 + u < rows ? r0 + u : rows - 1;
            sq[u] = dot8<BF16, DK>((const char*)q + r * row_bytes, off, wqr);
            sk[u] = k ? dot8<BF16, DK>((const char*)k + r * row_bytes, off, wkr) : 0.f;
        }
#pragma unroll
        for (int u = 0; u < kPUnroll; ++u) {
            const float a = head_sum<LPH>(sq[u]), b = head_sum<LPH>(sk[u]);
            if (writer && r0 + u < rows) {
                ql[(r0 + u) * H + h] = a;
                if (k) kl[(r0 + u) * H + h] = b;
            }
        }
    }
}

template <bool BF16>
int launch_dk(int dk, dim3 grid, hipStream_t stream, const void* q, const void* k, const float* wq, const float* wk,
              float* ql, float* kl, size_t rows, int H, int groups) {
    switch (dk) {
        case 64:
            hipLaunchKernelGGL((sla_gate_logits_kernel<BF16, 64>), grid, dim3(kPThreads), 0, stream, q, k, wq, wk, ql,
                               kl, rows, H, groups);
            break;
        case 128:
            hipLaunchKernelGGL((sla_gate_logits_kernel<BF16, 128>), grid, dim3(kPThreads), 0, stream, q, k, wq, wk, ql,
                               kl, rows, H, groups);
            break;
        default: return SLA_ERR_UNSUPPORTED;
    }
    return hipGetLastError() == hipSuccess ? SLA_OK : SLA_ERR_HIP;
}

}  // namespace

int launch_gate_logits(const sla_params& p, const void* q, const void* k, const float* wq, const float* wk, float* ql,
                       float* kl, int compute_units, hipStream_t stream) {
    const size_t rows = (size_t)p.B * p.T;
    const int heads_per_wave = 64 / (p.dk / 8);
    const int groups = (p.H + heads_per_wave - 1) / heads_per_wave;
    // enough waves to fill the device several times over, a whole number of stripes, never more stripes than
    // there are token quads
    size_t stripes = ((size_t)compute_units * 32 + groups - 1) / groups;
    const size_t quads = (rows + kPUnroll - 1) / kPUnroll;
    if (stripes > quads) stripes = quads;
    const size_t waves = stripes * groups, blocks = (waves * 64 + kPThreads - 1) / kPThreads;
    const dim3 grid((unsigned)blocks);
    if (p.dtype == SLA_BF16) return launch_dk<true>(p.dk, grid, stream, q, k, wq, wk, ql, kl, rows, p.H, groups);
    return launch_dk<false>(p.dk, grid, stream, q, k, wq, wk, ql, kl, rows, p.H, groups);
}

}  // namespace sla
