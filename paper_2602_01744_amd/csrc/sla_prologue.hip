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

// sum over the LPH adjacent lanes of one head (LPH = 4, 8 or 16, aligned inside a 16-lane row); valid in the last lane
template <int LPH>
__device__ __forceinline__ float head_sum(float s) {
    s += pdpp<0x111>(s);
    s += pdpp<0x112>(s);
    if constexpr (LPH >= 8) s += pdpp<0x114>(s);
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
        case 32:
            hipLaunchKernelGGL((sla_gate_logits_kernel<BF16, 32>), grid, dim3(kPThreads), 0, stream, q, k, wq, wk, ql,
                               kl, rows, H, groups);
            break;
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

// ------------------------------------------------------------------------------------------------------------
// Short causal convolution along the tokens followed by SiLU, per channel: the feature map Sec. 5.1 ("Model
// Configuration") names for the Gated DeltaNet blocks in front of q, k (and v),
//     y[b,t,c] = silu( sum_{i < K} w[c,i] * x[b, t - (K-1) + i, c] ),    x = 0 before the sequence.
// A streaming kernel: one thread owns eight adjacent channels (16 bytes of a token row) and walks a segment of
// 64 tokens with the last K-1 inputs in registers; a wave covers 1 KB of every token row it touches.
// ------------------------------------------------------------------------------------------------------------
constexpr int kConvSeg = 64;   // tokens per thread
constexpr int kConvMaxTaps = 4;

template <bool BF16>
__device__ __forceinline__ void load8(const void* x, size_t off, float* f) {
    if constexpr (BF16) {
        const pu4 v = *(const pu4*)((const uint16_t*)x + off);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(v[i] << 16);
            f[2 * i + 1] = __uint_as_float(v[i] & 0xffff0000u);
        }
    } else {
        const pf4 a = *(const pf4*)((const float*)x + off), b = *(const pf4*)((const float*)x + off + 4);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[i] = a[i];
            f[4 + i] = b[i];
        }
    }
}

template <bool BF16>
__device__ __forceinline__ void store8(void* y, size_t off, const float* f) {
    if constexpr (BF16) {
        typedef __attribute__((ext_vector_type(2))) __bf16 pbf2;
        pu4 v;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            pbf2 t;
            t.x = (__bf16)f[2 * i];
            t.y = (__bf16)f[2 * i + 1];
            v[i] = __builtin_bit_cast(uint32_t, t);
        }
        __builtin_nontemporal_store(v, (pu4*)((uint16_t*)y + off));
    } else {
        __builtin_nontemporal_store(pf4{f[0], f[1], f[2], f[3]}, (pf4*)((float*)y + off));
        __builtin_nontemporal_store(pf4{f[4], f[5], f[6], f[7]}, (pf4*)((float*)y + off + 4));
    }
}

template <bool BF16, int K>
__global__ __launch_bounds__(kPThreads) void sla_short_conv_silu_kernel(const void* x, const float* w, void* y, int B,
                                                                         int T, int C) {
    const int groups = C / 8, segs = (T + kConvSeg - 1) / kConvSeg;
    const size_t idx = (size_t)blockIdx.x * kPThreads + threadIdx.x;
    if (idx >= (size_t)B * segs * groups) return;
    const int cg = (int)(idx % groups), seg = (int)((idx / groups) % segs), b = (int)(idx / ((size_t)groups * segs));
    float wt[K][8];  // wt[i][c]: tap i of channel 8 cg + c
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
        for (int i = 0; i < K; ++i) wt[i][c] = w[(size_t)(8 * cg + c) * K + i];
    const int t0 = seg * kConvSeg, t1 = min(T, t0 + kConvSeg);
    const size_t row0 = (size_t)b * T;
    float hist[K][8];  // hist[i] = x[t - (K-1) + i] for the token t being produced
#pragma unroll
    for (int i = 0; i < K - 1; ++i) {
        const int t = t0 - (K - 1) + i;
        if (t >= 0) {
            load8<BF16>(x, (row0 + t) * C + 8 * cg, hist[i + 1]);
        } else {
#pragma unroll
            for (int c = 0; c < 8; ++c) hist[i + 1][c] = 0.f;
        }
    }
    // eight tokens at a time: their loads are issued together, before any of them is used
    constexpr int U = 8;
    for (int tb = t0; tb < t1; tb += U) {
        float in[U][8];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = min(tb + u, t1 - 1);  // past the segment: a repeat of its last token, never stored
            load8<BF16>(x, (row0 + t) * C + 8 * cg, in[u]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int i = 0; i < K - 1; ++i)
#pragma unroll
                for (int c = 0; c < 8; ++c) hist[i][c] = hist[i + 1][c];
#pragma unroll
            for (int c = 0; c < 8; ++c) hist[K - 1][c] = in[u][c];
            float out[8];
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                float s = 0.f;
#pragma unroll
                for (int i = 0; i < K; ++i) s += wt[i][c] * hist[i][c];
                out[c] = s / (1.f + __builtin_amdgcn_exp2f(-s * 1.4426950408889634f));  // silu(s) = s * sigmoid(s)
            }
            if (tb + u < t1) store8<BF16>(y, (row0 + tb + u) * C + 8 * cg, out);
        }
    }
}

template <bool BF16>
int launch_conv_taps(int taps, dim3 grid, hipStream_t stream, const void* x, const float* w, void* y, int B, int T,
                     int C) {
    switch (taps) {
        case 1: hipLaunchKernelGGL((sla_short_conv_silu_kernel<BF16, 1>), grid, dim3(kPThreads), 0, stream, x, w, y, B, T, C); break;
        case 2: hipLaunchKernelGGL((sla_short_conv_silu_kernel<BF16, 2>), grid, dim3(kPThreads), 0, stream, x, w, y, B, T, C); break;
        case 3: hipLaunchKernelGGL((sla_short_conv_silu_kernel<BF16, 3>), grid, dim3(kPThreads), 0, stream, x, w, y, B, T, C); break;
        case 4: hipLaunchKernelGGL((sla_short_conv_silu_kernel<BF16, 4>), grid, dim3(kPThreads), 0, stream, x, w, y, B, T, C); break;
        default: return SLA_ERR_UNSUPPORTED;
    }
    return hipGetLastError() == hipSuccess ? SLA_OK : SLA_ERR_HIP;
}

}  // namespace

int launch_short_conv_silu(int dtype, int B, int T, int C, int taps, const void* x, const float* w, void* y,
                           hipStream_t stream) {
    const size_t threads = (size_t)B * ((T + kConvSeg - 1) / kConvSeg) * (C / 8);
    const dim3 grid((unsigned)((threads + kPThreads - 1) / kPThreads));
    if (dtype == SLA_BF16) return launch_conv_taps<true>(taps, grid, stream, x, w, y, B, T, C);
    return launch_conv_taps<false>(taps, grid, stream, x, w, y, B, T, C);
}

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
