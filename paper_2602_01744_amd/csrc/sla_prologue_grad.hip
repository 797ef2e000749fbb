// Gradients of what sits in front of the SLA mixer, and the feature map's optional L2 normalisation, for gfx950:
//
//   * gate projections (Eq. 4's scores, logits[b,t,h] = x[b,t,h,:] . W[:,h]): the mixer's backward returns the
//     cotangents of the logits; this adds their share to dq, dk (dx[b,t,h,:] += dlogits[b,t,h] W[:,h]) and sums
//     dW[:,h] = sum_{b,t} dlogits[b,t,h] x[b,t,h,:];
//   * the Gated DeltaNet blocks' feature map (Sec. 5.1, Model Configuration: short convolution, then SiLU), with
//     an optional division of every head's vector by sqrt(sum of squares + eps), forward and backward.
//
// All of it streams: a thread owns eight adjacent channels (16 bytes of a token row), a wave covers 1 KB of every
// row it touches.  Sums over tokens (dW, dw) are taken in two deterministic stages: every thread leaves the sum
// over its own tokens in the workspace, a second kernel adds those partial sums in a fixed order.  No atomics.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sla.h"

namespace sla {

namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t gu4;
typedef __attribute__((ext_vector_type(4))) float gf4;

constexpr int kGThreads = 256;
constexpr int kSeg = 64;  // tokens per thread of the convolution kernels
constexpr float kLog2e = 1.4426950408889634f;

template <bool BF16>
__device__ __forceinline__ void ld8(const void* x, size_t off, float* f) {
    if constexpr (BF16) {
        const gu4 v = *(const gu4*)((const uint16_t*)x + off);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(v[i] << 16);
            f[2 * i + 1] = __uint_as_float(v[i] & 0xffff0000u);
        }
    } else {
        const gf4 a = *(const gf4*)((const float*)x + off), b = *(const gf4*)((const float*)x + off + 4);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[i] = a[i];
            f[4 + i] = b[i];
        }
    }
}

template <bool BF16, bool STREAM>
__device__ __forceinline__ void st8(void* y, size_t off, const float* f) {
    if constexpr (BF16) {
        typedef __attribute__((ext_vector_type(2))) __bf16 gbf2;
        gu4 v;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            gbf2 t;
            t.x = (__bf16)f[2 * i];
            t.y = (__bf16)f[2 * i + 1];
            v[i] = __builtin_bit_cast(uint32_t, t);
        }
        if constexpr (STREAM)
            __builtin_nontemporal_store(v, (gu4*)((uint16_t*)y + off));
        else
            *(gu4*)((uint16_t*)y + off) = v;
    } else {
        if constexpr (STREAM) {
            __builtin_nontemporal_store(gf4{f[0], f[1], f[2], f[3]}, (gf4*)((float*)y + off));
            __builtin_nontemporal_store(gf4{f[4], f[5], f[6], f[7]}, (gf4*)((float*)y + off + 4));
        } else {
            *(gf4*)((float*)y + off) = gf4{f[0], f[1], f[2], f[3]};
            *(gf4*)((float*)y + off + 4) = gf4{f[4], f[5], f[6], f[7]};
        }
    }
}

template <int CTRL>
__device__ __forceinline__ float gdpp(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}

// Sum over the LPH adjacent lanes of a head (LPH = 4, 8 or 16, aligned inside a 16-lane row), left in every one
// of them: exchanges inside quads, then between the quads of a half row, then between the halves.
template <int LPH>
__device__ __forceinline__ float head_allsum(float s) {
    s += gdpp<0xB1>(s);                           // quad_perm [1,0,3,2]
    s += gdpp<0x4E>(s);                           // quad_perm [2,3,0,1]
    if constexpr (LPH >= 8) s += gdpp<0x141>(s);  // row_half_mirror
    if constexpr (LPH == 16) s += gdpp<0x140>(s); // row_mirror
    return s;
}

__device__ __forceinline__ float sigmoidf(float s) { return 1.f / (1.f + __builtin_amdgcn_exp2f(-s * kLog2e)); }

// ------------------------------------------------------------------------------------------------------------
// Feature map with the L2 option: y = silu(conv(x)), then every head (LPH lanes x 8 channels) divided by
// sqrt(sum of squares + eps).  LPH = 0: no normalisation.  Thread -> (batch row, 64-token segment, 8 channels);
// the lanes of a head sit in one 16-lane row and walk the same tokens in step.
// ------------------------------------------------------------------------------------------------------------
template <bool BF16, int K, int LPH>
__global__ __launch_bounds__(kGThreads) void sla_feature_map_kernel(const void* x, const float* w, void* y, int B, int T,
                                                                     int C, float eps) {
    const int groups = C / 8, segs = (T + kSeg - 1) / kSeg;
    const size_t idx = (size_t)blockIdx.x * kGThreads + threadIdx.x;
    const size_t total = (size_t)B * segs * groups;
    // threads past the end repeat the last one (so that the cross-lane sums stay defined) and store nothing
    const bool live = idx < total;
    const size_t id = live ? idx : total - 1;
    const int cg = (int)(id % groups), seg = (int)((id / groups) % segs), b = (int)(id / ((size_t)groups * segs));
    float wt[K][8];
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
        for (int i = 0; i < K; ++i) wt[i][c] = w[(size_t)(8 * cg + c) * K + i];
    const int t0 = seg * kSeg, t1 = min(T, t0 + kSeg);
    const size_t row0 = (size_t)b * T;
    float hist[K][8];
#pragma unroll
    for (int i = 0; i < K - 1; ++i) {
        const int t = t0 - (K - 1) + i;
        if (t >= 0) {
            ld8<BF16>(x, (row0 + t) * C + 8 * cg, hist[i + 1]);
        } else {
#pragma unroll
            for (int c = 0; c < 8; ++c) hist[i + 1][c] = 0.f;
        }
    }
    constexpr int U = 4;
    for (int tb = t0; tb < t0 + kSeg; tb += U) {  // every lane of a row runs the same trip count
        float in[U][8];
#pragma unroll
        for (int u = 0; u < U; ++u) ld8<BF16>(x, (row0 + min(tb + u, t1 - 1)) * C + 8 * cg, in[u]);
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int i = 0; i < K - 1; ++i)
#pragma unroll
                for (int c = 0; c < 8; ++c) hist[i][c] = hist[i + 1][c];
#pragma unroll
            for (int c = 0; c < 8; ++c) hist[K - 1][c] = in[u][c];
            float out[8], ss = 0.f;
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                float s = 0.f;
#pragma unroll
                for (int i = 0; i < K; ++i) s += wt[i][c] * hist[i][c];
                out[c] = s * sigmoidf(s);
                ss += out[c] * out[c];
            }
            if constexpr (LPH > 0) {
                const float r = __builtin_amdgcn_rsqf(head_allsum<LPH>(ss) + eps);
#pragma unroll
                for (int c = 0; c < 8; ++c) out[c] *= r;
            }
            if (live && tb + u < t1) st8<BF16, true>(y, (row0 + tb + u) * C + 8 * cg, out);
        }
    }
}

// ------------------------------------------------------------------------------------------------------------
// Its backward.  With s the convolution, a = silu(s), r = (sum_head a^2 + eps)^-1/2, y = a r:
//     da = r dy - a r^3 sum_head(a dy),   ds = da sigmoid(s) (1 + s (1 - sigmoid(s))),
//     dx[u] = sum_i w[i] ds[u + (K-1) - i],   dw[i] = sum_t ds[t] x[t - (K-1) + i].
// A thread recomputes s for its 64 tokens and for the K-1 tokens after them (whose ds reaches back into its
// segment), keeps the last K values of ds, and writes dx[u] once ds[u + K - 1] is known.  Its share of dw (own
// tokens only) goes to part[(b * segs + seg)][channel][tap].
// ------------------------------------------------------------------------------------------------------------
template <bool BF16, int K, int LPH>
__global__ __launch_bounds__(kGThreads) void sla_feature_map_bwd_kernel(const void* x, const float* w, const void* dy,
                                                                         void* dx, float* part, int B, int T, int C,
                                                                         float eps) {
    const int groups = C / 8, segs = (T + kSeg - 1) / kSeg;
    const size_t idx = (size_t)blockIdx.x * kGThreads + threadIdx.x;
    const size_t total = (size_t)B * segs * groups;
    const bool live = idx < total;
    const size_t id = live ? idx : total - 1;
    const int cg = (int)(id % groups), seg = (int)((id / groups) % segs), b = (int)(id / ((size_t)groups * segs));
    float wt[K][8];
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
        for (int i = 0; i < K; ++i) wt[i][c] = w[(size_t)(8 * cg + c) * K + i];
    const int t0 = seg * kSeg, t1 = min(T, t0 + kSeg);
    const size_t row0 = (size_t)b * T;
    float hist[K][8];  // hist[i] = x[t - (K-1) + i]
#pragma unroll
    for (int i = 0; i < K - 1; ++i) {
        const int t = t0 - (K - 1) + i;
        if (t >= 0) {
            ld8<BF16>(x, (row0 + t) * C + 8 * cg, hist[i + 1]);
        } else {
#pragma unroll
            for (int c = 0; c < 8; ++c) hist[i + 1][c] = 0.f;
        }
    }
    float dsh[K][8];  // dsh[j] = ds[t - (K-1) + j]: the last K values, dsh[K-1] the newest
    float dwacc[K][8];
#pragma unroll
    for (int i = 0; i < K; ++i)
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            dsh[i][c] = 0.f;
            dwacc[i][c] = 0.f;
        }
    // tokens t0 .. t0 + 63 + (K-1): beyond min(T, ...) the cotangent is zero (nothing flows back from there)
    for (int t = t0; t < t0 + kSeg + K - 1; ++t) {
        const bool inside = t < T;               // a real token (maybe of the next segment)
        const bool own = t < t1;                 // a token of this thread's segment
        const int tc = min(t, T - 1);
        float xin[8], g[8];
        ld8<BF16>(x, (row0 + tc) * C + 8 * cg, xin);
        ld8<BF16>(dy, (row0 + tc) * C + 8 * cg, g);
#pragma unroll
        for (int i = 0; i < K - 1; ++i)
#pragma unroll
            for (int c = 0; c < 8; ++c) hist[i][c] = hist[i + 1][c];
#pragma unroll
        for (int c = 0; c < 8; ++c) hist[K - 1][c] = xin[c];
        float s[8], sg[8], a[8], ss = 0.f, ag = 0.f;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            float acc = 0.f;
#pragma unroll
            for (int i = 0; i < K; ++i) acc += wt[i][c] * hist[i][c];
            s[c] = acc;
            sg[c] = sigmoidf(acc);
            a[c] = acc * sg[c];
            ss += a[c] * a[c];
            ag += a[c] * g[c];
        }
        float da[8];
        if constexpr (LPH > 0) {
            const float r = __builtin_amdgcn_rsqf(head_allsum<LPH>(ss) + eps);
            const float coef = r * r * r * head_allsum<LPH>(ag);
#pragma unroll
            for (int c = 0; c < 8; ++c) da[c] = r * g[c] - a[c] * coef;
        } else {
#pragma unroll
            for (int c = 0; c < 8; ++c) da[c] = g[c];
        }
#pragma unroll
        for (int i = 0; i < K - 1; ++i)
#pragma unroll
            for (int c = 0; c < 8; ++c) dsh[i][c] = dsh[i + 1][c];
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const float ds = inside ? da[c] * sg[c] * (1.f + s[c] * (1.f - sg[c])) : 0.f;
            dsh[K - 1][c] = ds;
            if (own) {
#pragma unroll
                for (int i = 0; i < K; ++i) dwacc[i][c] += ds * hist[i][c];
            }
        }
        // dx[u] for u = t - (K-1): ds[u + (K-1) - i] = dsh[K-1-i]
        const int u = t - (K - 1);
        if (live && u >= t0 && u < t1) {
            float o[8];
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                float acc = 0.f;
#pragma unroll
                for (int i = 0; i < K; ++i) acc += wt[i][c] * dsh[K - 1 - i][c];
                o[c] = acc;
            }
            st8<BF16, true>(dx, (row0 + u) * C + 8 * cg, o);
        }
    }
    if (live) {
        float* p = part + ((size_t)(b * segs + seg) * C + 8 * cg) * K;
#pragma unroll
        for (int c = 0; c < 8; ++c)
#pragma unroll
            for (int i = 0; i < K; ++i) p[c * K + i] = dwacc[i][c];
    }
}

// out[j] = sum_{n < nparts} part[n * stride + j]: the second stage of every sum over tokens.  A workgroup of 16
// waves owns 64 adjacent outputs; wave w adds the parts n = w, w + 16, ... (eight loads in flight), the sixteen
// sums meet in LDS and are added in wave order: a fixed order, so the result is bitwise reproducible.
constexpr int kSumWaves = 16;
__global__ __launch_bounds__(kSumWaves * 64) void sla_partial_sum_kernel(const float* part, float* out, size_t stride,
                                                                         int nparts) {
    __shared__ float red[kSumWaves][64];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const size_t j = (size_t)blockIdx.x * 64 + lane;
    float acc = 0.f;
    if (j < stride) {
#pragma unroll 8
        for (int n = wv; n < nparts; n += kSumWaves) acc += part[(size_t)n * stride + j];
    }
    red[wv][lane] = acc;
    __syncthreads();
    if (wv == 0 && j < stride) {
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < kSumWaves; ++w) s += red[w][lane];
        out[j] = s;
    }
}

// ------------------------------------------------------------------------------------------------------------
// Backward of the gate projections.  Layout as in the forward kernel: a wave owns a fixed group of heads (lane l
// holds eight adjacent elements of head l / (dk/8) of the group) and a stripe of tokens; dx is updated in place,
// the wave's share of dW stays in registers until the end and goes to part[stripe][H][dk].
// ------------------------------------------------------------------------------------------------------------
template <bool BF16, int DK>
__global__ __launch_bounds__(kGThreads) void sla_gate_logits_bwd_kernel(const void* x, const float* w, const float* dl,
                                                                         void* dx, float* part, size_t rows, int H,
                                                                         int groups) {
    constexpr int LPH = DK / 8, HPW = 64 / LPH;
    const int lane = threadIdx.x & 63;
    const size_t wave = ((size_t)blockIdx.x * kGThreads + threadIdx.x) >> 6;
    const size_t nwaves = ((size_t)gridDim.x * kGThreads) >> 6;
    const int grp = (int)(wave % groups);
    const size_t stripe = wave / groups, nstripes = nwaves / groups;
    if (stripe >= nstripes) return;
    const int h = grp * HPW + lane / LPH, e = lane % LPH;
    const bool live = h < H;
    const int hc = live ? h : H - 1;
    float wr[8], acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        wr[i] = w[(size_t)hc * DK + 8 * e + i];
        acc[i] = 0.f;
    }
    const size_t row_elems = (size_t)H * DK;
    const int off = hc * DK + 8 * e;
    constexpr int U = 4;  // rows in flight per wave
    for (size_t r0 = stripe * U; r0 < rows; r0 += nstripes * U) {
        float xin[U][8], din[U][8], g[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t r = r0 + u < rows ? r0 + u : rows - 1;  // past the end: a repeat, weighted zero, not stored
            ld8<BF16>(x, r * row_elems + off, xin[u]);
            ld8<BF16>(dx, r * row_elems + off, din[u]);
            g[u] = r0 + u < rows ? dl[r * H + hc] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                acc[i] += g[u] * xin[u][i];
                din[u][i] += g[u] * wr[i];
            }
            if (live && r0 + u < rows) st8<BF16, false>(dx, (r0 + u) * row_elems + off, din[u]);
        }
    }
    if (live) {
        float* p = part + (stripe * H + h) * DK + 8 * e;
        *(gf4*)p = gf4{acc[0], acc[1], acc[2], acc[3]};
        *(gf4*)(p + 4) = gf4{acc[4], acc[5], acc[6], acc[7]};
    }
}

template <bool BF16, int K>
int feature_map_lph(int lph, bool bwd, dim3 grid, hipStream_t st, const void* x, const float* w, const void* dy, void* out,
                    float* part, int B, int T, int C, float eps) {
#define SLA_FM(LPH)                                                                                                  \
    if (bwd)                                                                                                         \
        hipLaunchKernelGGL((sla_feature_map_bwd_kernel<BF16, K, LPH>), grid, dim3(kGThreads), 0, st, x, w, dy, out,  \
                           part, B, T, C, eps);                                                                      \
    else                                                                                                             \
        hipLaunchKernelGGL((sla_feature_map_kernel<BF16, K, LPH>), grid, dim3(kGThreads), 0, st, x, w, out, B, T, C, \
                           eps);                                                                                     \
    break;
    switch (lph) {
        case 0: SLA_FM(0)
        case 4: SLA_FM(4)
        case 8: SLA_FM(8)
        case 16: SLA_FM(16)
        default: return SLA_ERR_UNSUPPORTED;
    }
#undef SLA_FM
    return hipGetLastError() == hipSuccess ? SLA_OK : SLA_ERR_HIP;
}

template <bool BF16>
int feature_map_taps(int taps, int lph, bool bwd, dim3 grid, hipStream_t st, const void* x, const float* w, const void* dy,
                     void* out, float* part, int B, int T, int C, float eps) {
    switch (taps) {
        case 1: return feature_map_lph<BF16, 1>(lph, bwd, grid, st, x, w, dy, out, part, B, T, C, eps);
        case 2: return feature_map_lph<BF16, 2>(lph, bwd, grid, st, x, w, dy, out, part, B, T, C, eps);
        case 3: return feature_map_lph<BF16, 3>(lph, bwd, grid, st, x, w, dy, out, part, B, T, C, eps);
        case 4: return feature_map_lph<BF16, 4>(lph, bwd, grid, st, x, w, dy, out, part, B, T, C, eps);
        default: return SLA_ERR_UNSUPPORTED;
    }
}

int sum_partials(const float* part, float* out, size_t stride, int nparts, hipStream_t st) {
    hipLaunchKernelGGL(sla_partial_sum_kernel, dim3((unsigned)((stride + 63) / 64)), dim3(kSumWaves * 64), 0, st, part,
                       out, stride, nparts);
    return hipGetLastError() == hipSuccess ? SLA_OK : SLA_ERR_HIP;
}

}  // namespace

// Segments of 64 tokens per batch row: the number of partial sums of dw is B times this.
size_t feature_map_partials(int B, int T) { return (size_t)B * ((T + kSeg - 1) / kSeg); }

int launch_feature_map(int dtype, int B, int T, int C, int taps, int head_width, float eps, const void* x, const float* w,
                       void* y, hipStream_t stream) {
    const size_t threads = feature_map_partials(B, T) * (C / 8);
    const dim3 grid((unsigned)((threads + kGThreads - 1) / kGThreads));
    if (dtype == SLA_BF16)
        return feature_map_taps<true>(taps, head_width / 8, false, grid, stream, x, w, nullptr, y, nullptr, B, T, C, eps);
    return feature_map_taps<false>(taps, head_width / 8, false, grid, stream, x, w, nullptr, y, nullptr, B, T, C, eps);
}

int launch_feature_map_backward(int dtype, int B, int T, int C, int taps, int head_width, float eps, const void* x,
                                const float* w, const void* dy, void* dx, float* dw, float* workspace,
                                hipStream_t stream) {
    const size_t nparts = feature_map_partials(B, T), threads = nparts * (C / 8);
    const dim3 grid((unsigned)((threads + kGThreads - 1) / kGThreads));
    const int rc = dtype == SLA_BF16 ? feature_map_taps<true>(taps, head_width / 8, true, grid, stream, x, w, dy, dx,
                                                              workspace, B, T, C, eps)
                                     : feature_map_taps<false>(taps, head_width / 8, true, grid, stream, x, w, dy, dx,
                                                               workspace, B, T, C, eps);
    if (rc != SLA_OK) return rc;
    return sum_partials(workspace, dw, (size_t)C * taps, (int)nparts, stream);
}

// Stripes of tokens the gate projections' backward cuts the batch into (= partial sums of dW per gate).
int gate_logits_backward_stripes(const sla_params& p) {
    const size_t rows = (size_t)p.B * p.T;
    const size_t quads = (rows + 3) / 4;  // a stripe walks four rows at a time
    return (int)(quads < 1024 ? (quads ? quads : 1) : 1024);
}

int launch_gate_logits_backward(const sla_params& p, const void* x, const float* w, const float* dl, void* dx, float* dw,
                                float* workspace, hipStream_t stream) {
    const size_t rows = (size_t)p.B * p.T;
    const int hpw = 64 / (p.dk / 8), groups = (p.H + hpw - 1) / hpw;
    const int stripes = gate_logits_backward_stripes(p);
    const size_t waves = (size_t)stripes * groups, blocks = (waves * 64 + kGThreads - 1) / kGThreads;
    // the grid holds a whole number of waves per block: pad the stripe count seen by the kernel to what the grid has
    const dim3 grid((unsigned)blocks);
    const bool bf = p.dtype == SLA_BF16;
#define SLA_GL(DK)                                                                                                     \
    if (bf)                                                                                                            \
        hipLaunchKernelGGL((sla_gate_logits_bwd_kernel<true, DK>), grid, dim3(kGThreads), 0, stream, x, w, dl, dx,     \
                           workspace, rows, p.H, groups);                                                              \
    else                                                                                                               \
        hipLaunchKernelGGL((sla_gate_logits_bwd_kernel<false, DK>), grid, dim3(kGThreads), 0, stream, x, w, dl, dx,    \
                           workspace, rows, p.H, groups);                                                              \
    break;
    switch (p.dk) {
        case 32: SLA_GL(32)
        case 64: SLA_GL(64)
        case 128: SLA_GL(128)
        default: return SLA_ERR_UNSUPPORTED;
    }
#undef SLA_GL
    if (hipGetLastError() != hipSuccess) return SLA_ERR_HIP;
    // the kernel ran nwaves / groups stripes
    const int nstripes = (int)((blocks * kGThreads / 64) / groups);
    return sum_partials(workspace, dw, (size_t)p.H * p.dk, nstripes, stream);
}

// Floats of workspace for nstripes as the launcher will see them.
size_t gate_logits_backward_workspace_floats(const sla_params& p) {
    const int hpw = 64 / (p.dk / 8), groups = (p.H + hpw - 1) / hpw;
    const size_t waves = (size_t)gate_logits_backward_stripes(p) * groups;
    const size_t blocks = (waves * 64 + kGThreads - 1) / kGThreads;
    return ((blocks * kGThreads / 64) / groups) * (size_t)p.H * p.dk;
}

}  // namespace sla
