// SLA recurrent decode step for gfx950 (MI355X): Eq. 5-6 with the Sec. 5.1 recurrences for ONE token per
// (batch, head), the constant-memory inference form (Sec. 3.2, Recurrent Implementation; derived in Appendix A).
//
// The step reads and rewrites the whole state, 2 * dk * dv * 4 bytes per head against O(dk * dv) flops: it is
// HBM-bound, so the kernel is a streaming read-modify-write.  One workgroup of 256 threads per (batch, head);
// thread (rg, c4) owns four adjacent value columns of the rows rg, rg + NRG, rg + 2 NRG, ...: a wave touches
// whole 512-byte (dv = 128) row segments, every thread has all of its 16-byte loads in flight at once
// (64 KB per workgroup), and the state tile stays in registers between the read and the write -- also for the
// delta rule, whose write depends on a reduction (k S) over the whole tile.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sla.h"

namespace sla {

typedef __attribute__((ext_vector_type(4))) float d_f32x4;

namespace {

constexpr float kDecLog2e = 1.4426950408889634f;
constexpr int kDecThreads = 256;

struct DArgs {
    const void* q;
    const void* k;
    const void* v;
    const float* ql;
    const float* kl;
    const float* wq;        // fused gate projection: [H,dk] fp32 (then ql, kl are not read), else null
    const float* wk;        // [H,dk] fp32 or null (G^K = 1)
    const void* ld;
    const float* beta;
    float* state;
    void* out;
    int B, H;
};

__device__ __forceinline__ float dec_exp(float x) { return __builtin_amdgcn_exp2f(x * kDecLog2e); }

template <bool BF16>
__device__ __forceinline__ float load_elem(const void* p, size_t i) {
    if constexpr (BF16)
        return __uint_as_float((uint32_t)((const uint16_t*)p)[i] << 16);
    else
        return ((const float*)p)[i];
}

// N adjacent elements starting at element i (N a multiple of 4; the address is 8- or 16-byte aligned), as wide loads
template <bool BF16, int N>
__device__ __forceinline__ void load_run(const void* p, size_t i, float (&x)[N]) {
    if constexpr (BF16) {
        typedef __attribute__((ext_vector_type(2))) uint32_t u2;
#pragma unroll
        for (int e = 0; e < N; e += 4) {
            const u2 t = *(const u2*)((const uint16_t*)p + i + e);
            x[e] = __uint_as_float(t.x << 16);
            x[e + 1] = __uint_as_float(t.x & 0xffff0000u);
            x[e + 2] = __uint_as_float(t.y << 16);
            x[e + 3] = __uint_as_float(t.y & 0xffff0000u);
        }
    } else {
#pragma unroll
        for (int e = 0; e < N; e += 4) {
            const d_f32x4 t = *(const d_f32x4*)((const float*)p + i + e);
            x[e] = t[0]; x[e + 1] = t[1]; x[e + 2] = t[2]; x[e + 3] = t[3];
        }
    }
}

__device__ __forceinline__ uint32_t dec_pack_bf16(float lo, float hi) {
    typedef __attribute__((ext_vector_type(2))) __bf16 bf2;
    bf2 t;
    t.x = (__bf16)lo;
    t.y = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, t);
}

// softmax over the H logits of one batch row, evaluated for head h (Eq. 4); every lane of the wave returns it
__device__ __forceinline__ float decode_gate(const float* logits, int H, int h, int lane) {
    const float x = lane < H ? logits[lane] : -INFINITY;
    float m = x;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    float s = lane < H ? dec_exp(x - m) : 0.f;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) s += __shfl_xor(s, o);
    return dec_exp(logits[h] - m) / s;
}

template <bool BF16, int VAR, int DK, int DV>
__global__ __launch_bounds__(kDecThreads) void sla_decode_kernel(const DArgs a) {
    constexpr int NC4 = DV / 4;            // threads along a row
    constexpr int NRG = kDecThreads / NC4; // row groups
    constexpr int RPT = DK / NRG;          // rows per thread
    static_assert(DK % NRG == 0 && RPT >= 1, "rows divide among the row groups");
    __shared__ float red[NRG][DV];  // per-row-group partial sums over the state rows

    const int tid = threadIdx.x, lane = tid & 63;
    const int bh = blockIdx.x, b = bh / a.H, h = bh % a.H;
    const int c4 = tid % NC4, rg = tid / NC4;

    // the state tile of this thread: issue every load before anything waits for one (the gates, which need a
    // round trip of their own, are formed while these are in flight)
    d_f32x4* srow = (d_f32x4*)(a.state + (size_t)bh * DK * DV) + c4;
    d_f32x4 S[RPT];
#pragma unroll
    for (int i = 0; i < RPT; ++i) S[i] = srow[(size_t)(rg + NRG * i) * NC4];

    float gq, gk;
    if (a.wq) {
        // Fused gate projection (Eq. 4 needs the logits of every head of the token): TPH threads per head (16; 8 for
        // dk = 32), each thread DK/TPH >= 4 adjacent elements of q[b,h',:] . W_GQ[:,h'] and k[b,h',:] . W_GK[:,h'],
        // summed over the TPH threads with shuffles -- 2 H dk multiply-adds against the dk dv of the state update, and
        // one launch less in front of every decode step.
        __shared__ float lg[2][64];
        constexpr int TPH = DK >= 64 ? 16 : 8, EPT = DK / TPH;
        const int sub = tid % TPH;
        for (int h2 = tid / TPH; h2 < a.H; h2 += kDecThreads / TPH) {
            const size_t at = ((size_t)b * a.H + h2) * DK + sub * EPT, wat = (size_t)h2 * DK + sub * EPT;
            float xq[EPT], xk[EPT], wq[EPT], wk[EPT];
            load_run<BF16, EPT>(a.q, at, xq);
            load_run<false, EPT>(a.wq, wat, wq);
            if (a.wk) {
                load_run<BF16, EPT>(a.k, at, xk);
                load_run<false, EPT>(a.wk, wat, wk);
            }
            float sq = 0.f, sk = 0.f;
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                sq += xq[e] * wq[e];
                if (a.wk) sk += xk[e] * wk[e];
            }
#pragma unroll
            for (int o = TPH / 2; o >= 1; o >>= 1) {
                sq += __shfl_xor(sq, o);
                sk += __shfl_xor(sk, o);
            }
            if (sub == 0) {
                lg[0][h2] = sq;
                lg[1][h2] = sk;
            }
        }
        __syncthreads();
        gq = decode_gate(lg[0], a.H, h, lane);
        gk = a.wk ? decode_gate(lg[1], a.H, h, lane) : 1.f;
    } else {
        gq = decode_gate(a.ql + (size_t)b * a.H, a.H, h, lane);
        gk = a.kl ? decode_gate(a.kl + (size_t)b * a.H, a.H, h, lane) : 1.f;
    }

    float qd[RPT], kd[RPT], ad[RPT];
    float a_scalar = 1.f;
    if constexpr (VAR == SLA_RETNET) a_scalar = dec_exp(((const float*)a.ld)[h]);
    if constexpr (VAR == SLA_GDN) a_scalar = dec_exp(((const float*)a.ld)[bh]);
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
        const size_t d = (size_t)bh * DK + rg + NRG * i;
        qd[i] = load_elem<BF16>(a.q, d);
        kd[i] = load_elem<BF16>(a.k, d);
        ad[i] = VAR == SLA_GLA ? dec_exp(load_elem<BF16>(a.ld, d)) : a_scalar;
    }
    float v4[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) v4[j] = load_elem<BF16>(a.v, (size_t)bh * DV + 4 * c4 + j);

    // Sec. 5.1: the write.  RetNet / GLA: S <- a S + (G^K k)^T v.  Delta rule: Sb = a S, u = beta (G^K v - k Sb),
    // S <- Sb + k^T u, which needs k Sb over all rows first.
    float w4[4];  // what is added as k_d * w
    if constexpr (VAR == SLA_GDN) {
        float ks[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < RPT; ++i) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                S[i][j] *= a_scalar;
                ks[j] += kd[i] * S[i][j];
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) red[rg][4 * c4 + j] = ks[j];
        __syncthreads();
        const float bt = a.beta[bh];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float t = 0.f;
            for (int g = 0; g < NRG; ++g) t += red[g][4 * c4 + j];
            w4[j] = bt * (gk * v4[j] - t);
        }
        __syncthreads();
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) w4[j] = gk * v4[j];
    }

    float y[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float decayed = VAR == SLA_GDN ? S[i][j] : ad[i] * S[i][j];
            S[i][j] = decayed + kd[i] * w4[j];
            y[j] += qd[i] * S[i][j];  // Eq. 6: the read-out uses the updated state
        }
        srow[(size_t)(rg + NRG * i) * NC4] = S[i];
    }

    // out = G^Q (q S): sum the row groups
#pragma unroll
    for (int j = 0; j < 4; ++j) red[rg][4 * c4 + j] = y[j];
    __syncthreads();
    if (tid < DV / 2) {
        float o0 = 0.f, o1 = 0.f;
        for (int g = 0; g < NRG; ++g) {
            o0 += red[g][2 * tid];
            o1 += red[g][2 * tid + 1];
        }
        o0 *= gq;
        o1 *= gq;
        if constexpr (BF16)
            ((uint32_t*)a.out)[((size_t)bh * DV) / 2 + tid] = dec_pack_bf16(o0, o1);
        else
            ((float2*)a.out)[((size_t)bh * DV) / 2 + tid] = make_float2(o0, o1);
    }
}

template <bool BF16, int VAR, int DK>
int launch_dv(const DArgs& a, int dv, hipStream_t stream) {
    const dim3 grid((unsigned)(a.B * a.H)), block(kDecThreads);
    switch (dv) {
        case 64: hipLaunchKernelGGL((sla_decode_kernel<BF16, VAR, DK, 64>), grid, block, 0, stream, a); break;
        case 128: hipLaunchKernelGGL((sla_decode_kernel<BF16, VAR, DK, 128>), grid, block, 0, stream, a); break;
        case 256: hipLaunchKernelGGL((sla_decode_kernel<BF16, VAR, DK, 256>), grid, block, 0, stream, a); break;
        default: return SLA_ERR_UNSUPPORTED;
    }
    return hipGetLastError() == hipSuccess ? SLA_OK : SLA_ERR_HIP;
}

template <bool BF16, int VAR>
int launch_dk(const DArgs& a, int dk, int dv, hipStream_t stream) {
    switch (dk) {
        case 32: return launch_dv<BF16, VAR, 32>(a, dv, stream);
        case 64: return launch_dv<BF16, VAR, 64>(a, dv, stream);
        case 128: return launch_dv<BF16, VAR, 128>(a, dv, stream);
        default: return SLA_ERR_UNSUPPORTED;
    }
}

template <bool BF16>
int launch_var(const DArgs& a, int variant, int dk, int dv, hipStream_t stream) {
    switch (variant) {
        case SLA_RETNET: return launch_dk<BF16, SLA_RETNET>(a, dk, dv, stream);
        case SLA_GLA: return launch_dk<BF16, SLA_GLA>(a, dk, dv, stream);
        case SLA_GDN: return launch_dk<BF16, SLA_GDN>(a, dk, dv, stream);
        default: return SLA_ERR_UNSUPPORTED;
    }
}

}  // namespace

int launch_decode(const sla_params& p, const void* q, const void* k, const void* v, const float* ql, const float* kl,
                  const float* wq, const float* wk, const void* ld, const float* beta, float* state, void* out,
                  hipStream_t stream) {
    DArgs a;
    a.q = q; a.k = k; a.v = v; a.ql = ql; a.kl = kl; a.wq = wq; a.wk = wk; a.ld = ld; a.beta = beta; a.state = state;
    a.out = out;
    a.B = p.B; a.H = p.H;
    if (p.dtype == SLA_BF16) return launch_var<true>(a, p.variant, p.dk, p.dv, stream);
    return launch_var<false>(a, p.variant, p.dk, p.dv, stream);
}

}  // namespace sla
