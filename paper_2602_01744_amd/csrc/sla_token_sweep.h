// Pieces shared by the token-by-token fp32 sweeps of the backward passes (the delta rule's fp32 path and the fp32 path
// of RetNet and GLA): the tile layout of a wave, the cross-lane sums, the staging of 16 tokens from global memory into
// LDS, and what a workgroup owns.
//
// Tile layout of a wave: lane = 16 * (column group) + (row group); a lane holds ROWS/16 rows by 2 columns of the tile,
// a wave 8 columns.  A product that contracts the rows is a per-lane partial sum followed by a rotate-and-add over the
// 16 lanes of a DPP row, which leaves the total in every lane.  A workgroup is eight such waves (64 columns, two waves
// per SIMD so that one computes while the other waits for the LDS) plus four loader waves that stage the next 16
// tokens (as fp32) into the other half of a double-buffered LDS area; one barrier per 16 tokens.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sla {
namespace tok {

typedef __attribute__((ext_vector_type(4))) float f4;
typedef __attribute__((ext_vector_type(4))) uint32_t u4;
typedef __attribute__((ext_vector_type(2))) uint32_t u2;
typedef __attribute__((ext_vector_type(2))) float fc;  // the CW columns of a lane

constexpr int kChunk = 16;          // tokens staged per barrier
constexpr int CW = 2;               // columns of the tile per lane
constexpr int kWaves = 8;           // compute waves (4 * CW columns each): two per SIMD, to hide each other's LDS latency
constexpr int kLoaders = 256;       // threads of the four loader waves
constexpr int kThreads = 64 * kWaves + kLoaders;
constexpr int kSlice = 4 * CW * kWaves;  // columns per workgroup
static_assert(CW == 2 && kSlice == 64, "the staging of the sliced tensors is sized for 64 columns");
constexpr int kEw = 256;
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ float bf_lo(uint32_t p) { return __uint_as_float(p << 16); }
__device__ __forceinline__ float bf_hi(uint32_t p) { return __uint_as_float(p & 0xffff0000u); }
typedef __attribute__((ext_vector_type(2))) __bf16 bf2;
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {  // the hardware conversion: nearest even, NaN kept
    bf2 t;
    t.x = (__bf16)lo;
    t.y = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, t);
}

template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
    return __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(x), CTRL, 0xf, 0xf, true));
}
// Sum over the 16 lanes of a DPP row (the row groups of a tile); every lane gets the total.
__device__ __forceinline__ float row_all(float x) {
    x += dpp_move<0x128>(x);  // row_ror:8
    x += dpp_move<0x124>(x);  // row_ror:4
    x += dpp_move<0x122>(x);  // row_ror:2
    x += dpp_move<0x121>(x);  // row_ror:1
    return x;
}
// Sum over the four DPP rows of the wave (the column groups); every lane gets the total.
__device__ __forceinline__ float all_groups(float x) {
    const uint32_t xi = __float_as_uint(x);
    const u2 a = __builtin_amdgcn_permlane16_swap(xi, xi, false, false);
    const uint32_t yi = __float_as_uint(__uint_as_float(a[0]) + __uint_as_float(a[1]));
    const u2 b = __builtin_amdgcn_permlane32_swap(yi, yi, false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// A token's row-side vector (length 16 * RT: the dimension the tile contracts) is stored so that the 16 lanes of a
// DPP row, which own RT consecutive elements each, read 16 consecutive 16-byte pieces per instruction (no bank
// conflicts): element c = rg * RT + 4 m + e sits at float m * 64 + rg * 4 + e.  `c` is a multiple of 4.
template <int RT>
__device__ __forceinline__ int row_slot(int c) {
    return ((c % RT) >> 2) * 64 + (c / RT) * 4;
}

// ---- staging: NC columns of 16 tokens of one head, global -> registers -> LDS (fp32 [16][NC]) ----------------
// Loads are unconditional (token clamped into the sequence) and zeroed when written; `lt` is the loader thread.
template <int NC>
struct RegsB {
    static constexpr int items = kChunk * NC / 8, N = (items + kLoaders - 1) / kLoaders;
    u4 x[N];
    __device__ __forceinline__ void load(const uint16_t* base, size_t tokstride, int t0, int T, int lt) {
#pragma unroll
        for (int n = 0; n < N; ++n) {
            const int it = min(lt + kLoaders * n, items - 1), tok = it / (NC / 8), c8 = it % (NC / 8);
            x[n] = *(const u4*)(base + (size_t)min(t0 + tok, T - 1) * tokstride + 8 * c8);
        }
    }
    __device__ __forceinline__ void put(float* dst, int t0, int T, int lt) const {
#pragma unroll
        for (int n = 0; n < N; ++n) {
            const int it = lt + kLoaders * n, tok = it / (NC / 8), c8 = it % (NC / 8);
            if (it < items) {
                const bool ok = t0 + tok < T;
                const u4 y = ok ? x[n] : u4{0u, 0u, 0u, 0u};
                float* d = dst + tok * NC + 8 * c8;
                *(f4*)d = f4{bf_lo(y[0]), bf_hi(y[0]), bf_lo(y[1]), bf_hi(y[1])};
                *(f4*)(d + 4) = f4{bf_lo(y[2]), bf_hi(y[2]), bf_lo(y[3]), bf_hi(y[3])};
            }
        }
    }
    // The same for a tensor whose columns are the ROWS of the tile: see row_slot().
    __device__ __forceinline__ void put_rows(float* dst, int t0, int T, int lt) const {
#pragma unroll
        for (int n = 0; n < N; ++n) {
            const int it = lt + kLoaders * n, tok = it / (NC / 8), c8 = it % (NC / 8);
            if (it < items) {
                const bool ok = t0 + tok < T;
                const u4 y = ok ? x[n] : u4{0u, 0u, 0u, 0u};
                float* d = dst + tok * NC;
                *(f4*)(d + row_slot<NC / 16>(8 * c8)) = f4{bf_lo(y[0]), bf_hi(y[0]), bf_lo(y[1]), bf_hi(y[1])};
                *(f4*)(d + row_slot<NC / 16>(8 * c8 + 4)) = f4{bf_lo(y[2]), bf_hi(y[2]), bf_lo(y[3]), bf_hi(y[3])};
            }
        }
    }
};
template <int NC>
struct RegsF {
    static constexpr int items = kChunk * NC / 4, N = (items + kLoaders - 1) / kLoaders;
    f4 x[N];
    __device__ __forceinline__ void load(const float* base, size_t tokstride, int t0, int T, int lt) {
#pragma unroll
        for (int n = 0; n < N; ++n) {
            const int it = min(lt + kLoaders * n, items - 1), tok = it / (NC / 4), c4 = it % (NC / 4);
            x[n] = *(const f4*)(base + (size_t)min(t0 + tok, T - 1) * tokstride + 4 * c4);
        }
    }
    __device__ __forceinline__ void put(float* dst, int t0, int T, int lt) const {
#pragma unroll
        for (int n = 0; n < N; ++n) {
            const int it = lt + kLoaders * n, tok = it / (NC / 4), c4 = it % (NC / 4);
            if (it < items) *(f4*)(dst + tok * NC + 4 * c4) = t0 + tok < T ? x[n] : f4{0.f, 0.f, 0.f, 0.f};
        }
    }
    __device__ __forceinline__ void put_rows(float* dst, int t0, int T, int lt) const {
#pragma unroll
        for (int n = 0; n < N; ++n) {
            const int it = lt + kLoaders * n, tok = it / (NC / 4), c4 = it % (NC / 4);
            if (it < items)
                *(f4*)(dst + tok * NC + row_slot<NC / 16>(4 * c4)) = t0 + tok < T ? x[n] : f4{0.f, 0.f, 0.f, 0.f};
        }
    }
};
// Staging registers for a tensor of element type E (uint16_t: bf16, float), and a store of two adjacent outputs.
template <class E, int NC> struct PickRegs { typedef RegsB<NC> type; };
template <int NC> struct PickRegs<float, NC> { typedef RegsF<NC> type; };
template <class E, int NC> using RegsIn = typename PickRegs<E, NC>::type;
__device__ __forceinline__ void store2(uint16_t* p, float lo, float hi) { *(uint32_t*)p = pack2(lo, hi); }
__device__ __forceinline__ void store2(float* p, float lo, float hi) { *(fc*)p = fc{lo, hi}; }

template <int RT>
__device__ __forceinline__ void get_rows(float (&x)[RT], const float* src) {  // src: the token's vector + 4 * rg
#pragma unroll
    for (int i = 0; i < RT / 4; ++i) {
        const f4 y = *(const f4*)(src + 64 * i);
        x[4 * i] = y[0]; x[4 * i + 1] = y[1]; x[4 * i + 2] = y[2]; x[4 * i + 3] = y[3];
    }
}

struct Where {  // what a workgroup and its lanes own (Args: B, T, H, cu as in the kernels' argument blocks)
    int tid, wave, lane, rg, cg, slice, bh, b, h, col;  // col: first of the lane's CW columns of the sliced dim
    int lcol;                                            // the same inside the workgroup's 64-column slice
    int T;                                               // tokens of this sequence
    size_t tok0;                                         // index of its first token
};
template <class Args>
__device__ __forceinline__ Where where(const Args& a, int nslices) {
    Where w;
    w.tid = threadIdx.x;
    w.wave = __builtin_amdgcn_readfirstlane(w.tid >> 6);
    w.lane = w.tid & 63;
    w.rg = w.lane & 15;
    w.cg = w.lane >> 4;
    // blockIdx.x % 8 is the XCD a workgroup lands on; the slices of a (sequence, head) pair go to one XCD so that
    // the L2 they share fetches k, q, d_out and the intermediates once.  Rectangular batches: every XCD a contiguous
    // range of pairs; packed ones: pairs dealt round-robin, which spreads the heads of one long sequence over all
    // XCDs.  The grid is 8 * nslices * ceil(pairs / 8); the padding gets bh = -1 and leaves at once.
    {
        const int pairs = a.B * a.H, xcd = blockIdx.x & 7, place = blockIdx.x >> 3;
        int wg;
        if (a.cu) {
            const int pair = (place / nslices) * 8 + xcd;
            wg = pair < pairs ? pair * nslices + place % nslices : -1;
        } else {
            wg = xcd * (int)(gridDim.x >> 3) + place;
            if (wg >= pairs * nslices) wg = -1;
        }
        w.slice = wg < 0 ? 0 : wg % nslices;
        w.bh = wg < 0 ? -1 : wg / nslices;
    }
    if (w.bh < 0) {
        w.b = w.h = w.col = w.lcol = w.T = 0;
        w.tok0 = 0;
        return w;
    }
    w.b = w.bh / a.H;
    w.h = w.bh % a.H;
    w.col = w.slice * kSlice + (w.wave & (kWaves - 1)) * 4 * CW + w.cg * CW;
    w.lcol = w.col - w.slice * kSlice;
    w.T = a.T;
    w.tok0 = (size_t)w.b * a.T;
    if (a.cu) {  // offsets are clamped into the tensors whatever cu holds
        const int start = min(max(a.cu[w.b], 0), a.T), end = min(max(a.cu[w.b + 1], start), a.T);
        w.T = end - start;
        w.tok0 = (size_t)start;
    }
    return w;
}

}  // namespace tok
}  // namespace sla
