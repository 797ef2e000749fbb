// Backward pass of the gated delta rule (Softmax-GatedDeltaNet, Sec. 5.1) in block form on the matrix cores, bf16.
//
// Tokens are taken in blocks of C = 32.  Inside a block, with c_t the running sum of the log-decays, p_t = e^(c_t),
// A = p_C and D[t][j] = p_t / p_j (j <= t), the recurrence
//     res_t = G^K_t v_t - k_t (a_t S_{t-1})      u_t = beta_t res_t      S_t = a_t S_{t-1} + k_t^T u_t
// (the chunkwise form of Sec. 3.2 applied to the delta rule) becomes, for the block's entry state S0,
//     (I + Lk diag(beta)) Res = G^K V - diag(p) K S0,    Lk = strict_tril(D * K K^T),      U = diag(beta) Res,
//     S_C = A S0 + K^T diag(A / p) U,                     Y = diag(p) Q S0 + Lq U,          Lq = tril(D * Q K^T),
// and its derivative, for the cotangent X1 of S_C and dY = diag(G^Q) dOut:
//     dU  = Lq^T dY + diag(A / p) K X1
//     w   = (I + Lk diag(beta))^-T (beta * dU)      (the cotangent of res, what the token recurrence calls beta du)
//     du  = dU - Lk^T w
//     dv  = G^K w      dG^K = w . v      dbeta = du . res
//     X0  = A X1 + Q^T diag(p) dY - K^T diag(p) w
//     dq' = diag(p) dOut S0^T + N' K                 N' = tril(D * dOut U^T)      dq = G^Q dq'    dG^Q = q . dq'
//     dk  = diag(A / p) U X1^T - diag(p) w S0^T + (M + M^T) K + N^T Q
//           M = strict_tril(-D * w U^T)              N = diag(G^Q) N'
// The decay gradient needs no state product (see sla_backward_gdn.hip), but is re-derived as <X0, S0> at every 512th
// token of a sequence, where its running sum would otherwise have drifted (kGdnAnchor in sla_gdn_block.h).  The
// 32 x 32 matrices depend on one block only: T' = (I + Lk diag(beta))^-1 comes from a kernel that runs over all blocks
// in parallel (`pre`); the others are formed by the sweep that uses them from the rows it holds anyway (Lq and Lk in
// sweep 2, M and N' in sweep 3, N' in sweep 4).  What remains serial are four sweeps that each carry one state tile in
// fp32 matrix-core accumulators, as in the token-recurrent version: (1) forward, S sliced over value columns -> res;
// (2) backward, X sliced over value columns -> w, dv, dG^K, dbeta, d_initial_state; (3) backward, X^T sliced over key
// columns -> the part of dk that needs X; (4) forward, S^T sliced over key columns -> dq, dG^Q, dk, <d_final, S_T>.
//
// A sweep workgroup: four compute waves (16 columns of the 64-column slice each, the whole contraction dimension)
// and four loader waves that copy the coming blocks' rows from global memory to LDS, row-major and unchanged, several
// blocks ahead in registers, into the next of two or three LDS stages (run_sweep() and its modes: who makes the
// block-local matrices, and when).  Every operand orientation comes from the same row-major
// arrays: rows as they are (`op_rows`), columns through the transposing LDS read of gfx950 (`op_cols`,
// ds_read_b64_tr_b16: the 16 lanes of a group fetch 4 rows x 16 columns and each receives one column), and an
// accumulator tile serves directly as the next product's operand (rows 4g..4g+3 of lane group g are its contraction
// slots).  All products are v_mfma_f32_16x16x32_bf16; the contraction index of slot (half, g, e) is 16 half + 4 g + e
// in both operands.
//
// Intermediates in the workspace: res and w as bf16 [block][head][column][32 tokens] (a lane's four tokens of an
// accumulator tile are one 8-byte store), T' as bf16, per-token scalars as fp32, the X-part of dk as
// bf16 [block][head][dk/4][32 tokens][4], and at the anchors the state cotangent in fp32.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "sla.h"
#include "sla_block_ops.h"
#include "sla_gdn_block.h"

namespace sla {
namespace {

using namespace blk;

constexpr int kThreads = 512;    // four compute waves + four loader waves
constexpr int kLoaders = 256;
constexpr int kCols = 64;        // columns of a state slice per workgroup
constexpr int kMat = C * C;                  // elements of a 32 x 32 matrix
enum { mT1 = 0, kPreMats = 1 };   // pre-pass: T' 

// ---- rows of a 2-D array, global -> registers -> LDS, by the 256 loader threads, 16 bytes a piece -----------
template <int R, int RB>
struct Rows {
    static constexpr int per = RB / 16, pieces = R * per, N = (pieces + kLoaders - 1) / kLoaders;
    u4 x[N];
    int valid;  // rows >= valid are written as zero
    // Nothing here looks at the loaded values (a piece outside the array reads its first piece instead, valid >= 1;
    // the zeroing happens in put), so the loads stay in flight until the block is due.
    __device__ __forceinline__ void load(const void* g, size_t gstride, int valid_rows, int lt) {
        valid = valid_rows;
#pragma unroll
        for (int n = 0; n < N; ++n) {
            const int it = lt + kLoaders * n, row = it / per, c = it - row * per;
            const bool ok = it < pieces && row < valid_rows;
            x[n] = *(const u4*)((const unsigned char*)g + (size_t)(ok ? row : 0) * gstride + 16 * (ok ? c : 0));
        }
    }
    // A thread without a piece of its own holds piece 0 (see load) and writes it where piece 0 goes: no branch.
    __device__ __forceinline__ void put(unsigned char* lds, int lstride, int lt) const {
#pragma unroll
        for (int n = 0; n < N; ++n) {
            const int it = lt + kLoaders * n, row0 = it / per;
            const bool in = it < pieces;
            const int row = in ? row0 : 0, c = in ? it - row0 * per : 0;
            *(u4*)(lds + row * lstride + 16 * c) = row < valid ? x[n] : u4{0u, 0u, 0u, 0u};
        }
    }
};

// ---- what a workgroup owns ----------------------------------------------------------------------------------
struct Seq {
    int bh, b, h, slice;   // bh < 0: nothing to do
    int T, nblk;           // tokens and blocks of the sequence
    size_t tok0;           // its first token
    size_t blk0;           // its first block in the workspace
};
// blocks of the workspace: rectangular batches B * ceil(T/C); packed ones floor(T/C) + B + 1, sequence b starting at
// block cu[b]/C + b (the ranges of consecutive sequences cannot overlap: floor(x) + ceil(y) <= floor(x + y) + 1).
__host__ __device__ inline size_t ws_blocks(int B, int T, bool packed) {
    return packed ? (size_t)T / C + (size_t)B + 1 : (size_t)B * ((T + C - 1) / C);
}
__device__ __forceinline__ void seq_of(const GdnBlockArgs& a, int b, Seq& s) {
    s.T = a.T;
    s.tok0 = (size_t)b * a.T;
    s.blk0 = (size_t)b * ((a.T + C - 1) / C);
    if (a.cu) {  // offsets are clamped into the tensors whatever cu holds
        const int start = min(max(a.cu[b], 0), a.T), end = min(max(a.cu[b + 1], start), a.T);
        s.T = end - start;
        s.tok0 = (size_t)start;
        s.blk0 = (size_t)(start / C) + (size_t)b;
    }
    s.nblk = (s.T + C - 1) / C;
}
constexpr int kAnchorBlocks = kGdnAnchor / C;
__device__ __forceinline__ size_t anchor_id(const Seq& s, int I) { return (s.tok0 + (size_t)C * I) / kGdnAnchor; }
// blockIdx.x % 8 is the XCD a workgroup lands on; the slices of a (sequence, head) pair go to one XCD, whose L2 then
// fetches what they share once.  The grid is 8 * nslices * ceil(pairs / 8); the padding has nothing to do.
__device__ __forceinline__ Seq where(const GdnBlockArgs& a, int nslices) {
    Seq s;
    const int pairs = a.B * a.H, xcd = blockIdx.x & 7, place = blockIdx.x >> 3;
    int wg;
    if (a.cu) {
        const int pair = (place / nslices) * 8 + xcd;
        wg = pair < pairs ? pair * nslices + place % nslices : -1;
    } else {
        wg = xcd * (int)(gridDim.x >> 3) + place;
        if (wg >= pairs * nslices) wg = -1;
    }
    s.bh = wg < 0 ? -1 : wg / nslices;
    s.slice = wg < 0 ? 0 : wg % nslices;
    s.b = s.h = s.T = s.nblk = 0;
    s.tok0 = s.blk0 = 0;
    if (s.bh >= 0) {
        s.b = s.bh / a.H;
        s.h = s.bh % a.H;
        seq_of(a, s.b, s);
    }
    return s;
}

// workspace areas
struct Areas {
    float* scal;   // [blocks][H][kKinds][C]
    bf* pre;       // [blocks][H][kPreMats][C][C]
    bf* res;       // [blocks][H][dv][C]
    bf* w;         // [blocks][H][dv][C]
    bf* dk2;       // [blocks][H][dk/4][C][4]: the X-part of dk, four adjacent key columns of a token together
};
__host__ __device__ inline size_t round4(size_t n) { return (n + 3) & ~(size_t)3; }
__host__ __device__ inline Areas areas(float* ws, size_t blocks, size_t rows, int H, int dk, int dv) {
    Areas r;
    const size_t bh = blocks * (size_t)H;
    float* p = ws;
    r.scal = p; p += bh * kScal;
    r.pre = (bf*)p; p += bh * kPreMats * kMat / 2;
    r.res = (bf*)p; p += bh * (size_t)dv * C / 2;
    r.w = (bf*)p; p += bh * (size_t)dv * C / 2;
    r.dk2 = (bf*)p;
    (void)rows; (void)dk;
    return r;
}

// ------------------------------------------------------------------------------------------------------------
// Pre-pass: one wave per (block, head).  The per-token scalars and T' = (I + Lk diag(beta))^-1.
// ------------------------------------------------------------------------------------------------------------
// The workspace block `wb` belongs to sequence b when blk0(b) <= wb < blk0(b) + nblk(b).
__device__ __forceinline__ bool find_block(const GdnBlockArgs& a, size_t wb, Seq& s, int& I) {
    if (!a.cu) {
        const int per = (a.T + C - 1) / C;
        if (per == 0) return false;
        s.b = (int)(wb / per);
        if (s.b >= a.B) return false;
        seq_of(a, s.b, s);
        I = (int)(wb - s.blk0);
        return true;
    }
    int lo = 0, hi = a.B - 1;  // last sequence whose first block is <= wb
    while (lo < hi) {
        const int m = (lo + hi + 1) >> 1;
        const size_t first = (size_t)(min(max(a.cu[m], 0), a.T) / C) + (size_t)m;
        if (first <= wb) lo = m; else hi = m - 1;
    }
    s.b = lo;
    seq_of(a, lo, s);
    if (wb < s.blk0 || wb >= s.blk0 + (size_t)s.nblk) return false;
    I = (int)(wb - s.blk0);
    return true;
}

// 16 bytes of a row of k or q as half an operand: slot (g, e) is element k0 + 8g + e (both operands of the Gram
// products come from memory, so any slot order they share will do).
__device__ __forceinline__ s8 gram_op(const bf* rows, size_t gstride, int row, int valid, int k0, int g) {
    const u4 z = {0u, 0u, 0u, 0u};
    const u4 v = row < valid ? *(const u4*)(rows + (size_t)row * gstride + k0 + 8 * g) : z;
    return __builtin_bit_cast(s8, v);
}

template <int DK>
__global__ __launch_bounds__(64) void gdn_blk_pre_kernel(const GdnBlockArgs a, const Areas ar) {
    constexpr int LS = 36;  // row stride of the fp32 matrices
    __shared__ __align__(16) float Lf[C * LS];   // Lk diag(beta)
    __shared__ __align__(16) float Tf[C * LS];   // T'
    __shared__ __align__(16) float cs[C], bs[C];
    const int lane = threadIdx.x, r = lane & 15, g = lane >> 4;
    const int h = blockIdx.x % a.H;
    const size_t wb = blockIdx.x / a.H;
    Seq s;
    int I = 0;
    if (!find_block(a, wb, s, I)) return;
    const int valid = min(C, s.T - C * I);
    const size_t row0 = s.tok0 + (size_t)C * I;
    // per-token scalars: lane t (and t + 32, which repeats it)
    const int t = lane & 31;
    const bool tv = t < valid;
    const size_t si = (row0 + (tv ? t : 0)) * a.H + h;
    const float ldt = tv ? a.ld[si] * kLog2e : 0.f;
    const float bt = tv ? a.beta[si] : 0.f, gqt = tv ? a.gq[si] : 0.f, gkt = tv ? a.gk[si] : 0.f;
    float c = ldt;  // inclusive running sum over the 32 tokens (both halves of the wave run the same scan)
#pragma unroll
    for (int d = 1; d < C; d *= 2) {
        const float o = __shfl_up(c, d, C);
        if (t >= d) c += o;
    }
    const float c_end = __shfl(c, C - 1, C);
    if (lane < C) {
        cs[t] = c;
        bs[t] = bt;
        float* sc = ar.scal + ((wb * a.H + h) * (size_t)kScal);
        sc[kP * C + t] = __builtin_amdgcn_exp2f(c);
        sc[kAP * C + t] = __builtin_amdgcn_exp2f(c_end - c);
        sc[kBeta * C + t] = bt;
        sc[kGq * C + t] = gqt;
        sc[kGk * C + t] = gkt;
        sc[kCl * C + t] = c;
        sc[kA * C + t] = __builtin_amdgcn_exp2f(c_end);
        sc[7 * C + t] = 0.f;
    }
    // Gram tiles (tau, tau') of K K^T, operands straight from global memory: lane (r, g) ends up with rows
    // t = 16 tau + 4g + i, column j = 16 tau' + r
    const size_t gstride = (size_t)a.H * DK;
    const bf* kg = a.k + (row0 * a.H + h) * DK;
    f4 kk[3];  // tiles (0,0), (1,0), (1,1)
#pragma unroll
    for (int i = 0; i < 3; ++i) kk[i] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k0 = 0; k0 < DK; k0 += 32) {
        const s8 k_lo = gram_op(kg, gstride, r, valid, k0, g), k_hi = gram_op(kg, gstride, 16 + r, valid, k0, g);
        mma(kk[0], k_lo, k_lo);
        mma(kk[1], k_hi, k_lo);
        mma(kk[2], k_hi, k_hi);
    }
    __syncthreads();
    bf* mats = ar.pre + (wb * a.H + h) * (size_t)(kPreMats * kMat);
#pragma unroll
    for (int tile = 0; tile < 3; ++tile) {
        const int ta = tile > 0, tb = tile > 1;
        const int j = 16 * tb + r;
        const float cj = cs[j], bj = bs[j];
        const f4 ct = *(const f4*)(cs + 16 * ta + 4 * g);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int tt = 16 * ta + 4 * g + i;
            Lf[tt * LS + j] = j < tt ? __builtin_amdgcn_exp2f(ct[i] - cj) * kk[tile][i] * bj : 0.f;
        }
    }
    __syncthreads();
    // T' = (I + L)^-1, L = Lk diag(beta) strictly lower, by 16 x 16 blocks: T11 = (I + L11)^-1 and T22 = (I + L22)^-1
    // by forward substitution (lane groups 0 and 2: column r of T11; groups 1 and 3: column r of T22), then
    // T21 = -T22 L21 T11 as two fp32 matrix-core products.
    {
        const int o = 16 * (g & 1);  // this lane's diagonal block
        float x[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            float acc = (j == r) ? 1.f : 0.f;
#pragma unroll
            for (int i4 = 0; i4 < j; i4 += 4) {
                const f4 l = *(const f4*)(Lf + (o + j) * LS + o + i4);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (i4 + e < j) acc -= l[e] * x[i4 + e];
            }
            x[j] = acc;
        }
        if (g < 2) {
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                Tf[(o + j) * LS + o + r] = x[j];
                if (g == 0) Tf[j * LS + 16 + r] = 0.f;  // the block above the diagonal
            }
        }
    }
    __syncthreads();
    f4 pr = {0.f, 0.f, 0.f, 0.f};  // P = L21 T11: rows 4g + i, column r
#pragma unroll
    for (int k4 = 0; k4 < 16; k4 += 4) mma_f32(pr, Lf[(16 + r) * LS + k4 + g], Tf[(k4 + g) * LS + r]);
#pragma unroll
    for (int i = 0; i < 4; ++i) Tf[(16 + 4 * g + i) * LS + r] = pr[i];
    __syncthreads();
    f4 t21 = {0.f, 0.f, 0.f, 0.f};  // T22 P
#pragma unroll
    for (int k4 = 0; k4 < 16; k4 += 4) mma_f32(t21, Tf[(16 + r) * LS + 16 + k4 + g], Tf[(16 + k4 + g) * LS + r]);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) Tf[(16 + 4 * g + i) * LS + r] = -t21[i];
    __syncthreads();
    if (lane < C) {  // T1[t][j] = T'[t][j]: row t
        bf* t1 = mats + mT1 * kMat + t * C;
#pragma unroll
        for (int j = 0; j < C; j += 8) {
            const f4 lo = *(const f4*)(Tf + t * LS + j), hi = *(const f4*)(Tf + t * LS + j + 4);
            *(u4*)(t1 + j) = u4{pack2(lo[0], lo[1]), pack2(lo[2], lo[3]), pack2(hi[0], hi[1]), pack2(hi[2], hi[3])};
        }
    }
}

// ------------------------------------------------------------------------------------------------------------
// The sweeps.  Common frame: loaders fill stage (step + 1) % 2 while the compute waves work on stage step % 2.
// ------------------------------------------------------------------------------------------------------------
struct Frame {
    const GdnBlockArgs& a;
    const Areas& ar;
    const Seq& s;
    __device__ __forceinline__ int valid(int I) const { return min(C, s.T - C * I); }
    __device__ __forceinline__ size_t row0(int I) const { return s.tok0 + (size_t)C * I; }
    __device__ __forceinline__ size_t bhi(int I) const { return (s.blk0 + (size_t)I) * a.H + s.h; }
};

// The 16 x 16 tile of a block-local 32 x 32 matrix that wave w of four makes: (0,0), (1,0), (1,1), (0,1).
__device__ __forceinline__ void tile_of_wave(int w, int& ta, int& tb) {
    ta = ((w + 1) >> 1) & 1;
    tb = w >> 1;
}

// LOADER: struct with load(frame, I, lt) and put(stage, lt); BODY: callable (stage, I).  The loaders keep PF blocks in
// flight in registers (block b in set b % PF): a block's rows are requested PF + 1 steps before the compute waves
// need them, which covers the latency of HBM under load (with one block in flight a step lasted as long as a load).
// How the block-local matrices that a sweep forms itself get into the stage:
//   kPlain  none; two stages, one barrier per step;
//   kHalves two stages; a step has two halves with a barrier between them: FIRST (stage, I) lets the compute waves
//           write the matrices (and do what needs only the carried state), BODY reads them;
//   kAhead  three stages: the loader waves, otherwise idle between their copies, make the matrices of block
//           step + 1 with MATS (stage, loader wave, lane) from the rows they staged a step earlier, while the
//           compute waves work on block step and the copies of block step + 2 land; one barrier per step.
enum { kPlain = 0, kHalves = 1, kAhead = 2 };
struct NoFirst {
    __device__ __forceinline__ void operator()(unsigned char*, int) const {}
};
struct NoMats {
    __device__ __forceinline__ void operator()(unsigned char*, int, int) const {}
};
template <bool FWD, int PF, class LOADER, int MODE = kPlain, class BODY, class INIT, class FINI, class FIRST = NoFirst,
          class MATS = NoMats>
__device__ __forceinline__ void run_sweep(const Frame& f, unsigned char* smem, int stage_bytes, INIT&& init, BODY&& body,
                                          FINI&& fini, FIRST&& first = NoFirst(), MATS&& mats = NoMats()) {
    const int tid = threadIdx.x, nblk = f.s.nblk;
    // Both sides run the same number of steps, a multiple of PF, so that the loaders' loop body has no branch in it
    // (the compiler then lets the loads of the other register sets stay outstanding across a put); steps past the
    // last block stage that block again and compute nothing.
    const int nsteps = (nblk + PF - 1) / PF * PF;
    auto blk = [&](int step) {
        const int sclamp = min(step, nblk - 1);
        return FWD ? sclamp : nblk - 1 - sclamp;
    };
    constexpr int NS = MODE == kAhead ? 3 : 2;
    auto stage = [&](int step) { return smem + (step % NS) * stage_bytes; };
    if (tid >= kThreads - kLoaders) {
        if (nblk == 0) return;
        const int lt = tid - (kThreads - kLoaders);
        LOADER R[PF];
#pragma unroll
        for (int u = 0; u < PF; ++u) R[u].load(f, blk(u), lt);
        R[0].put(smem, lt);
        R[0].load(f, blk(PF), lt);
        __syncthreads();
        if constexpr (MODE == kAhead) {
            static_assert(PF >= 2, "two blocks are staged before the first step");
            const int lw = __builtin_amdgcn_readfirstlane(lt >> 6), lane = lt & 63;
            R[1].put(stage(1), lt);
            R[1].load(f, blk(PF + 1), lt);
            mats(stage(0), lw, lane);
            __syncthreads();
            for (int base = 0; base < nsteps; base += PF) {
#pragma unroll
                for (int u = 0; u < PF; ++u) {
                    const int step = base + u;
                    LOADER& set = R[(u + 2) % PF];  // holds block step + 2 (base is a multiple of PF)
                    set.put(stage(step + 2), lt);
                    set.load(f, blk(step + 2 + PF), lt);
                    mats(stage(step + 1), lw, lane);
                    __syncthreads();
                }
            }
        } else {
            for (int base = 0; base < nsteps; base += PF) {
#pragma unroll
                for (int u = 0; u < PF; ++u) {
                    const int step = base + u;
                    LOADER& set = R[(u + 1) % PF];  // holds block step + 1 (base is a multiple of PF)
                    set.put(stage(step + 1), lt);
                    set.load(f, blk(step + 1 + PF), lt);
                    if constexpr (MODE == kHalves) __syncthreads();
                    __syncthreads();
                }
            }
        }
    } else {
        init();
        if (nblk > 0) {
            __syncthreads();
            if constexpr (MODE == kAhead) __syncthreads();
            for (int step = 0; step < nsteps; ++step) {
                if constexpr (MODE == kHalves) {
                    if (step < nblk) first(stage(step), blk(step));
                    __syncthreads();
                }
                if (step < nblk) body(stage(step), blk(step));
                __syncthreads();
            }
        }
        fini();
    }
}

// ---- sweep 1: forward, S[dk, 16 value columns per wave] -> res ------------------------------------------------
template <int DK>
struct Stage1 {
    static constexpr int RKr = rows_stride(DK), RKc = cols_stride(DK);
    static constexpr int oK = 0, oKc = oK + C * RKr * 2, oV = oKc + C * RKc * 2, oT = oV + C * kSlC * 2,
                         oS = oT + C * kSmR * 2, bytes = oS + kScal * 4;
};
template <int DK, int DV>
struct Load1 {
    Rows<C, DK * 2> k;
    Rows<C, kCols * 2> v;
    Rows<C, 64> t1;
    Rows<kKinds, C * 4> sc;
    __device__ __forceinline__ void load(const Frame& f, int I, int lt) {
        const size_t row = f.row0(I) * f.a.H + f.s.h, bhi = f.bhi(I);
        k.load(f.a.k + row * DK, (size_t)f.a.H * DK * 2, f.valid(I), lt);
        v.load(f.a.v + row * DV + f.s.slice * kCols, (size_t)f.a.H * DV * 2, f.valid(I), lt);
        t1.load(f.ar.pre + bhi * (size_t)(kPreMats * kMat) + mT1 * kMat, C * 2, C, lt);
        sc.load(f.ar.scal + bhi * (size_t)kScal, C * 4, kKinds, lt);
    }
    __device__ __forceinline__ void put(unsigned char* st, int lt) const {
        typedef Stage1<DK> L;
        k.put(st + L::oK, L::RKr * 2, lt);
        k.put(st + L::oKc, L::RKc * 2, lt);
        v.put(st + L::oV, kSlC * 2, lt);
        t1.put(st + L::oT, kSmR * 2, lt);
        sc.put(st + L::oS, C * 4, lt);
    }
};

template <int DK, int DV>
__global__ __launch_bounds__(kThreads) void gdn_blk_state_kernel(const GdnBlockArgs a, const Areas ar) {
    typedef Stage1<DK> L;
    constexpr int NT = DK / 16, RKr = L::RKr, RKc = L::RKc;
    extern __shared__ __align__(16) unsigned char smem[];
    const Seq s = where(a, DV / kCols);
    if (s.bh < 0) return;
    const Frame f{a, ar, s};
    const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane((threadIdx.x >> 6) & 3), r = lane & 15,
              g = lane >> 4;
    const int n = s.slice * kCols + 16 * w + r;  // this lane's value column
    f4 S[NT];
    run_sweep<true, 4, Load1<DK, DV>>(
        f, smem, L::bytes,
        [&]() {
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    S[t][i] = a.s0 ? a.s0[((size_t)s.bh * DK + 16 * t + 4 * g + i) * DV + n] : 0.f;
        },
        [&](const unsigned char* st, int I) {
            const bf* Kr = (const bf*)(st + L::oK);
            const bf* Kc = (const bf*)(st + L::oKc);
            const bf* Vs = (const bf*)(st + L::oV);
            const bf* T1 = (const bf*)(st + L::oT);
            const float* sc = (const float*)(st + L::oS);
            f4 X[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
            for (int t = 0; t < NT; t += 2) {
                const s8 bS = pack8(S[t], S[t + 1]);
                mma(X[0], op_rows(Kr, RKr, r, 16 * t, g), bS);
                mma(X[1], op_rows(Kr, RKr, 16 + r, 16 * t, g), bS);
            }
            f4 Rp[2];
#pragma unroll
            for (int ta = 0; ta < 2; ++ta)
                Rp[ta] = sc4(sc, kGk, 16 * ta + 4 * g) * tile_cols(Vs, kSlC, 16 * ta, 16 * w, r, g) -
                         sc4(sc, kP, 16 * ta + 4 * g) * X[ta];
            const s8 bR = pack8(Rp[0], Rp[1]);
            bf* dst = ar.res + (f.bhi(I) * (size_t)DV + n) * C + 4 * g;
            f4 Up[2];
#pragma unroll
            for (int ta = 0; ta < 2; ++ta) {
                f4 rs = {0.f, 0.f, 0.f, 0.f};
                mma(rs, op_rows(T1, kSmR, 16 * ta + r, 0, g), bR);
                const u2 pk = pack4(rs);
                *(u2*)(dst + 16 * ta) = pk;
                Up[ta] = sc4(sc, kBeta, 16 * ta + 4 * g) * sc4(sc, kAP, 16 * ta + 4 * g) * unpack4(pk);
            }
            const s8 bU = pack8(Up[0], Up[1]);
            const float A = sc[kA * C];
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                S[t] *= A;
                mma(S[t], op_cols(Kc, RKc, 0, 16 * t, r, g), bU);
            }
        },
        [&]() {});
}

// ---- sweep 2: backward, X[dk, 16 value columns per wave] -> w, dv, dG^K, dbeta, d_initial_state -----------------
template <int DK>
struct Stage2 {
    static constexpr int RKr = rows_stride(DK), RKc = cols_stride(DK);
    static constexpr int oK = 0, oKc = oK + C * RKr * 2, oQ = oKc + C * RKc * 2, oO = oQ + C * RKc * 2,
                         oV = oO + C * kSlC * 2, oR = oV + C * kSlR * 2, oT = oR + kCols * kSmC * 2,  // T' (by columns)
                         oL = oT + C * kSmC * 2,                                             // Lq, -Lk: made by the sweep
                         oS = oL + 2 * C * kSmR * 2, bytes = oS + kScal * 4;
};
template <int DK, int DV>
struct Load2 {
    Rows<C, DK * 2> k, q;
    Rows<C, kCols * 2> o, v;
    Rows<kCols, 64> rs;
    Rows<C, 64> t;
    Rows<kKinds, C * 4> sc;
    __device__ __forceinline__ void load(const Frame& f, int I, int lt) {
        const size_t row = f.row0(I) * f.a.H + f.s.h, bhi = f.bhi(I);
        const int valid = f.valid(I), n0 = f.s.slice * kCols;
        k.load(f.a.k + row * DK, (size_t)f.a.H * DK * 2, valid, lt);
        q.load(f.a.q + row * DK, (size_t)f.a.H * DK * 2, valid, lt);
        o.load(f.a.dout + row * DV + n0, (size_t)f.a.H * DV * 2, valid, lt);
        v.load(f.a.v + row * DV + n0, (size_t)f.a.H * DV * 2, valid, lt);
        rs.load(f.ar.res + (bhi * (size_t)DV + n0) * C, C * 2, kCols, lt);
        t.load(f.ar.pre + bhi * (size_t)(kPreMats * kMat) + mT1 * kMat, C * 2, C, lt);
        sc.load(f.ar.scal + bhi * (size_t)kScal, C * 4, kKinds, lt);
    }
    __device__ __forceinline__ void put(unsigned char* st, int lt) const {
        typedef Stage2<DK> L;
        k.put(st + L::oK, L::RKr * 2, lt);
        k.put(st + L::oKc, L::RKc * 2, lt);
        q.put(st + L::oQ, L::RKc * 2, lt);
        o.put(st + L::oO, kSlC * 2, lt);
        v.put(st + L::oV, kSlR * 2, lt);
        rs.put(st + L::oR, kSmC * 2, lt);
        t.put(st + L::oT, kSmC * 2, lt);
        sc.put(st + L::oS, C * 4, lt);
    }
};

// Sweep 2's block-local matrices, diag(G^Q) Lq = diag(G^Q) tril(D * Q K^T) and -Lk = -strict_tril(D * K K^T), from
// the staged rows of q and k; one 16 x 16 tile per wave as in local_matrices().
template <int DK>
__device__ __forceinline__ void gram_matrices(unsigned char* st, int w, int r, int g) {
    typedef Stage2<DK> L;
    const bf* Kr = (const bf*)(st + L::oK);
    const bf* Qr = (const bf*)(st + L::oQ);
    const float* sc = (const float*)(st + L::oS);
    bf* Lq = (bf*)(st + L::oL);
    bf* Lkn = Lq + C * kSmR;
    int ta, tb;
    tile_of_wave(w, ta, tb);
    const int tt = 16 * ta + r;
    f4 qk = {0.f, 0.f, 0.f, 0.f}, kk = {0.f, 0.f, 0.f, 0.f};  // [i]: row tt, column 16 tb + 4g + i
#pragma unroll
    for (int k0 = 0; k0 < DK; k0 += 32) {
        const s8 aK = op_rows(Kr, L::RKr, 16 * tb + r, k0, g);
        mma(qk, aK, op_rows(Qr, L::RKc, tt, k0, g));
        mma(kk, aK, op_rows(Kr, L::RKr, tt, k0, g));
    }
    const float ct = sc[kCl * C + tt], gqt = sc[kGq * C + tt];
    const f4 cj = sc4(sc, kCl, 16 * tb + 4 * g);
    f4 lq, lk;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int j = 16 * tb + 4 * g + i;
        const float d = __builtin_amdgcn_exp2f(ct - cj[i]);
        lq[i] = j <= tt ? d * qk[i] * gqt : 0.f;
        lk[i] = j < tt ? -d * kk[i] : 0.f;
    }
    *(u2*)(Lq + tt * kSmR + 16 * tb + 4 * g) = pack4(lq);
    *(u2*)(Lkn + tt * kSmR + 16 * tb + 4 * g) = pack4(lk);
}

template <int DK, int DV>
__global__ __launch_bounds__(kThreads) void gdn_blk_cotangent_kernel(const GdnBlockArgs a, const Areas ar) {
    typedef Stage2<DK> L;
    constexpr int NT = DK / 16, RKr = L::RKr, RKc = L::RKc;
    extern __shared__ __align__(16) unsigned char smem[];
    const Seq s = where(a, DV / kCols);
    if (s.bh < 0) return;
    const Frame f{a, ar, s};
    const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane((threadIdx.x >> 6) & 3), r = lane & 15,
              g = lane >> 4;
    const int n0 = s.slice * kCols, n = n0 + 16 * w + r;
    const int plane = (n0 >> 4) + w;
    f4 X[NT];
    run_sweep<false, 4, Load2<DK, DV>, kAhead>(
        f, smem, L::bytes,
        [&]() {
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    X[t][i] = a.dsf ? a.dsf[((size_t)s.bh * DK + 16 * t + 4 * g + i) * DV + n] : 0.f;
        },
        [&](const unsigned char* st, int I) {
            const bf* Kr = (const bf*)(st + L::oK);
            const bf* Kc = (const bf*)(st + L::oKc);
            const bf* Qr = (const bf*)(st + L::oQ);
            const bf* Os = (const bf*)(st + L::oO);
            const bf* Vs = (const bf*)(st + L::oV);
            const bf* Rs = (const bf*)(st + L::oR);
            const bf* T1 = (const bf*)(st + L::oT);
            const bf* Lq = (const bf*)(st + L::oL);
            const bf* Lkn = Lq + C * kSmR;
            const float* sc = (const float*)(st + L::oS);
            const s8 bO = op_cols(Os, kSlC, 0, 16 * w, r, g);  // dOut[t slots][column n]
            const f4 p0 = sc4(sc, kP, 4 * g), p1 = sc4(sc, kP, 16 + 4 * g);
            const f4 gq0 = sc4(sc, kGq, 4 * g), gq1 = sc4(sc, kGq, 16 + 4 * g);
            f4 dU[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};  // K X1, this wave's columns
#pragma unroll
            for (int t = 0; t < NT; t += 2) {
                const s8 bX = pack8(X[t], X[t + 1]);
                mma(dU[0], op_rows(Kr, RKr, r, 16 * t, g), bX);
                mma(dU[1], op_rows(Kr, RKr, 16 + r, 16 * t, g), bX);
            }
            {   // the part of X's step that does not need w: A X1 + Q^T diag(p) dY
                const s8 bq = scale8(bO, p0 * gq0, p1 * gq1);
                const float A = sc[kA * C];
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    X[t] *= A;
                    mma(X[t], op_cols(Qr, RKc, 0, 16 * t, r, g), bq);
                }
            }
#pragma unroll
            for (int ta = 0; ta < 2; ++ta) {
                dU[ta] *= sc4(sc, kAP, 16 * ta + 4 * g);
                mma(dU[ta], op_cols(Lq, kSmR, 0, 16 * ta, r, g), bO);  // Lq^T dY, G^Q folded into Lq's rows
            }
            const f4 be0 = sc4(sc, kBeta, 4 * g), be1 = sc4(sc, kBeta, 16 + 4 * g);
            const s8 pdU = pack8(dU[0], dU[1]);
            // identity as an operand: slot (half, g, e) is token 16 half + 4g + e; column 16 tau + r
            s8 id[2];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const short one = (4 * g + e == r) ? (short)0x3f80 : (short)0;
                id[0][e] = one; id[0][4 + e] = 0;
                id[1][e] = 0;   id[1][4 + e] = one;
            }
            f4 wv[2], wT[2], duT[2];
            s8 aT2[2];
#pragma unroll
            for (int ta = 0; ta < 2; ++ta) {
                aT2[ta] = scale8(op_cols(T1, kSmC, 0, 16 * ta, r, g), be0, be1);  // (T' diag(beta))^T, row 16 ta + r
                wv[ta] = f4{0.f, 0.f, 0.f, 0.f};
                wT[ta] = f4{0.f, 0.f, 0.f, 0.f};
                duT[ta] = f4{0.f, 0.f, 0.f, 0.f};
                mma(wv[ta], aT2[ta], pdU);   // w[t = 16 ta + 4g + i][column r]
                mma(wT[ta], pdU, aT2[ta]);   // w[t = 16 ta + r][column 4g + i]
                mma(duT[ta], pdU, id[ta]);   // dU, transposed the same way
            }
            const u2 pw0 = pack4(wv[0]), pw1 = pack4(wv[1]);
            const s8 pw = __builtin_bit_cast(s8, u4{pw0.x, pw0.y, pw1.x, pw1.y});
            {
                bf* dst = ar.w + (f.bhi(I) * (size_t)DV + n) * C + 4 * g;
                *(u2*)dst = pw0;
                *(u2*)(dst + 16) = pw1;
            }
            const int valid = f.valid(I);
            const size_t row0 = f.row0(I);
#pragma unroll
            for (int ta = 0; ta < 2; ++ta) {
                mma(duT[ta], pw, op_cols(Lkn, kSmR, 0, 16 * ta, r, g));  // du = dU - Lk^T w, token 16 ta + r
                const int tt = 16 * ta + r;
                const f4 rs4 = tile_cols(Rs, kSmC, 16 * w, 16 * ta, r, g);            // res[token tt][column 16w + 4g + i]
                const f4 v4 = unpack4(*(const s4*)(Vs + tt * kSlR + 16 * w + 4 * g));  // v[token tt][the same columns]
                float pb = 0.f, pk = 0.f;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    pb += duT[ta][i] * rs4[i];
                    pk += wT[ta][i] * v4[i];
                }
                pb = all_groups(pb);
                pk = all_groups(pk);
                if (tt < valid) {
                    const size_t at = (row0 + tt) * a.H + s.h;
                    if (g == 0) {
                        a.part_b[(size_t)plane * a.plane + at] = pb;
                        a.part_k[(size_t)plane * a.plane + at] = pk;
                    }
                    *(u2*)(a.dv + at * DV + n0 + 16 * w + 4 * g) = pack4(wT[ta] * sc[kGk * C + tt]);
                }
            }
            const s8 bw = scale8(pw, -p0, -p1);  // X0 = (A X1 + Q^T diag(p) dY: above) - K^T diag(p) w
#pragma unroll
            for (int t = 0; t < NT; ++t) mma(X[t], op_cols(Kc, RKc, 0, 16 * t, r, g), bw);
        },
        [&]() {
            if (a.ds0) {
#pragma unroll
                for (int t = 0; t < NT; ++t)
#pragma unroll
                    for (int i = 0; i < 4; ++i) a.ds0[((size_t)s.bh * DK + 16 * t + 4 * g + i) * DV + n] = X[t][i];
            }
        },
        NoFirst(), [&](unsigned char* st, int lw, int ll) { gram_matrices<DK>(st, lw, ll & 15, ll >> 4); });
}

// ---- sweeps 3 and 4: X^T / S^T [dv, 16 key columns per wave] ---------------------------------------------------
// The block-local matrices of these sweeps, M = strict_tril(-D * w U^T) (sweep 3 only) and N' = tril(D * dOut U^T),
// made from the rows the stage already holds (res and w as [dv][C], d_out as [C][dv]) by four waves (the compute waves
// in the first half of a step, or the loader waves a step ahead): wave 0, 1, 2, 3 the 16 x 16 tile (0,0), (1,0),
// (1,1), (0,1), transposed so that a lane ends with four adjacent columns of one row; the triangular mask makes tile
// (0,1) zero, so the four waves run the same code.  Written as bf16 [C][kSmR].
// BRANCH: wave 3 only writes its zeros (for the compute waves; the loader waves' loop must stay free of branches).
template <int DV, bool WITH_M, bool BRANCH = false>
__device__ __forceinline__ void local_matrices(const bf* Rf, int SR, const bf* Wf, int SW, const bf* Of, int RD,
                                               const float* sc, bf* Mm, bf* Np, int w, int r, int g) {
    if (BRANCH && w == 3) {
        if (WITH_M) *(u2*)(Mm + r * kSmR + 16 + 4 * g) = u2{0u, 0u};
        *(u2*)(Np + r * kSmR + 16 + 4 * g) = u2{0u, 0u};
        return;
    }
    int ta, tb;
    tile_of_wave(w, ta, tb);
    const int tt = 16 * ta + r;
    f4 wu = {0.f, 0.f, 0.f, 0.f}, ou = {0.f, 0.f, 0.f, 0.f};  // [i]: row tt, column 16 tb + 4g + i
#pragma unroll
    for (int n0 = 0; n0 < DV; n0 += 32) {
        const s8 aU = op_cols(Rf, SR, n0, 16 * tb, r, g);
        if (WITH_M) mma(wu, aU, op_cols(Wf, SW, n0, 16 * ta, r, g));
        mma(ou, aU, op_rows(Of, RD, tt, n0, g));
    }
    const float ct = sc[kCl * C + tt];
    const f4 cj = sc4(sc, kCl, 16 * tb + 4 * g), bj = sc4(sc, kBeta, 16 * tb + 4 * g);
    f4 m, np;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int j = 16 * tb + 4 * g + i;
        const float d = __builtin_amdgcn_exp2f(ct - cj[i]) * bj[i];
        m[i] = j < tt ? -d * wu[i] : 0.f;
        np[i] = j <= tt ? d * ou[i] : 0.f;
    }
    if (WITH_M) *(u2*)(Mm + tt * kSmR + 16 * tb + 4 * g) = pack4(m);
    *(u2*)(Np + tt * kSmR + 16 * tb + 4 * g) = pack4(np);
}

template <int DV, bool FWD>
struct Stage3 {
    static constexpr int RD = FWD ? rows_stride(DV) : cols_stride(DV);   // d_out rows
    static constexpr int SR = FWD ? kSmR : kSmC, SW = FWD ? kSmC : kSmR;  // res, w
    static constexpr int SQ = FWD ? kSlR : kSlC;                          // the q slice (k slice: by columns in both)
    static constexpr int NM = FWD ? 1 : 2;                                // block-local matrices the compute waves make
    static constexpr int oR = 0, oW = oR + DV * SR * 2, oO = oW + DV * SW * 2, oQ = oO + C * RD * 2,
                         oK = oQ + C * SQ * 2, oM = oK + C * kSlC * 2, oD = oM + NM * C * kSmR * 2,
                         oS = oD + (FWD ? kCols * C * 2 : 0),             // sweep 4: the slice's X-part of dk
                         bytes = oS + kScal * 4;
};
template <int DK, int DV, bool FWD>
struct Load3 {
    Rows<DV, 64> rs, wv;
    Rows<C, DV * 2> o;
    Rows<C, kCols * 2> q, k;
    Rows<kKinds, C * 4> sc;
    Rows<C, 128> d2;  // sweep 4: [16 groups of four key columns][32 tokens][4], contiguous
    __device__ __forceinline__ void load(const Frame& f, int I, int lt) {
        const size_t row = f.row0(I) * f.a.H + f.s.h, bhi = f.bhi(I);
        const int valid = f.valid(I), d0 = f.s.slice * kCols;
        rs.load(f.ar.res + bhi * (size_t)DV * C, C * 2, DV, lt);
        wv.load(f.ar.w + bhi * (size_t)DV * C, C * 2, DV, lt);
        o.load(f.a.dout + row * DV, (size_t)f.a.H * DV * 2, valid, lt);
        q.load(f.a.q + row * DK + d0, (size_t)f.a.H * DK * 2, valid, lt);
        k.load(f.a.k + row * DK + d0, (size_t)f.a.H * DK * 2, valid, lt);
        sc.load(f.ar.scal + bhi * (size_t)kScal, C * 4, kKinds, lt);
        if constexpr (FWD) d2.load(f.ar.dk2 + bhi * (size_t)(DK * C) + (size_t)d0 * C, 128, C, lt);
    }
    __device__ __forceinline__ void put(unsigned char* st, int lt) const {
        typedef Stage3<DV, FWD> L;
        rs.put(st + L::oR, L::SR * 2, lt);
        wv.put(st + L::oW, L::SW * 2, lt);
        o.put(st + L::oO, L::RD * 2, lt);
        q.put(st + L::oQ, L::SQ * 2, lt);
        k.put(st + L::oK, kSlC * 2, lt);
        sc.put(st + L::oS, C * 4, lt);
        if constexpr (FWD) d2.put(st + L::oD, 128, lt);
    }
};

template <int DK, int DV>
__global__ __launch_bounds__(kThreads) void gdn_blk_key_kernel(const GdnBlockArgs a, const Areas ar) {
    typedef Stage3<DV, false> L;
    constexpr int NT = DV / 16, RD = L::RD;
    extern __shared__ __align__(16) unsigned char smem[];
    const Seq s = where(a, DK / kCols);
    if (s.bh < 0) return;
    const Frame f{a, ar, s};
    const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane((threadIdx.x >> 6) & 3), r = lane & 15,
              g = lane >> 4;
    const int d0 = s.slice * kCols, d = d0 + 16 * w + r;  // this lane's key column
    f4 Xt[NT];  // Xt[t][i] = X[d][16 t + 4g + i]
    f4 dkT[2];  // dk2^T[key column 4g + i][token 16 tau + r]: from the first half of a step to the second
    auto init = [&]() {
#pragma unroll
        for (int t = 0; t < NT; ++t)
            Xt[t] = a.dsf ? *(const f4*)(a.dsf + ((size_t)s.bh * DK + d) * DV + 16 * t + 4 * g)
                          : f4{0.f, 0.f, 0.f, 0.f};
    };
    // what needs only the staged rows and the carried state
    auto state = [&](unsigned char* st, int I) {
        const bf* Rf = (const bf*)(st + L::oR);
        const bf* Wf = (const bf*)(st + L::oW);
        const bf* Of = (const bf*)(st + L::oO);
        const bf* Qs = (const bf*)(st + L::oQ);
        const bf* Ks = (const bf*)(st + L::oK);
        const float* sc = (const float*)(st + L::oS);
        // (A/p beta)_t sum_n X[d][n] res[t][n], scaled in the second half
        dkT[0] = dkT[1] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < NT; t += 2) {
            const s8 aX = pack8(Xt[t], Xt[t + 1]);
            mma(dkT[0], aX, op_cols(Rf, kSmC, 16 * t, 0, r, g));
            mma(dkT[1], aX, op_cols(Rf, kSmC, 16 * t, 16, r, g));
        }
        const s8 aK = op_cols(Ks, kSlC, 0, 16 * w, r, g), aQ = op_cols(Qs, kSlC, 0, 16 * w, r, g);
        const f4 p0 = sc4(sc, kP, 4 * g), p1 = sc4(sc, kP, 16 + 4 * g);
        const s8 bq = scale8(aQ, p0 * sc4(sc, kGq, 4 * g), p1 * sc4(sc, kGq, 16 + 4 * g));
        const s8 bk = scale8(aK, -p0, -p1);
        const float A = sc[kA * C];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            Xt[t] *= A;
            mma(Xt[t], op_cols(Of, RD, 0, 16 * t, r, g), bq);
            mma(Xt[t], op_rows(Wf, kSmR, 16 * t + r, 0, g), bk);
        }
        if (I > 0 && (I & (kAnchorBlocks - 1)) == 0) {  // X entering token C * I: kept for the decay gradient
            float* dst = a.anchor_x + ((anchor_id(s, I) * a.H + s.h) * DK + d) * (size_t)DV + 4 * g;
#pragma unroll
            for (int t = 0; t < NT; ++t) *(f4*)(dst + 16 * t) = Xt[t];
        }
    };
    // the local terms, which read the block's matrices
    auto local = [&](const unsigned char* st, int I) {
        const bf* Qs = (const bf*)(st + L::oQ);
        const bf* Ks = (const bf*)(st + L::oK);
        const bf* Mm = (const bf*)(st + L::oM);
        const bf* Np = Mm + C * kSmR;
        const float* sc = (const float*)(st + L::oS);
        const s8 aK = op_cols(Ks, kSlC, 0, 16 * w, r, g), aQ = op_cols(Qs, kSlC, 0, 16 * w, r, g);
        const s8 aQg = scale8(aQ, sc4(sc, kGq, 4 * g), sc4(sc, kGq, 16 + 4 * g));  // N = diag(G^Q) N'
        bf* dk2 = ar.dk2 + f.bhi(I) * (size_t)(DK * C);
#pragma unroll
        for (int ta = 0; ta < 2; ++ta) {
            const int tt = 16 * ta + r;
            dkT[ta] *= sc[kAP * C + tt] * sc[kBeta * C + tt];
            mma(dkT[ta], aK, op_rows(Mm, kSmR, tt, 0, g));            // M K
            mma(dkT[ta], aK, op_cols(Mm, kSmR, 0, 16 * ta, r, g));   // M^T K
            mma(dkT[ta], aQg, op_cols(Np, kSmR, 0, 16 * ta, r, g));  // N^T Q
            *(u2*)(dk2 + ((size_t)(((d0 + 16 * w) >> 2) + g) * C + tt) * 4) = pack4(dkT[ta]);  // rows >= valid: never read
        }
    };
    auto fini = [&]() {
    };
    auto mats = [&](unsigned char* st, int mw, int ml) {
        bf* Mm = (bf*)(st + L::oM);
        local_matrices<DV, true>((const bf*)(st + L::oR), L::SR, (const bf*)(st + L::oW), L::SW, (const bf*)(st + L::oO),
                                 RD, (const float*)(st + L::oS), Mm, Mm + C * kSmR, mw, ml & 15, ml >> 4);
    };
    constexpr int PF = DV > 128 ? 2 : 3;  // register sets of the loaders: what fits next to the code that makes the matrices
    if constexpr (DV > 128) {  // three stages do not fit: the compute waves make the matrices, a barrier, the local terms
        run_sweep<false, PF, Load3<DK, DV, false>, kHalves>(f, smem, L::bytes, init, local, fini,
                                                          [&](unsigned char* st, int I) {
                                                              mats(st, w, lane);
                                                              state(st, I);
                                                          });
    } else {  // the loader waves make them a step ahead
        run_sweep<false, PF, Load3<DK, DV, false>, kAhead>(
            f, smem, L::bytes, init,
            [&](const unsigned char* st, int I) {
                state(const_cast<unsigned char*>(st), I);
                local(st, I);
            },
            fini, NoFirst(), mats);
    }
}

template <int DK, int DV>
__global__ __launch_bounds__(kThreads) void gdn_blk_query_kernel(const GdnBlockArgs a, const Areas ar) {
    typedef Stage3<DV, true> L;
    constexpr int NT = DV / 16, RD = L::RD;
    extern __shared__ __align__(16) unsigned char smem[];
    const Seq s = where(a, DK / kCols);
    if (s.bh < 0) return;
    const Frame f{a, ar, s};
    const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane((threadIdx.x >> 6) & 3), r = lane & 15,
              g = lane >> 4;
    const int d0 = s.slice * kCols, d = d0 + 16 * w + r;
    const int plane = (d0 >> 4) + w;
    constexpr bool kLoadersMakeThem = false;
    f4 St[NT];  // St[t][i] = S[d][16 t + 4g + i]
    f4 dqT[2], dkT[2];  // from the first half of a step (the products with S0) to the second (local terms, stores)
    auto init = [&]() {
#pragma unroll
        for (int t = 0; t < NT; ++t)
            St[t] = a.s0 ? *(const f4*)(a.s0 + ((size_t)s.bh * DK + d) * DV + 16 * t + 4 * g)
                         : f4{0.f, 0.f, 0.f, 0.f};
    };
    // what needs only the staged rows and the carried state
    auto state = [&](unsigned char* st, int I) {
        const bf* Rf = (const bf*)(st + L::oR);
        const bf* Wf = (const bf*)(st + L::oW);
        const bf* Of = (const bf*)(st + L::oO);
        const bf* Ks = (const bf*)(st + L::oK);
        const float* sc = (const float*)(st + L::oS);
        // <X, S> at an anchor, the end of this block (this wave's 16 key columns): X is requested here and used
        // once S has moved on to the end of the block
        const bool anchored = I + 1 < s.nblk && ((I + 1) & (kAnchorBlocks - 1)) == 0;
        f4 xa[NT];
        if (anchored) {
            const float* src = a.anchor_x + ((anchor_id(s, I + 1) * a.H + s.h) * DK + d) * (size_t)DV + 4 * g;
#pragma unroll
            for (int t = 0; t < NT; ++t) xa[t] = *(const f4*)(src + 16 * t);
        }
        dqT[0] = dqT[1] = dkT[0] = dkT[1] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < NT; t += 2) {
            const s8 aS = pack8(St[t], St[t + 1]);
            mma(dqT[0], aS, op_rows(Of, RD, r, 16 * t, g));
            mma(dqT[1], aS, op_rows(Of, RD, 16 + r, 16 * t, g));
            mma(dkT[0], aS, op_cols(Wf, kSmC, 16 * t, 0, r, g));
            mma(dkT[1], aS, op_cols(Wf, kSmC, 16 * t, 16, r, g));
        }
        const s8 aK = op_cols(Ks, kSlC, 0, 16 * w, r, g);
        const s8 bk = scale8(aK, sc4(sc, kBeta, 4 * g) * sc4(sc, kAP, 4 * g),
                             sc4(sc, kBeta, 16 + 4 * g) * sc4(sc, kAP, 16 + 4 * g));
        const float A = sc[kA * C];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            St[t] *= A;
            mma(St[t], op_rows(Rf, kSmR, 16 * t + r, 0, g), bk);
        }
        if (anchored) {
            float acc = 0.f;
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int i = 0; i < 4; ++i) acc += xa[t][i] * St[t][i];
            acc = all_groups(row_all(acc));
            if (lane == 0) a.anchor_phi[(anchor_id(s, I + 1) * a.H + s.h) * (size_t)(DK / 16) + plane] = acc;
        }
    };
    // the local terms, which read the block's matrices
    auto local = [&](const unsigned char* st, int I) {
        const bf* Qs = (const bf*)(st + L::oQ);
        const bf* Ks = (const bf*)(st + L::oK);
        const bf* Np = (const bf*)(st + L::oM);
        const float* sc = (const float*)(st + L::oS);
        const int valid = f.valid(I);
        const size_t row0 = f.row0(I);
        const bf* D2 = (const bf*)(st + L::oD) + ((4 * w + g) * C + r) * 4;  // the X-part of dk, this lane's columns
        const s8 aK = op_cols(Ks, kSlC, 0, 16 * w, r, g);
#pragma unroll
        for (int ta = 0; ta < 2; ++ta) {
            const int tt = 16 * ta + r;
            const float pt = sc[kP * C + tt];
            dqT[ta] *= pt;
            mma(dqT[ta], aK, op_rows(Np, kSmR, tt, 0, g));
            const f4 q4 = unpack4(*(const s4*)(Qs + tt * kSlR + 16 * w + 4 * g));
            float pq = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) pq += q4[i] * dqT[ta][i];
            pq = all_groups(pq);
            if (tt < valid) {
                const size_t at = (row0 + tt) * a.H + s.h;
                if (g == 0) a.part_q[(size_t)plane * a.plane + at] = pq;
                *(u2*)(a.dq + at * DK + d0 + 16 * w + 4 * g) = pack4(dqT[ta] * sc[kGq * C + tt]);
                *(u2*)(a.dk + at * DK + d0 + 16 * w + 4 * g) = pack4(unpack4(*(const s4*)(D2 + 16 * ta * 4)) - pt * dkT[ta]);
            }
        }
    };
    auto fini = [&]() {
        if (a.dsf) {  // <d_final, S_T> over this wave's 16 key columns
            float acc = 0.f;
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const f4 x = *(const f4*)(a.dsf + ((size_t)s.bh * DK + d) * DV + 16 * t + 4 * g);
#pragma unroll
                for (int i = 0; i < 4; ++i) acc += x[i] * St[t][i];
            }
            acc = all_groups(row_all(acc));
            if (lane == 0) a.corr[(size_t)plane * a.B * a.H + s.bh] = acc;
        }
    };
    auto mats = [&](unsigned char* st, int mw, int ml) {
        local_matrices<DV, false, !kLoadersMakeThem>((const bf*)(st + L::oR), L::SR, nullptr, 0, (const bf*)(st + L::oO),
                                                     RD, (const float*)(st + L::oS), nullptr, (bf*)(st + L::oM), mw,
                                                     ml & 15, ml >> 4);
    };
    // This sweep moves the most bytes and wants four blocks in flight, which leaves its loader waves no registers for
    // the matrix code: the compute waves make N' in the first half of a step (measured: 259 us against 277 us).
    constexpr int PF = DV > 128 ? 2 : 4;
    if constexpr (DV > 128 || !kLoadersMakeThem) {
        run_sweep<true, PF, Load3<DK, DV, true>, kHalves>(f, smem, L::bytes, init, local, fini,
                                                          [&](unsigned char* st, int I) {
                                                              mats(st, w, lane);
                                                              state(st, I);
                                                          });
    } else {  // the loader waves make them a step ahead
        run_sweep<true, PF, Load3<DK, DV, true>, kAhead>(
            f, smem, L::bytes, init,
            [&](const unsigned char* st, int I) {
                state(const_cast<unsigned char*>(st), I);
                local(st, I);
            },
            fini, NoFirst(), mats);
    }
}

template <typename K>
bool allow_lds(K kernel, int lds) {
    if (hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds) == hipSuccess)
        return true;
    (void)hipGetLastError();
    return false;
}

template <int DK, int DV>
int launch_all(const GdnBlockArgs& a, const Areas& ar, size_t blocks, hipStream_t stream) {
    constexpr int ns3 = DV > 128 ? 2 : 3;  // stages of sweep 3 (see run_sweep); sweep 2 has three, sweep 4 two
    constexpr int lds1 = 2 * Stage1<DK>::bytes, lds2 = 3 * Stage2<DK>::bytes, lds3 = ns3 * Stage3<DV, false>::bytes,
                  lds4 = 2 * Stage3<DV, true>::bytes;
    static_assert(lds1 <= 160 * 1024 && lds2 <= 160 * 1024 && lds3 <= 160 * 1024 && lds4 <= 160 * 1024, "LDS");
    static std::atomic<uint64_t> configured{0};  // bit d: attributes set on device d
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();
        return SLA_ERR_HIP;
    }
    if (!((configured.load(std::memory_order_acquire) >> dev) & 1u)) {
        if (!allow_lds(gdn_blk_state_kernel<DK, DV>, lds1) || !allow_lds(gdn_blk_cotangent_kernel<DK, DV>, lds2) ||
            !allow_lds(gdn_blk_key_kernel<DK, DV>, lds3) || !allow_lds(gdn_blk_query_kernel<DK, DV>, lds4))
            return SLA_ERR_HIP;
        configured.fetch_or(uint64_t(1) << dev, std::memory_order_release);
    }
    const unsigned bh = (unsigned)(a.B * a.H), local = (unsigned)(blocks * (size_t)a.H);
    auto grid = [bh](unsigned slices) { return dim3(((bh + 7u) / 8u) * 8u * slices); };
    hipLaunchKernelGGL((gdn_blk_pre_kernel<DK>), dim3(local), dim3(64), 0, stream, a, ar);
    hipLaunchKernelGGL((gdn_blk_state_kernel<DK, DV>), grid(DV / kCols), dim3(kThreads), (size_t)lds1, stream, a, ar);
    hipLaunchKernelGGL((gdn_blk_cotangent_kernel<DK, DV>), grid(DV / kCols), dim3(kThreads), (size_t)lds2, stream, a, ar);
    hipLaunchKernelGGL((gdn_blk_key_kernel<DK, DV>), grid(DK / kCols), dim3(kThreads), (size_t)lds3, stream, a, ar);
    hipLaunchKernelGGL((gdn_blk_query_kernel<DK, DV>), grid(DK / kCols), dim3(kThreads), (size_t)lds4, stream, a, ar);
    return hipGetLastError() == hipSuccess ? SLA_OK : SLA_ERR_HIP;
}

template <int DK>
int launch_dv(const GdnBlockArgs& a, const Areas& ar, size_t blocks, hipStream_t stream) {
    switch (a.dim_v) {
        case 64: return launch_all<DK, 64>(a, ar, blocks, stream);
        case 128: return launch_all<DK, 128>(a, ar, blocks, stream);
        case 256: return launch_all<DK, 256>(a, ar, blocks, stream);
        default: return SLA_ERR_UNSUPPORTED;
    }
}

}  // namespace

size_t gdn_block_workspace_floats(int B, int T, int H, int dk, int dv, bool packed) {
    const size_t blocks = ws_blocks(B, T, packed), rows = packed ? (size_t)T : (size_t)B * T, bh = blocks * (size_t)H;
    (void)rows;
    return bh * kScal + bh * kPreMats * kMat / 2 + 2 * (bh * (size_t)dv * C / 2) + bh * (size_t)dk * C / 2;
}

int launch_gdn_block_sweeps(const GdnBlockArgs& a, hipStream_t stream) {
    const size_t blocks = ws_blocks(a.B, a.T, a.cu != nullptr);
    if (blocks == 0 || a.rows == 0) return SLA_OK;
    const Areas ar = areas(a.block_ws, blocks, a.rows, a.H, a.dim_k, a.dim_v);
    if (a.dim_k == 64) return launch_dv<64>(a, ar, blocks, stream);
    if (a.dim_k == 128) return launch_dv<128>(a, ar, blocks, stream);
    return SLA_ERR_UNSUPPORTED;
}

}  // namespace sla
