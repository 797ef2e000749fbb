// SLA chunkwise-parallel forward for gfx950 (MI355X): device kernels and their launch templates.
// Included by one translation unit per element type (sla_kernels_bf16.hip, sla_kernels_f32.hip).
//
// Algorithm (Sec. 3.2 "Chunkwise Parallel Training" applied to the recurrences of Sec. 5.1, with the
// gates of Eq. 4 absorbed into the operands as in Appendix A):
//
//   One workgroup owns one (batch or batch-segment, head) pair and DVW of its dv value columns; its state
//   slice S[dk, DVW] lives in fp32 MFMA accumulators for the whole sequence.  Tokens are processed in
//   blocks of 16.  For a block entered with state S0, with p_t = prod_{i<=t in block} alpha_i (per key
//   dimension for GLA, scalar otherwise) and A = p_16:
//
//       qa_t = q_t * p_t          kd_j = k_j / p_j          kb_j = k_j * A / p_j          v'_j = G^K_j v_j
//       P[t,j] = qa_t . kd_j  for j <= t, else 0            (decay between j and t: p_t / p_j)
//       out_t  = G^Q_t ( qa_t S0 + sum_j P[t,j] v'_j )      (Eq. 5-6: read-out of the updated state)
//       S_next = diag(A) S0 + sum_j kb_j^T v'_j
//
//   Every factor except 1/p_j is <= 1; 1/p_j is bounded by e^(16*5) because a block has 16 tokens
//   and GLA log-decays are required to be >= -5, so nothing overflows in fp32 or bf16.
//   (The scalar-decay variants apply their decay after the matrix products, as factors <= 1 only, and
//   have no such bound.)
//
//   Producer waves (eight where the LDS ring has eight slots, else four; producer p stages blocks p,
//   p + NP, ... into slot p): buffer loads into registers a whole ring period ahead (out-of-range tokens
//   read as zero, no branches); head softmax (Eq. 4) on DPP; decay products; operands written to LDS as
//   qa, kd (row-major), kb^T, v'^T (token-major), and the block's masked scores P^T as a ready MFMA operand.
//   Consumer waves (wave w owns value columns 16w..16w+15 of the slice): read-out, epilogue store and
//   state update on MFMA with fp32 accumulation, from registers only; no cross-wave traffic.  Blocks are
//   handed over through two LDS counters per slot; there is no workgroup barrier after start-up.
//
// MFMA layouts relied upon (16x16 tiles, wave64; r = lane%16, g = lane/16):
//   A operand: row r, contraction slots owned by group g;  B operand: column r, same slots;
//   C/D: column r, rows 4g..4g+3 in the four accumulator registers.
// A C tile of X is therefore directly the B operand of X and the A operand of X^T for a contraction
// whose slot set for group g is {4g..4g+3}; all LDS fragments are read in that slot order.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "sla.h"
#include "sla_fwd_args.h"

namespace sla {

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) short i16x4;
typedef __attribute__((ext_vector_type(8))) short i16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

static constexpr float kLog2e = 1.4426950408889634f;
static constexpr float kMinBlockDecay = 1.0e-35f;  // just under e^-80 = 1.8e-35, the smallest in-range decay of a block
static constexpr int kBlock = 16;   // tokens per state step
// A producer lane owns kEPL<DK> adjacent key dimensions of all 16 tokens of a block; with dk = 32 only the first
// 32 lanes of the wave own any (the others run along and store nothing).
template <int DK> inline constexpr int kEPL = DK >= 64 ? DK / 64 : 1;
template <int DK> inline constexpr int kOwners = DK / kEPL<DK>;
static constexpr int kWaves = 4;
static constexpr uint32_t kRsrcWord3 = 0x00020000u;  // raw buffer descriptor, 32-bit data format

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    bf16x2 t;
    t.x = (__bf16)lo;
    t.y = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, t);
}
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }

// ---------------------------------------------------------------------------------------------
// Precision policies: how two adjacent elements travel through registers, LDS and MFMA.
// ---------------------------------------------------------------------------------------------
struct PrecBF16 {
    typedef uint16_t elem;
    typedef i16x4 frag;      // four consecutive contraction slots
    typedef uint32_t pair;   // two adjacent elements
    static __device__ __forceinline__ pair zero_pair() { return 0u; }
    static __device__ __forceinline__ float lo(pair p) { return bf16_lo(p); }
    static __device__ __forceinline__ float hi(pair p) { return bf16_hi(p); }
    static __device__ __forceinline__ pair make(float a, float b) { return pack_bf16(a, b); }
    // buffer loads: a pair of adjacent elements, or a single element returned in the .lo slot
    static __device__ __forceinline__ pair bload2(__amdgpu_buffer_rsrc_t r, int voff, int soff) {
        return __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0);
    }
    static __device__ __forceinline__ pair bload1(__amdgpu_buffer_rsrc_t r, int voff, int soff) {
        return (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(r, voff, soff, 0);
    }
    static __device__ __forceinline__ float lo1(pair p) { return bf16_lo(p); }
    static __device__ __forceinline__ void store1(elem* p, float a) { *p = (uint16_t)(pack_bf16(a, 0.f) & 0xffffu); }
    static __device__ __forceinline__ frag from_acc(f32x4 c) {
        u32x2 t;
        t.x = pack_bf16(c[0], c[1]);
        t.y = pack_bf16(c[2], c[3]);
        return __builtin_bit_cast(frag, t);
    }
    static __device__ __forceinline__ f32x4 to_acc(frag f) {
        const u32x2 t = __builtin_bit_cast(u32x2, f);
        return f32x4{bf16_lo(t.x), bf16_hi(t.x), bf16_lo(t.y), bf16_hi(t.y)};
    }
    static __device__ __forceinline__ void mma32(f32x4& c, frag a0, frag a1, frag b0, frag b1) {
        i16x8 a = __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7);
        i16x8 b = __builtin_shufflevector(b0, b1, 0, 1, 2, 3, 4, 5, 6, 7);
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                    0, 0);
    }
    // A 16-slot contraction is issued as the 32-slot instruction with the upper slots zero, so that
    // every accumulation chain consists of one MFMA opcode only: a 16x16x16 issued right behind a
    // 16x16x32 on the same accumulator read a partially written C on gfx950 (the first two result
    // registers lacked the last 16x16x32's contribution).
    static __device__ __forceinline__ void mma16(f32x4& c, frag a, frag b) {
        const frag z = {0, 0, 0, 0};
        mma32(c, a, z, b, z);
    }
    // The 16-slot opcode itself, for accumulators that the 32-slot opcode never writes (the state tiles).
    static __device__ __forceinline__ void mma16_only(f32x4& c, frag a, frag b) {
        c = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, b, c, 0, 0, 0);
    }
};

struct PrecF32 {
    typedef float elem;
    typedef f32x4 frag;
    typedef f32x2 pair;
    static __device__ __forceinline__ pair zero_pair() { return f32x2{0.f, 0.f}; }
    static __device__ __forceinline__ float lo(pair p) { return p.x; }
    static __device__ __forceinline__ float hi(pair p) { return p.y; }
    static __device__ __forceinline__ pair make(float a, float b) { return f32x2{a, b}; }
    static __device__ __forceinline__ pair bload2(__amdgpu_buffer_rsrc_t r, int voff, int soff) {
        return __builtin_bit_cast(f32x2, __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0));
    }
    static __device__ __forceinline__ pair bload1(__amdgpu_buffer_rsrc_t r, int voff, int soff) {
        return f32x2{__uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0)), 0.f};
    }
    static __device__ __forceinline__ float lo1(pair p) { return p.x; }
    static __device__ __forceinline__ void store1(elem* p, float a) { *p = a; }
    static __device__ __forceinline__ frag from_acc(f32x4 c) { return c; }
    static __device__ __forceinline__ f32x4 to_acc(frag f) { return f; }
    static __device__ __forceinline__ void mma16(f32x4& c, frag a, frag b) {
#pragma unroll
        for (int i = 0; i < 4; ++i) c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[i], b[i], c, 0, 0, 0);
    }
    static __device__ __forceinline__ void mma16_only(f32x4& c, frag a, frag b) { mma16(c, a, b); }
    static __device__ __forceinline__ void mma32(f32x4& c, frag a0, frag a1, frag b0, frag b1) {
        mma16(c, a0, b0);
        mma16(c, a1, b1);
    }
};

// Store N consecutive elements (N*sizeof(elem) is 4, 8, 16, 32 or 64 bytes; dst aligned to min(16, bytes),
// or to min(8, bytes) with W8, which limits 2-byte element stores to 8 bytes each).
template <class P, int N, bool W8 = false>
__device__ __forceinline__ void store_run(typename P::elem* dst, const float (&x)[N]) {
    if constexpr (sizeof(typename P::elem) == 2) {
        static_assert(N % 2 == 0, "bf16 runs are stored in pairs");
        uint32_t w[N / 2];
#pragma unroll
        for (int i = 0; i < N / 2; ++i) w[i] = pack_bf16(x[2 * i], x[2 * i + 1]);
        if constexpr (N == 2) {
            *(uint32_t*)dst = w[0];
        } else if constexpr (N == 4) {
            *(u32x2*)dst = u32x2{w[0], w[1]};
        } else if constexpr (W8) {
#pragma unroll
            for (int i = 0; i < N / 4; ++i) ((u32x2*)dst)[i] = u32x2{w[2 * i], w[2 * i + 1]};
        } else {
#pragma unroll
            for (int i = 0; i < N / 8; ++i) ((u32x4*)dst)[i] = u32x4{w[4 * i], w[4 * i + 1], w[4 * i + 2], w[4 * i + 3]};
        }
    } else {
        if constexpr (N == 1) {
            *dst = x[0];
        } else if constexpr (N == 2) {
            *(f32x2*)dst = f32x2{x[0], x[1]};
        } else {
#pragma unroll
            for (int i = 0; i < N / 4; ++i) ((f32x4*)dst)[i] = f32x4{x[4 * i], x[4 * i + 1], x[4 * i + 2], x[4 * i + 3]};
        }
    }
}

// ---------------------------------------------------------------------------------------------
// LDS geometry
// ---------------------------------------------------------------------------------------------
// Key dimensions inside the row-major q and k rows are stored permuted within groups of 32:
// d = 32 S + 16 u + 4 g + i sits at 32 S + 8 g + 4 u + i.  Lane group g of an MFMA feeds the slots
// {4g..4g+3} of two adjacent 16-dimension tiles; with this order they are 8 adjacent elements (one
// 16-byte read with 2-byte elements).  Adjacent even/odd dimensions stay adjacent.
__host__ __device__ constexpr int perm32(int d) { return (d & ~31) | ((d & 12) << 1) | ((d & 16) >> 2) | (d & 3); }
// Row and column (of token group 0) of key dimension d in the k^T array.
__host__ __device__ constexpr int kbt_row(int d) { return ((d >> 5) << 4) | (d & 15); }
__host__ __device__ constexpr int kbt_col(int d) { return ((d >> 4) & 1) * 4; }
template <class P, int VAR, int DK, int DVW>
struct Smem {
    typedef typename P::elem elem;
    static constexpr int kPad = 16 / sizeof(elem);   // 16 bytes of padding per row
    static constexpr int RS = DK + kPad;             // row stride of the row-major [token][d] arrays
    // Token-major [d or n][token] arrays: a producer lane writes rows 2l and 2l+1, a consumer lane
    // reads row r.  With 2-byte elements a stride of 40 bytes (10 banks) puts the 16 lanes that an
    // 8-byte access serves per cycle on 16 distinct bank pairs for the consumers' pattern.
    static constexpr int TS = kBlock + 4;
    // k^T of the block ("KBT"): row (d / 32) * 16 + d % 16 holds key dimensions d and d + 16 of the 16
    // tokens, ordered [token / 4][(d / 16) % 2][token % 4], so that the two 4-token fragments a consumer
    // lane feeds to the tiles of d and d + 16 are one 16-byte read.  Rows are padded to 40 elements.
    static constexpr int KTS = 2 * kBlock + 8;
    // One slot holds the operands of one 16-token block.
    static constexpr size_t oQA = 0;
    static constexpr size_t oKD = oQA + sizeof(elem) * kBlock * RS;
    static constexpr size_t oKBT = oKD + sizeof(elem) * kBlock * RS;
    // Scalar-decay variants with 2-byte elements stage no k^T: their k rows go to LDS unscaled, and the consumers take
    // the transposed fragments from those rows with the transposing LDS read (ds_read_b64_tr_b16).
    static constexpr bool kTR = VAR != SLA_GLA && sizeof(elem) == 2;
    static constexpr size_t oVT = oKBT + (kTR ? 0 : sizeof(elem) * (DK / 2) * KTS);
    static constexpr size_t oEA = oVT + sizeof(elem) * DVW * TS;
    static constexpr size_t oGQ = oEA + (VAR == SLA_GLA ? sizeof(float) * DK : 0);
    static constexpr size_t oGK = oGQ + sizeof(float) * kBlock;
    // masked scores P^T of the block as the consumers' MFMA operand: one 4-slot fragment per lane
    static constexpr size_t oPT = oGK + sizeof(float) * kBlock;
    // scalar-decay variants: per token the cumulative log2-decay c_t ("P1") and beta_t ("BT"); delta
    // rule: the inverse Tm = (I + L)^-1 [16][16] of the block (built in fp32 in this area, left in the element type)
    static constexpr size_t oP1 = oPT + 64 * 4 * sizeof(elem);
    static constexpr size_t oBT = oP1 + sizeof(float) * kBlock;
    // scalar-decay variants, for the consumers: per token 2^c_t ("E1"), 2^(c_16 - c_t) ("EB") and, delta rule,
    // beta_t 2^c_t ("EJ"), so that the consumer waves spend no transcendental instructions on them
    static constexpr size_t oE1 = oBT + sizeof(float) * kBlock;
    static constexpr size_t oEB = oE1 + (VAR != SLA_GLA ? sizeof(float) * kBlock : 0);
    static constexpr size_t oEJ = oEB + (VAR != SLA_GLA ? sizeof(float) * kBlock : 0);
    static constexpr size_t oTM = oEJ + (VAR == SLA_GDN ? sizeof(float) * kBlock : 0);
    // The block's output tile [16 tokens][DVW], written by the consumer waves (each its 16 columns) and stored to
    // global memory by the slot's producer wave as whole rows.  A row is UPR units of four elements; unit c of
    // token t sits at position c ^ (t % UPR) of its row, which spreads both access patterns over the banks.
    static constexpr int UPR = DVW / 4;
    static constexpr size_t oOUT = oTM + (VAR == SLA_GDN ? sizeof(float) * kBlock * kBlock : 0);
    static constexpr size_t bytes = oOUT + sizeof(elem) * kBlock * DVW;
    static_assert(bytes % 16 == 0, "slots keep 16-byte alignment");
    static constexpr size_t limit = 160 * 1024;
    static constexpr size_t flag_bytes = 2 * kMaxSlots * sizeof(int);  // ready[] and done[] counters
    // Ring of slots, one producer wave per slot: eight where they fit in the LDS of a CU, else four.
    static constexpr int slots = (kMaxSlots * bytes + flag_bytes <= limit) ? kMaxSlots : 4;
    // Consumers request a block's operands a block ahead into a second set of registers -- except for the
    // delta rule, whose operand set is large: with twelve waves per CU there are 168 registers per lane.
    static constexpr bool prefetch = VAR != SLA_GDN;
    static constexpr size_t oFlags = slots * bytes;
    static constexpr size_t total = oFlags + flag_bytes;
    static constexpr int threads = (kWaves + slots) * 64;
};

// Output of a block.  A consumer lane holds four adjacent value columns (unit 4 cw + g) of token r and parks them
// in the slot's output tile; the slot's producer wave later writes the tile to global memory, a whole row of the
// slice per token, with the non-temporal hint.  Measured on the benchmark's address streams (loads as the kernel
// issues them, no arithmetic): 32-byte pieces written by four waves at different times with ordinary stores 84 us,
// whole 128-byte rows with streaming stores 48.5 us (reads alone: 40 us) -- written lines otherwise compete with
// the input streams in the L2.
template <class P, int DVW>
__device__ __forceinline__ void park_out4(typename P::elem* tile, int r, int unit, const float (&x)[4]) {
    constexpr int UPR = DVW / 4;
    typename P::elem* dst = tile + (r * UPR + (unit ^ (r & (UPR - 1)))) * 4;
    if constexpr (sizeof(typename P::elem) == 2) {
        *(u32x2*)dst = u32x2{pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3])};
    } else {
        *(f32x4*)dst = f32x4{x[0], x[1], x[2], x[3]};
    }
}

// out_row: address of column n0 of the block's first token; tstride: elements per token; nvalid: tokens of the
// block inside the sequence.  Lane l handles unit l % UPR of tokens l / UPR, l / UPR + 64 / UPR, ...
template <class P, int DVW>
__device__ __forceinline__ void store_out_tile(const typename P::elem* tile, typename P::elem* out_row, size_t tstride,
                                               int nvalid, int lane) {
    constexpr int UPR = DVW / 4;
    constexpr int TPI = 64 / UPR;  // tokens per store instruction
    const int u = lane % UPR;
#pragma unroll
    for (int i = 0; i < kBlock / TPI; ++i) {
        const int t = lane / UPR + TPI * i;
        const typename P::elem* src = tile + (t * UPR + (u ^ (t & (UPR - 1)))) * 4;
        typename P::elem* dst = out_row + (size_t)t * tstride + 4 * u;
        if constexpr (sizeof(typename P::elem) == 2) {
            const u32x2 w = *(const u32x2*)src;
            if (t < nvalid) __builtin_nontemporal_store(w, (u32x2*)dst);
        } else {
            const f32x4 w = *(const f32x4*)src;
            if (t < nvalid) __builtin_nontemporal_store(w, (f32x4*)dst);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Per-lane staging registers for one 16-token block (what a producer wave works on).
// Lane l owns EPL = max(DK/64, 1) adjacent key dimensions (d = EPL*l ...) of all 16 tokens of the block,
// and for V two adjacent value columns of NI = DVW/8 consecutive tokens.  For the gates, lane l
// holds the logits of token l/4 for heads l%4, l%4 + 4, ... (HG registers per gate), so that the
// reduction over heads stays inside a quad and runs on DPP.
// ---------------------------------------------------------------------------------------------
template <class P, int VAR, int DK, int DVW, int HG>
struct Stage {
    typedef typename P::pair pair;
    static constexpr int NI = DVW / 8;
    pair q[kBlock], k[kBlock];
    pair ld[VAR == SLA_GLA ? kBlock : 1];
    pair v[NI];
    float ql[HG], kl[HG];
    float ql_own, kl_own;
    float sc_ld, sc_beta;  // delta rule: scalar log-decay and beta of token lane%16
};

// Buffer descriptors of one batch row and the per-lane byte offsets into them.  A descriptor spans
// exactly the T tokens of batch b, so any access to a token >= T is out of range and returns zero.
template <class P, int VAR, int DK, int DVW, int HG>
struct Loader {
    typedef typename P::elem elem;
    typedef Stage<P, VAR, DK, DVW, HG> stage_t;
    static constexpr int EPL = kEPL<DK>;
    static constexpr int NI = DVW / 8;
    static constexpr int LPR = DVW / 2;
    __amdgpu_buffer_rsrc_t rq, rk, rv, rld, rql, rkl, rbt;
    int voff_qk, voff_v, voff_lg, voff_own, voff_sc;
    int tstride_qk, tstride_v, tstride_lg;  // bytes per token
    int H;
    bool has_kl;

    // row_tok: index of the first token of the row in the [B*T] token space; T: tokens of the row.  With the
    // head-major layout the descriptors of q, k, v and the GLA decay start at this head's own rows.
    __device__ __forceinline__ void init(const KArgs& a, size_t row_tok, int T, int h, int n0, int lane) {
        H = a.H;
        has_kl = a.kl != nullptr;
        const int head = h;  // the logits keep their [B,T,H] layout
        const int HW = a.head_major ? 1 : H;  // heads interleaved within a token of q, k, v
        tstride_qk = HW * DK * (int)sizeof(elem);
        tstride_v = HW * a.dv * (int)sizeof(elem);
        tstride_lg = H * 4;
        size_t row_qk = row_tok * H * DK, row_v = row_tok * H * a.dv;
        const size_t row_lg = row_tok * H;
        if (a.head_major) {  // row_tok = b * T_all + t0  ->  ((b * H + h) * T_all + t0) tokens of width d
            const size_t bb = row_tok / a.T, t0 = row_tok % a.T, tok = (bb * H + h) * a.T + t0;
            row_qk = tok * DK;
            row_v = tok * a.dv;
            h = 0;
        }
        rq = __builtin_amdgcn_make_buffer_rsrc((void*)((const elem*)a.q + row_qk), 0, T * tstride_qk, kRsrcWord3);
        rk = __builtin_amdgcn_make_buffer_rsrc((void*)((const elem*)a.k + row_qk), 0, T * tstride_qk, kRsrcWord3);
        rv = __builtin_amdgcn_make_buffer_rsrc((void*)((const elem*)a.v + row_v), 0, T * tstride_v, kRsrcWord3);
        if constexpr (VAR == SLA_GLA)
            rld = __builtin_amdgcn_make_buffer_rsrc((void*)((const elem*)a.ld + row_qk), 0, T * tstride_qk, kRsrcWord3);
        rql = __builtin_amdgcn_make_buffer_rsrc((void*)(a.ql + row_lg), 0, T * tstride_lg, kRsrcWord3);
        // without write-gate logits the descriptor is empty: every load returns 0 and the gate is forced to 1
        rkl = __builtin_amdgcn_make_buffer_rsrc((void*)(has_kl ? a.kl + row_lg : a.ql), 0, has_kl ? T * tstride_lg : 0,
                                                kRsrcWord3);
        voff_qk = (h * DK + EPL * lane) * (int)sizeof(elem);
        const int p = lane % LPR, tb = (lane / LPR) * NI;
        voff_v = tb * tstride_v + (h * a.dv + n0 + 2 * p) * (int)sizeof(elem);
        voff_lg = (lane >> 2) * tstride_lg + (lane & 3) * 4;
        voff_own = (lane >> 2) * tstride_lg + head * 4;
        if constexpr (VAR == SLA_GDN) {
            rld = __builtin_amdgcn_make_buffer_rsrc((void*)((const float*)a.ld + row_lg), 0, T * tstride_lg, kRsrcWord3);
            rbt = __builtin_amdgcn_make_buffer_rsrc((void*)(a.beta + row_lg), 0, T * tstride_lg, kRsrcWord3);
            voff_sc = (lane & 15) * tstride_lg + head * 4;
        }
    }

    // The loads address token (base + i) of the row: base lives in the per-lane byte offsets, which
    // advance() moves from block to block; i * stride is wave-uniform and loop-invariant, so the scalar
    // offsets of all loads are constants held in SGPRs.
    __device__ __forceinline__ void advance(int ntok) {
        voff_qk += ntok * tstride_qk;
        voff_v += ntok * tstride_v;
        voff_lg += ntok * tstride_lg;
        voff_own += ntok * tstride_lg;
        if constexpr (VAR == SLA_GDN) voff_sc += ntok * tstride_lg;
    }
    __device__ __forceinline__ void load_q(stage_t& st, int i) const {
        const int so = i * tstride_qk;
        st.q[i] = (EPL == 2) ? P::bload2(rq, voff_qk, so) : P::bload1(rq, voff_qk, so);
    }
    __device__ __forceinline__ void load_k(stage_t& st, int i) const {
        const int so = i * tstride_qk;
        st.k[i] = (EPL == 2) ? P::bload2(rk, voff_qk, so) : P::bload1(rk, voff_qk, so);
    }
    __device__ __forceinline__ void load_ld(stage_t& st, int i) const {
        if constexpr (VAR == SLA_GLA) {
            const int so = i * tstride_qk;
            st.ld[i] = (EPL == 2) ? P::bload2(rld, voff_qk, so) : P::bload1(rld, voff_qk, so);
        }
    }
    __device__ __forceinline__ void load_v(stage_t& st) const {
#pragma unroll
        for (int i = 0; i < NI; ++i) st.v[i] = P::bload2(rv, voff_v, i * tstride_v);
    }
    __device__ __forceinline__ void load_logits(stage_t& st, int lane) const {
        const int sub = lane & 3;
#pragma unroll
        for (int i = 0; i < HG; ++i) {
            // heads beyond H never win the max and add exp(-inf) = 0; tokens beyond T read 0 (equal scores)
            const bool head_ok = sub + 4 * i < H;
            const float x = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rql, voff_lg, 16 * i, 0));
            const float y = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rkl, voff_lg, 16 * i, 0));
            st.ql[i] = head_ok ? x : -INFINITY;
            st.kl[i] = head_ok ? y : -INFINITY;
        }
        st.ql_own = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rql, voff_own, 0, 0));
        st.kl_own = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rkl, voff_own, 0, 0));
    }
    // delta rule: tokens beyond T read log-decay 0 (factor 1) and beta 0 (no write)
    __device__ __forceinline__ void load_scalars(stage_t& st) const {
        if constexpr (VAR == SLA_GDN) {
            st.sc_ld = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rld, voff_sc, 0, 0));
            st.sc_beta = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rbt, voff_sc, 0, 0));
        }
    }
    __device__ __forceinline__ void load(stage_t& st, int lane) const {
        load_logits(st, lane);
        load_scalars(st);
#pragma unroll
        for (int i = 0; i < kBlock; ++i) load_ld(st, i);
#pragma unroll
        for (int i = 0; i < kBlock; ++i) load_q(st, i);
#pragma unroll
        for (int i = 0; i < kBlock; ++i) load_k(st, i);
        load_v(st);
    }
};

// Exchange inside a quad of lanes on DPP: lane ^ 1 and lane ^ 2.
__device__ __forceinline__ float quad_xor1(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xf, 0xf, false));
}
__device__ __forceinline__ float quad_xor2(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x4E, 0xf, 0xf, false));
}

// Value of lane N of this lane's row of 16 lanes.
template <int N>
__device__ __forceinline__ float row_bcast(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x150 + N, 0xf, 0xf, false));
}

// GLA state decay: S[16s + 4g + i][.] *= A[16s + 4g + i], the factor taken from lane 4(s%4) + i of the
// row, register ea0 (s < 4) or ea1.
template <int NT, int s = 0>
__device__ __forceinline__ void scale_state_rows(f32x4 (&S)[NT], float ea0, float ea1) {
    if constexpr (s < NT) {
        const float e = s < 4 ? ea0 : ea1;
        S[s][0] *= row_bcast<4 * (s & 3) + 0>(e);
        S[s][1] *= row_bcast<4 * (s & 3) + 1>(e);
        S[s][2] *= row_bcast<4 * (s & 3) + 2>(e);
        S[s][3] *= row_bcast<4 * (s & 3) + 3>(e);
        scale_state_rows<NT, s + 1>(S, ea0, ea1);
    }
}

// Forward substitution for the 16x16 unit-lower-triangular inverse of the delta rule, one column per lane:
// x[j] = [j == c] - sum_{i<j} L[j][i] x[i], where lane i of the row holds Lc[j] = -L[j][i].  The sums are taken
// column by column ("right-looking"): once x[i] is final, every later row takes its term L[j][i] x[i], so that
// consecutive instructions write different registers and none waits for the one before it.
template <int I, int J>
__device__ __forceinline__ void tm_update(float (&x)[kBlock], const float (&Lc)[kBlock]) {
    if constexpr (J < kBlock) {
        // x[j] += (-L[j][i] from lane i of the row) * x[i] in one instruction.  Lc was written long before, so
        // the DPP read needs no wait states; x[i] and x[j] are ordinary operands.
        asm("v_fmac_f32_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf"
            : "+v"(x[J])
            : "v"(Lc[J]), "v"(x[I]), "n"(I));
        tm_update<I, J + 1>(x, Lc);
    }
}
template <int I>
__device__ __forceinline__ void tm_substitute(float (&x)[kBlock], const float (&Lc)[kBlock]) {
    if constexpr (I + 1 < kBlock) {
        tm_update<I, I + 1>(x, Lc);
        tm_substitute<I + 1>(x, Lc);
    }
}

// softmax over heads for the token of this quad (Eq. 4); returns the gate of head h.
template <int HG>
__device__ __forceinline__ float head_gate(const float (&x)[HG], float own) {
    float m = x[0];
#pragma unroll
    for (int i = 1; i < HG; ++i) m = fmaxf(m, x[i]);
    m = fmaxf(m, quad_xor1(m));
    m = fmaxf(m, quad_xor2(m));
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < HG; ++i) s += fast_exp2((x[i] - m) * kLog2e);
    s += quad_xor1(s);
    s += quad_xor2(s);
    return fast_exp2((own - m) * kLog2e) * fast_rcp(s);
}

// Gates of the 16 tokens of block blk (token lane/4) from the staged logits; parked in LDS for the
// epilogue (read gate) and for the values (write gate).  The logits are then reloaded for next_tok0.
template <class P, int VAR, int DK, int DVW, int HG>
__device__ __forceinline__ void stage_gates(Stage<P, VAR, DK, DVW, HG>& st, const Loader<P, VAR, DK, DVW, HG>& ldr,
                                            unsigned char* buf, int blk, int next_tok0, int lane) {
    typedef Smem<P, VAR, DK, DVW> L;
    float* GQ = (float*)(buf + L::oGQ);
    float* GK = (float*)(buf + L::oGK);
    const float gq = head_gate<HG>(st.ql, st.ql_own);
    const float gk = ldr.has_kl ? head_gate<HG>(st.kl, st.kl_own) : 1.f;
    if ((lane & 3) == 0) {
        GQ[kBlock * blk + (lane >> 2)] = gq;
        GK[kBlock * blk + (lane >> 2)] = gk;
    }
    ldr.load_logits(st, lane);
}

// Values of block blk: v' = G^K v (delta rule: beta G^K v), transposed to [column][token].  The gates
// (and beta) were written by this same wave earlier; LDS operations of one wave execute in order.
template <class P, int VAR, int DK, int DVW, int HG>
__device__ __forceinline__ void stage_values(Stage<P, VAR, DK, DVW, HG>& st, const Loader<P, VAR, DK, DVW, HG>& ldr,
                                             unsigned char* buf, int blk, int next_tok0, int lane) {
    typedef typename P::elem elem;
    typedef Smem<P, VAR, DK, DVW> L;
    constexpr int NI = DVW / 8;
    constexpr int LPR = DVW / 2;
    elem* VT = (elem*)(buf + L::oVT);
    const float* GK = (const float*)(buf + L::oGK);
    const float* BT = (const float*)(buf + L::oBT) + blk * kBlock;
    const int p = lane % LPR, tb = (lane / LPR) * NI;
    __builtin_amdgcn_wave_barrier();
    float gkv[NI];
    if constexpr (NI >= 4) {
#pragma unroll
        for (int i = 0; i < NI / 4; ++i) {
            const f32x4 t = *(const f32x4*)(GK + kBlock * blk + tb + 4 * i);
            gkv[4 * i] = t[0]; gkv[4 * i + 1] = t[1]; gkv[4 * i + 2] = t[2]; gkv[4 * i + 3] = t[3];
        }
    } else {
        const f32x2 t = *(const f32x2*)(GK + kBlock * blk + tb);
        gkv[0] = t[0]; gkv[1] = t[1];
    }
    if constexpr (VAR == SLA_GDN) {
        if constexpr (NI >= 4) {
#pragma unroll
            for (int i = 0; i < NI / 4; ++i) {
                const f32x4 t = *(const f32x4*)(BT + tb + 4 * i);
                gkv[4 * i] *= t[0]; gkv[4 * i + 1] *= t[1]; gkv[4 * i + 2] *= t[2]; gkv[4 * i + 3] *= t[3];
            }
        } else {
            const f32x2 t = *(const f32x2*)(BT + tb);
            gkv[0] *= t[0]; gkv[1] *= t[1];
        }
    }
    float c0[NI], c1[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        c0[i] = P::lo(st.v[i]) * gkv[i];
        c1[i] = P::hi(st.v[i]) * gkv[i];
    }
    ldr.load_v(st);
    store_run<P, NI, true>(VT + (2 * p) * L::TS + kBlock * blk + tb, c0);
    store_run<P, NI, true>(VT + (2 * p + 1) * L::TS + kBlock * blk + tb, c1);
}

// Inclusive sum over the 16 lanes of a DPP row (lane r gets x_0 + ... + x_r).
__device__ __forceinline__ float row_prefix_sum(float x) {
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x111, 0xf, 0xf, true));
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x112, 0xf, 0xf, true));
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x114, 0xf, 0xf, true));
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x118, 0xf, 0xf, true));
    return x;
}

// ---------------------------------------------------------------------------------------------
// Producer for the scalar-decay variants (RetNet, delta rule).  The decay of a token is one number per
// head, so it is applied after the matrix products instead of being folded into q and k: q and k go
// to LDS as loaded (k also transposed), and the block's cumulative log2-decay c_t = log2 p_t is staged
// for the consumers, which scale the read-out by 2^c_t, the state by A = 2^c_16 and the state-step
// values by 2^(c_16 - c_j).  Scores are scaled here: P[t,j] = (q_t . k_j) 2^(c_t - c_j) for j <= t.
// Every factor is <= 1, whatever the decay.
// ---------------------------------------------------------------------------------------------
template <class P, int VAR, int DK, int DVW, int HG, bool SO>
__device__ __forceinline__ void produce_block_scalar(Stage<P, VAR, DK, DVW, HG>& st,
                                                     const Loader<P, VAR, DK, DVW, HG>& ldr, unsigned char* buf, int blk,
                                                     int tok0, int next_tok0, int T, float log2_gamma, int lane) {
    typedef typename P::elem elem;
    typedef typename P::pair pair;
    typedef typename P::frag frag;
    typedef Smem<P, VAR, DK, DVW> L;
    constexpr int EPL = kEPL<DK>;
    const bool owner = lane < kOwners<DK>;  // always true for dk >= 64
    constexpr int NTILE = DK / 16;
    elem* QA = (elem*)(buf + L::oQA);
    elem* KD = (elem*)(buf + L::oKD);
    elem* KBT = (elem*)(buf + L::oKBT);
    float* TM = (float*)(buf + L::oTM) + blk * kBlock * kBlock;
    float* C2 = (float*)(buf + L::oP1) + blk * kBlock;  // cumulative log2-decay of the block's tokens
    float* BT = (float*)(buf + L::oBT) + blk * kBlock;
    const int r = lane & 15, g = lane >> 4;

    // c_t of token r (the four lane groups hold the same value)
    float c_lane;
    if constexpr (VAR == SLA_RETNET) {
        int nvalid = T - tok0;
        nvalid = nvalid < 0 ? 0 : (nvalid > kBlock ? kBlock : nvalid);
        const int n = r + 1 < nvalid ? r + 1 : nvalid;  // tokens past T do not decay the state
        c_lane = (float)n * log2_gamma;
    } else {
        c_lane = row_prefix_sum(st.sc_ld * kLog2e);
        if (lane < kBlock) BT[lane] = st.sc_beta;
    }
    if (lane < kBlock) {
        C2[lane] = c_lane;
        const float e1 = fast_exp2(c_lane);
        ((float*)(buf + L::oE1))[blk * kBlock + lane] = e1;
        ((float*)(buf + L::oEB))[blk * kBlock + lane] = fast_exp2(row_bcast<15>(c_lane) - c_lane);
        if constexpr (VAR == SLA_GDN) ((float*)(buf + L::oEJ))[blk * kBlock + lane] = st.sc_beta * e1;
    }
    ldr.load_scalars(st);

    stage_gates<P, VAR, DK, DVW, HG>(st, ldr, buf, blk, next_tok0, lane);

    // q and k as loaded (the state-only pass needs the k rows only where the consumers read k^T from them)
    elem* qrow = QA + (kBlock * blk) * L::RS + perm32(EPL * lane);
    elem* krow = KD + (kBlock * blk) * L::RS + perm32(EPL * lane);
    if constexpr (!SO || L::kTR) {
#pragma unroll
        for (int i = 0; i < kBlock; ++i) {
            if constexpr (EPL == 2) {
                if constexpr (!SO) *(pair*)(qrow + i * L::RS) = st.q[i];
                *(pair*)(krow + i * L::RS) = st.k[i];
            } else if (owner) {
                if constexpr (!SO) P::store1(qrow + i * L::RS, P::lo(st.q[i]));
                P::store1(krow + i * L::RS, P::lo(st.k[i]));
            }
            if constexpr (!SO) ldr.load_q(st, i);
        }
    }
    // k transposed (variants whose consumers cannot take it from the rows)
#pragma unroll
    for (int e = 0; e < (L::kTR ? 0 : EPL); ++e) {
        float kt[kBlock];
#pragma unroll
        for (int i = 0; i < kBlock; ++i) kt[i] = (EPL == 2 && e == 1) ? P::hi(st.k[i]) : P::lo(st.k[i]);
        elem* dst = KBT + kbt_row(EPL * lane + e) * L::KTS + kbt_col(EPL * lane + e);
#pragma unroll
        for (int tg = 0; tg < 4; ++tg) {
            const float four[4] = {kt[4 * tg], kt[4 * tg + 1], kt[4 * tg + 2], kt[4 * tg + 3]};
            if (owner) store_run<P, 4>(dst + 8 * tg, four);
        }
    }
#pragma unroll
    for (int i = 0; i < kBlock; ++i) ldr.load_k(st, i);

    // scores of the block from this wave's own rows
    __builtin_amdgcn_wave_barrier();
    [[maybe_unused]] frag fk_[NTILE];
    [[maybe_unused]] f32x4 cj;
    if constexpr (!SO) {
        f32x4 pT = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < NTILE; s += 2) {
            const frag q0 = *(const frag*)(QA + (kBlock * blk + r) * L::RS + 16 * s + 8 * g);
            const frag q1 = *(const frag*)(QA + (kBlock * blk + r) * L::RS + 16 * s + 8 * g + 4);
            fk_[s] = *(const frag*)(KD + (kBlock * blk + r) * L::RS + 16 * s + 8 * g);
            fk_[s + 1] = *(const frag*)(KD + (kBlock * blk + r) * L::RS + 16 * s + 8 * g + 4);
            P::mma32(pT, fk_[s], fk_[s + 1], q0, q1);  // P^T[j][t] = k_j . q_t
        }
        cj = *(const f32x4*)(C2 + 4 * g);  // rows j = 4g + i
#pragma unroll
        for (int i = 0; i < 4; ++i) pT[i] = (4 * g + i <= r) ? pT[i] * fast_exp2(c_lane - cj[i]) : 0.f;
        ((frag*)(buf + L::oPT))[blk * 64 + lane] = P::from_acc(pT);
    }

    stage_values<P, VAR, DK, DVW, HG>(st, ldr, buf, blk, next_tok0, lane);

    // delta rule: Tm = (I + L)^-1 with L[j][t] = beta_j 2^(c_j - c_t) (k_j . k_t) for t < j (strictly lower)
    if constexpr (VAR == SLA_GDN && !SO) {
        f32x4 G = {0.f, 0.f, 0.f, 0.f};  // G[j][t] = k_j . k_t: lane holds column t = r, rows j = 4g + i
#pragma unroll
        for (int s = 0; s < NTILE; s += 2) P::mma32(G, fk_[s], fk_[s + 1], fk_[s], fk_[s + 1]);
        const f32x4 btj = *(const f32x4*)(BT + 4 * g);
        // L goes through LDS once, transposed, so that every lane ends up with a whole column of it:
        // Lc[j] = L[j][r].  The substitution then runs on registers: the factor L[j][i] of step (j, i) is
        // taken from lane i of the row by a DPP broadcast.
        f32x4 lv;
#pragma unroll
        for (int i = 0; i < 4; ++i) lv[i] = (4 * g + i > r) ? -(btj[i] * fast_exp2(cj[i] - c_lane) * G[i]) : 0.f;  // -L
        *(f32x4*)(TM + r * kBlock + 4 * g) = lv;
        __builtin_amdgcn_wave_barrier();
        float Lc[kBlock];
#pragma unroll
        for (int j4 = 0; j4 < kBlock; j4 += 4) {
            const f32x4 t = *(const f32x4*)(TM + r * kBlock + j4);
            Lc[j4] = t[0]; Lc[j4 + 1] = t[1]; Lc[j4 + 2] = t[2]; Lc[j4 + 3] = t[3];  // -L, for the fmac
        }
        // forward substitution, column c = r of the inverse in every lane (the four lane groups repeat it):
        // x_j = [j == c] - sum_{i<j} L[j][i] x_i
        // A DPP operand must not have been written by the two instructions before its use: pin all sixteen
        // factors behind two wait states before the first of them is read across lanes.
        asm volatile("s_nop 1"
                     : "+v"(Lc[0]), "+v"(Lc[1]), "+v"(Lc[2]), "+v"(Lc[3]), "+v"(Lc[4]), "+v"(Lc[5]), "+v"(Lc[6]), "+v"(Lc[7]),
                       "+v"(Lc[8]), "+v"(Lc[9]), "+v"(Lc[10]), "+v"(Lc[11]), "+v"(Lc[12]), "+v"(Lc[13]), "+v"(Lc[14]),
                       "+v"(Lc[15]));
        float x[kBlock];
#pragma unroll
        for (int j = 0; j < kBlock; ++j) x[j] = (j == r) ? 1.f : 0.f;
        tm_substitute<0>(x, Lc);
        __builtin_amdgcn_wave_barrier();  // every lane has read L before it is overwritten
        // the inverse replaces L in the same area, in the element type, ready as the consumers' MFMA operand
        if (g == 0) {
            elem* TMo = (elem*)TM;
#pragma unroll
            for (int j = 0; j < kBlock; ++j) P::store1(TMo + j * kBlock + r, x[j]);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Producer: one 16-token block (index blk of the staged chunk) from registers to LDS.
// ---------------------------------------------------------------------------------------------
// Every staging register is reloaded with the same block of the next chunk (token next_tok0 + i) right
// after its last use, so the loads are spread through the arithmetic instead of queueing up in a burst.
// This is the path of GLA, whose decay is a vector over the key dimensions and has to be folded into
// q and k element by element.
template <class P, int VAR, int DK, int DVW, int HG, bool SO>
__device__ __forceinline__ void produce_block(Stage<P, VAR, DK, DVW, HG>& st, const Loader<P, VAR, DK, DVW, HG>& ldr,
                                              unsigned char* buf, int blk, int tok0, int next_tok0, int T,
                                              float decay_const, float (&dacc)[kEPL<DK>], int lane,
                                              unsigned int* status) {
    if constexpr (VAR != SLA_GLA) {
        produce_block_scalar<P, VAR, DK, DVW, HG, SO>(st, ldr, buf, blk, tok0, next_tok0, T, decay_const, lane);
        return;
    }
    typedef typename P::elem elem;
    typedef typename P::pair pair;
    typedef Smem<P, VAR, DK, DVW> L;
    constexpr int EPL = kEPL<DK>;
    const bool owner = lane < kOwners<DK>;  // always true for dk >= 64
    elem* QA = (elem*)(buf + L::oQA);
    elem* KD = (elem*)(buf + L::oKD);
    elem* KBT = (elem*)(buf + L::oKBT);
    float* EA = (float*)(buf + L::oEA);

    stage_gates<P, VAR, DK, DVW, HG>(st, ldr, buf, blk, next_tok0, lane);
    // per-token decay factors of the owned key dimensions
    float al[EPL][kBlock];
#pragma unroll
    for (int i = 0; i < kBlock; ++i) {
        al[0][i] = fast_exp2(P::lo(st.ld[i]) * kLog2e);
        if constexpr (EPL == 2) al[1][i] = fast_exp2(P::hi(st.ld[i]) * kLog2e);
        ldr.load_ld(st, i);
    }
    // forward: p_t = prod_{i<=t} alpha_i ; qa_t = q_t p_t
    float pre[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) pre[e] = 1.f;
    elem* qrow = QA + (kBlock * blk) * L::RS + perm32(EPL * lane);
    elem* krow = KD + (kBlock * blk) * L::RS + perm32(EPL * lane);
#pragma unroll
    for (int i = 0; i < kBlock; ++i) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) pre[e] *= al[e][i];
        if constexpr (!SO) {
            if constexpr (EPL == 2)
                *(pair*)(qrow + i * L::RS) = P::make(P::lo(st.q[i]) * pre[0], P::hi(st.q[i]) * pre[1]);
            else if (owner)
                P::store1(qrow + i * L::RS, P::lo(st.q[i]) * pre[0]);
            ldr.load_q(st, i);
        }
    }
    float invA[EPL];
    bool in_range = true;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        invA[e] = fast_rcp(pre[e]);
        if (owner) EA[blk * DK + EPL * lane + e] = pre[e];
        if constexpr (SO) dacc[e] *= pre[e];
        in_range = in_range && (pre[e] >= kMinBlockDecay || !owner);
    }
    // A block decay below e^-80 means a log-decay under -5 somewhere in the block (or a NaN): the quotients
    // below may then leave the fp32 range.  The call goes on; the status word tells the caller.
    if (!in_range) atomicOr(status, (unsigned int)SLA_DEVICE_DECAY_RANGE);
    // backward: kb_j = k_j prod_{i>j} alpha_i ; kd_j = kb_j / A
    float suf[EPL], kb[EPL][kBlock];
#pragma unroll
    for (int e = 0; e < EPL; ++e) suf[e] = 1.f;
#pragma unroll
    for (int i = kBlock - 1; i >= 0; --i) {
        kb[0][i] = P::lo(st.k[i]) * suf[0];
        if constexpr (EPL == 2) kb[1][i] = P::hi(st.k[i]) * suf[1];
        ldr.load_k(st, i);
        if constexpr (!SO) {
            if constexpr (EPL == 2)
                *(pair*)(krow + i * L::RS) = P::make(kb[0][i] * invA[0], kb[1][i] * invA[1]);
            else if (owner)
                P::store1(krow + i * L::RS, kb[0][i] * invA[0]);
        }
#pragma unroll
        for (int e = 0; e < EPL; ++e) suf[e] *= al[e][i];
    }
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        elem* dst = KBT + kbt_row(EPL * lane + e) * L::KTS + kbt_col(EPL * lane + e);
#pragma unroll
        for (int tg = 0; tg < 4; ++tg) {
            const float four[4] = {kb[e][4 * tg], kb[e][4 * tg + 1], kb[e][4 * tg + 2], kb[e][4 * tg + 3]};
            if (owner) store_run<P, 4>(dst + 8 * tg, four);
        }
    }
    // Scores of the block, P^T[j][t] = kd_j . qa_t for j <= t (else 0), from this wave's own rows
    // (its LDS operations execute in order, so the rows written above are visible to it), stored as the
    // MFMA operand every consumer wave reads: lane (r, g) keeps column t = r, rows j = 4g..4g+3.
    if constexpr (!SO) {
        typedef typename P::frag frag;
        constexpr int NTILE = DK / 16;
        const int r_ = lane & 15, g_ = lane >> 4;
        __builtin_amdgcn_wave_barrier();
        f32x4 pT = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < NTILE; s += 2) {
            const frag q0 = *(const frag*)(QA + (kBlock * blk + r_) * L::RS + 16 * s + 8 * g_);
            const frag q1 = *(const frag*)(QA + (kBlock * blk + r_) * L::RS + 16 * s + 8 * g_ + 4);
            const frag k0 = *(const frag*)(KD + (kBlock * blk + r_) * L::RS + 16 * s + 8 * g_);
            const frag k1 = *(const frag*)(KD + (kBlock * blk + r_) * L::RS + 16 * s + 8 * g_ + 4);
            P::mma32(pT, k0, k1, q0, q1);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) pT[i] = (4 * g_ + i <= r_) ? pT[i] : 0.f;
        ((frag*)(buf + L::oPT))[blk * 64 + lane] = P::from_acc(pT);
    }
    stage_values<P, VAR, DK, DVW, HG>(st, ldr, buf, blk, next_tok0, lane);
}

// ---------------------------------------------------------------------------------------------
// Consumer: the four 16-token blocks of one staged chunk for the 16 value columns of wave cw.
// The LDS fragments of block I+1 (and the state-step fragments of block I) are requested before the
// matrix work of block I starts, so their latency is covered by it.
// ---------------------------------------------------------------------------------------------
template <class P, int VAR, int DK>
struct BlockFrags {
    typedef typename P::frag frag;
    frag fq[DK / 16];                          // q rows of the block (GLA: decay-folded), all key dimensions
    frag fk[DK / 16];                          // k^T of the block (GLA: decayed to the block's end) for the state step
    frag fkd[VAR == SLA_GDN ? DK / 16 : 1];    // delta rule: k rows
    frag fp;                                   // masked, decayed scores P^T
    frag fv;                                   // v' of this wave's columns
    float gq;                                  // read gate of token r
    float ea0, ea1;                            // GLA: block decay of the state rows this lane hands out by DPP
    // scalar-decay variants: 2^c_t of token r, log2 of the block's decay, 2^(c_16 - c_j) for j = 4g..4g+3
    float e1, c16;
    f32x4 eb;
    f32x4 ej;                                  // delta rule: beta_j 2^c_j (j = 4g..4g+3)
    frag tm;                                   // delta rule: Tm[r][4g..4g+3], staged as an MFMA operand
};

// Requests the LDS operands of one block.  PART 0: all of them.  The delta rule asks in two parts: 1 = what
// its dependent chain starts with (k rows, v', decays, beta, Tm), 2 = the rest (q rows, k^T, scores, gate).
template <class P, int VAR, int DK, int DVW, bool SO, int PART = 0>
__device__ __forceinline__ void load_block_frags(BlockFrags<P, VAR, DK>& f, const unsigned char* buf, int cw, int lane) {
    typedef typename P::elem elem;
    typedef typename P::frag frag;
    typedef Smem<P, VAR, DK, DVW> L;
    constexpr int NTILE = DK / 16;
    constexpr bool EARLY = PART != 2, LATE = PART != 1;
    const int r = lane & 15, g = lane >> 4;
    const elem* QA = (const elem*)(buf + L::oQA);
    if constexpr (!SO && LATE) {
#pragma unroll
        for (int s = 0; s < NTILE; ++s) f.fq[s] = *(const frag*)(QA + r * L::RS + 32 * (s / 2) + 8 * g + 4 * (s & 1));
        f.fp = ((const frag*)(buf + L::oPT))[lane];
        f.gq = ((const float*)(buf + L::oGQ))[r];
    }
    if constexpr (VAR != SLA_GLA && EARLY) {
        f.e1 = ((const float*)(buf + L::oE1))[r];
        f.c16 = ((const float*)(buf + L::oP1))[kBlock - 1];
        f.eb = *(const f32x4*)((const float*)(buf + L::oEB) + 4 * g);
    }
    if constexpr (VAR == SLA_GDN && EARLY) {
        const elem* KD = (const elem*)(buf + L::oKD);
#pragma unroll
        for (int s = 0; s < NTILE; ++s) f.fkd[s] = *(const frag*)(KD + r * L::RS + 32 * (s / 2) + 8 * g + 4 * (s & 1));
        f.ej = *(const f32x4*)((const float*)(buf + L::oEJ) + 4 * g);
        f.tm = *(const frag*)((const elem*)(buf + L::oTM) + r * kBlock + 4 * g);
    }
    if constexpr (EARLY) f.fv = *(const frag*)((const elem*)(buf + L::oVT) + (16 * cw + r) * L::TS + 4 * g);
    if constexpr (LATE && L::kTR) {
        // k^T of tile s (rows d = 16 s + r, slots tokens 4g .. 4g + 3) from the k rows: lane l of a group of 16
        // addresses four stored elements of token 4g + l / 4 -- dimensions 16 s + 4 (l % 4) .. + 3, which the rows'
        // permutation keeps adjacent -- and receives dimension 16 s + l of the group's four tokens.
        typedef __attribute__((address_space(3))) frag lds_frag;
        const elem* kp = (const elem*)(buf + L::oKD) + (4 * g + (r >> 2)) * L::RS + 8 * (r & 3);
#pragma unroll
        for (int s = 0; s < NTILE; ++s)
            f.fk[s] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_frag*)(kp + 32 * (s / 2) + 4 * (s & 1)));
    } else if constexpr (LATE) {
        const elem* KBT = (const elem*)(buf + L::oKBT);
#pragma unroll
        for (int s = 0; s < NTILE; ++s)
            f.fk[s] = *(const frag*)(KBT + (16 * (s / 2) + r) * L::KTS + 8 * g + 4 * (s & 1));
    }
    // GLA: the block's decay per state row.  Lane group g needs A[16s + 4g + i] for every tile s; lane r
    // of the group fetches two of them (s = r/4 and s = 4 + r/4, i = r%4) and the multiply takes its
    // factor from the lane that holds it through a DPP row broadcast.
    if constexpr (VAR == SLA_GLA && LATE) {
        const float* EA = (const float*)(buf + L::oEA);
        f.ea0 = EA[16 * (r >> 2) + 4 * g + (r & 3)];
        if constexpr (NTILE > 4) f.ea1 = EA[64 + 16 * (r >> 2) + 4 * g + (r & 3)];
    }
}

// ---------------------------------------------------------------------------------------------
// Producer/consumer hand-over through two counters per LDS slot.  ready[s] counts the blocks a
// producer has finished writing into slot s, done[s] the consumer waves that have finished reading
// it; both only grow, so a waiter compares against the value its own block index implies.  The LDS
// operations of a wave complete in order: once lgkmcnt has drained, everything the wave wrote is in
// LDS and everything it read is in its registers, and the counter update that follows is ordered
// behind them.  Every wait is bounded: the hand-over cannot deadlock (a block depends only on blocks
// with smaller indices); should a wait ever exhaust its budget the wave records SLA_DEVICE_WAIT_EXPIRED in
// the device status word and goes on rather than hang (the call's results are then invalid, and
// sla_device_status tells the caller so).
// ---------------------------------------------------------------------------------------------
static constexpr int kSpinLimit = 1 << 22;
typedef __attribute__((address_space(3))) int lds_int;  // the counters are addressed as LDS, never as flat memory

__device__ __forceinline__ int flag_peek(const lds_int* f) { return *(const volatile lds_int*)f; }

__device__ __forceinline__ void flag_wait(const lds_int* f, int target, unsigned int* status) {
    int spin = 0;
#pragma nounroll
    while (flag_peek(f) < target && ++spin < kSpinLimit) __builtin_amdgcn_s_sleep(1);
    if (spin >= kSpinLimit && (threadIdx.x & 63) == 0) atomicOr(status, (unsigned int)SLA_DEVICE_WAIT_EXPIRED);
    asm volatile("" ::: "memory");
}

// Called with all 64 lanes active; lane 0 alone performs the add.  flag_signal_now skips the drain: for
// a caller whose LDS accesses are known to have completed.
__device__ __forceinline__ void flag_signal_now(lds_int* f) {
    const uint32_t addr = (uint32_t)(uintptr_t)f;
    const int one = 1;
    asm volatile(
        "s_mov_b64 exec, 1\n"
        "ds_add_u32 %0, %1\n"
        "s_mov_b64 exec, -1"
        :
        : "v"(addr), "v"(one)
        : "memory");
}

__device__ __forceinline__ void flag_signal(lds_int* f, int) {
    const uint32_t addr = (uint32_t)(uintptr_t)f;
    const int one = 1;
    asm volatile(
        "s_waitcnt lgkmcnt(0)\n"
        "s_mov_b64 exec, 1\n"
        "ds_add_u32 %0, %1\n"
        "s_mov_b64 exec, -1"
        :
        : "v"(addr), "v"(one)
        : "memory");
}

// One 16-token block, entirely from registers: read-out with the entry state, state step, epilogue
// store.  cur holds every LDS operand of the block (requested a block earlier), so nothing in here
// waits for LDS and the whole block is one scheduling region.
template <class P, int VAR, int DK, int DVW, bool SO>
__device__ __forceinline__ void consume_block(f32x4 (&S)[DK / 16], const BlockFrags<P, VAR, DK>& cur,
                                              typename P::elem* out_tile, int r, int unit) {
    typedef typename P::frag frag;
    constexpr int NTILE = DK / 16;

    frag fv = cur.fv;    // v' for the read-out
    frag fv2 = cur.fv;   // v' for the state step (scalar-decay variants: times 2^(c_16 - c_j))
    [[maybe_unused]] float A = 1.f;
    if constexpr (VAR != SLA_GLA) {
        A = fast_exp2(cur.c16);
        f32x4 vs = P::to_acc(cur.fv);
        if constexpr (VAR == SLA_GDN) {
            // Delta rule (Sec. 5.1, Softmax-GatedDeltaNet), all 16 tokens of the block at once:
            //   (I + L) U = beta G^K V - diag(beta p) K S   =>   U = Tm R,
            // and U takes the place of v' in the read-out and in the state step.
            // X[j][n] = k_j S : lane holds column n = r, rows j = 4g + i; two accumulation chains
            f32x4 X = {0.f, 0.f, 0.f, 0.f}, X2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < NTILE; s += 4) {
                P::mma32(X, cur.fkd[s], cur.fkd[s + 1], P::from_acc(S[s]), P::from_acc(S[s + 1]));
                if (s + 2 < NTILE)
                    P::mma32(X2, cur.fkd[s + 2], cur.fkd[s + 3], P::from_acc(S[s + 2]), P::from_acc(S[s + 3]));
            }
            f32x4 R;
#pragma unroll
            for (int i = 0; i < 4; ++i) R[i] = vs[i] - cur.ej[i] * (X[i] + X2[i]);
            f32x4 U = {0.f, 0.f, 0.f, 0.f};
            P::mma16_only(U, cur.tm, P::from_acc(R));  // U[t][n] = sum_j Tm[t][j] R[j][n]
            vs = U;
            fv = P::from_acc(U);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) vs[i] *= cur.eb[i];
        fv2 = P::from_acc(vs);
    }

    // O^T[n][t] = p_t sum_d S[d][n] q[t][d] + sum_j v'[j][n] P[t][j]   (GLA: p_t is folded into q)
    // as two independent accumulation chains, added in the epilogue
    f32x4 oS = {0.f, 0.f, 0.f, 0.f}, oP = {0.f, 0.f, 0.f, 0.f};
    if constexpr (!SO) {
        P::mma16_only(oP, fv, cur.fp);
#pragma unroll
        for (int s = 0; s < NTILE; s += 2)
            P::mma32(oS, P::from_acc(S[s]), P::from_acc(S[s + 1]), cur.fq[s], cur.fq[s + 1]);
    }

    // state step: S <- diag(A) S + kb^T v'
    if constexpr (VAR == SLA_GLA) scale_state_rows<NTILE>(S, cur.ea0, cur.ea1);
#pragma unroll
    for (int s = 0; s < NTILE; ++s) {
        if constexpr (VAR != SLA_GLA) {
#pragma unroll
            for (int i = 0; i < 4; ++i) S[s][i] *= A;
        }
        P::mma16_only(S[s], cur.fk[s], fv2);
    }

    // epilogue: read gate, cast, park 4 adjacent value columns of token t in the slot's output tile
    if constexpr (!SO) {
        float o[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = (VAR != SLA_GLA ? oS[i] * cur.e1 + oP[i] : oS[i] + oP[i]) * cur.gq;
        park_out4<P, DVW>(out_tile, r, unit, o);
    }
}

// ---------------------------------------------------------------------------------------------
// The kernel: waves 0..3 consume (wave w owns value columns 16w..16w+15 of the slice and the state
// rows x those columns), the other waves produce: producer p stages blocks p, p + NP, p + 2 NP, ...
// into slot p of an LDS ring, up to NP blocks ahead of the consumers.  There is no workgroup barrier
// after start-up: a consumer waits for the block it needs, a producer for its slot to be free.
// ---------------------------------------------------------------------------------------------
template <class P, int VAR, int DK, int DVW, int HG, bool SO>
__global__ __launch_bounds__((Smem<P, VAR, DK, DVW>::threads)) void sla_fwd_kernel(const KArgs a) {
    typedef typename P::elem elem;
    typedef Smem<P, VAR, DK, DVW> L;
    constexpr int NTILE = DK / 16;
    constexpr int NCW = DVW / 16;  // consumer waves that have columns
    constexpr int NP = L::slots;   // producer waves = ring slots
    static_assert(DK == 32 || DK == 64 || DK == 128, "dk");
    static_assert(DVW == 16 || DVW == 32 || DVW == 64, "value columns per workgroup");
    static_assert((NP & (NP - 1)) == 0, "slot index is taken with a mask");

    extern __shared__ __align__(16) unsigned char smem[];
    lds_int* ready = (lds_int*)(smem + L::oFlags);
    lds_int* done = ready + kMaxSlots;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool producer = wave >= kWaves;
    const int pw = wave - kWaves;  // producer index = slot
    const int r = lane & 15, g = lane >> 4;

    if (tid < 2 * kMaxSlots) ready[tid] = 0;
    __syncthreads();

    // Workgroup -> (batch row, head, value slice).  Consecutive hardware ids go to different XCDs (id % 8),
    // each with its own L2; the grid is padded to a multiple of 8 * nslice and ids past the last pair have
    // nothing to do.  The slices of one (row, head) read the same q, k, decay and logits, so they always share
    // an XCD.  Rectangular batches give every XCD a contiguous range of (row, head) pairs (the heads of a token
    // also share its logits).  Packed batches deal the pairs round-robin over the XCDs instead: the heads of one
    // long sequence would otherwise pile onto a single XCD's share of the memory bandwidth while the others idle.
    const int xcd = blockIdx.x & 7, place = blockIdx.x >> 3;
    int slice, rowh;
    if (a.cu) {
        slice = place % a.nslice;
        rowh = (place / a.nslice) * 8 + xcd;
    } else {
        const int logical = xcd * (gridDim.x >> 3) + place;
        slice = logical % a.nslice;
        rowh = logical / a.nslice;
    }
    if (rowh >= a.B * a.nseg_grid * a.H) return;
    const int row = rowh / a.H, h = rowh % a.H;          // row = (batch, segment)
    const int b = row / a.nseg_grid, seg = row % a.nseg_grid;
    const int n0 = slice * DVW;
    const int H = a.H, dv = a.dv;
    int T = min(a.Ls, a.T - seg * a.Ls);                  // tokens of this row
    size_t row_tok = (size_t)b * a.T + (size_t)seg * a.Ls;
    if (a.cu) {  // packed sequences (one segment each); offsets are clamped into the tensors whatever cu holds
        const int start = min(max(a.cu[b], 0), a.T), end = min(max(a.cu[b + 1], start), a.T);
        T = end - start;
        row_tok = (size_t)start;
    }
    const int nblocks = (T + kBlock - 1) / kBlock;

    if (producer) {
        float decay_const = 0.f;  // RetNet: log2 gamma_h
        if constexpr (VAR == SLA_RETNET) decay_const = ((const float*)a.ld)[h] * kLog2e;
        Loader<P, VAR, DK, DVW, HG> ldr;
        ldr.init(a, row_tok, T, h, n0, lane);
        // One register stage, refilled while it is consumed: the loads of a block are in flight while
        // the other producers' blocks are staged.  Past the end of the sequence every load is out of
        // range: it returns zero without touching memory, and nothing staged from it is ever read.
        Stage<P, VAR, DK, DVW, HG> st;
        ldr.advance(kBlock * pw);
        ldr.load(st, lane);
        float dacc[kEPL<DK>];  // pre-pass, GLA: decay of the blocks this wave staged, per owned key dimension
#pragma unroll
        for (int e = 0; e < kEPL<DK>; ++e) dacc[e] = 1.f;
        unsigned char* buf = smem + (size_t)pw * L::bytes;
        // The slot's output tile goes to global memory from here: column n0 of the row's first token.
        const size_t out_tstride = a.head_major ? (size_t)dv : (size_t)H * dv;
        const size_t out_tok = a.head_major ? ((row_tok / a.T) * H + h) * a.T + row_tok % a.T : row_tok * H + h;
        [[maybe_unused]] elem* out_row = (elem*)a.out + out_tok * dv + n0;
        [[maybe_unused]] const elem* tile = (const elem*)(buf + L::oOUT);
        int use = 0;
        for (int I = pw; I < nblocks; I += NP, ++use) {
            flag_wait(done + pw, NCW * use, a.status);  // the consumers have finished the block that was here ...
            if constexpr (!SO) {                // ... and left its output in the slot: store it
                if (use > 0)
                    store_out_tile<P, DVW>(tile, out_row + (size_t)(kBlock * (I - NP)) * out_tstride, out_tstride,
                                           T - kBlock * (I - NP), lane);
            }
            ldr.advance(kBlock * NP);          // every staging register is refilled for block I + NP
            produce_block<P, VAR, DK, DVW, HG, SO>(st, ldr, buf, 0, kBlock * I, kBlock * (I + NP), T, decay_const, dacc,
                                                   lane, a.status);
            flag_signal(ready + pw, lane);
        }
        if constexpr (!SO) {  // the output of this wave's last block
            if (use > 0) {
                const int I = pw + NP * (use - 1);
                flag_wait(done + pw, NCW * use, a.status);
                store_out_tile<P, DVW>(tile, out_row + (size_t)(kBlock * I) * out_tstride, out_tstride, T - kBlock * I, lane);
            }
        }
        if constexpr (SO && VAR == SLA_GLA) {
            float* dp = a.ws_decay + (((size_t)(b * (a.nseg - 1) + seg) * H + h) * kMaxSlots + pw) * DK + kEPL<DK> * lane;
            if (lane < kOwners<DK>) {
#pragma unroll
                for (int e = 0; e < kEPL<DK>; ++e) dp[e] = dacc[e];
            }
        }
        return;
    }

    // ---------------------------------------------------------------- consumer waves
    const int cw = wave;
    if (cw >= NCW) return;
    __builtin_amdgcn_s_setprio(2);  // the state recurrence is the serial part: let it issue first
    // State slice: tile s holds S[16s + 4g + i][n0 + 16*cw + r] in S[s][i].
    f32x4 S[NTILE];
#pragma unroll
    for (int s = 0; s < NTILE; ++s) S[s] = f32x4{0.f, 0.f, 0.f, 0.f};
    // Entry state: the caller's (or zero) in a single pass; with segments, slot seg of the workspace, which
    // the combine kernel has filled (slot 0 with the caller's state, so that final_state may alias it).
    // The pre-pass starts from zero and leaves the end state of segment seg in slot seg + 1.
    const size_t lane_off = (size_t)(4 * g) * dv + n0 + 16 * cw + r;
    const size_t head_sz = (size_t)DK * dv;
    const float* s_in = nullptr;
    float* s_out = nullptr;
    if constexpr (SO) {
        s_out = a.ws_state + ((size_t)(b * a.nseg + seg + 1) * H + h) * head_sz + lane_off;
    } else {
        if (a.nseg > 1)
            s_in = a.ws_state + ((size_t)(b * a.nseg + seg) * H + h) * head_sz + lane_off;
        else if (a.s0)
            s_in = a.s0 + ((size_t)b * H + h) * head_sz + lane_off;
        if (seg == a.nseg - 1 && a.sT) s_out = a.sT + ((size_t)b * H + h) * head_sz + lane_off;
    }
    if (s_in) {
#pragma unroll
        for (int s = 0; s < NTILE; ++s)
#pragma unroll
            for (int i = 0; i < 4; ++i) S[s][i] = s_in[(size_t)(16 * s + i) * dv];
    }
    // this lane parks 4 adjacent value columns (unit 4 cw + g of the slice) of token r of every block
    const int unit = 4 * cw + g;
    auto out_tile = [&](int slot) { return (elem*)(smem + (size_t)slot * L::bytes + L::oOUT); };
    int seen = 0;
    if constexpr (L::prefetch) {
        BlockFrags<P, VAR, DK> fa, fb;
        // Block I.  On entry every LDS operand of the block has been requested (a block ago, into cur) and
        // so has the counter of block I + 1.  Once they have landed -- and with them the output of block
        // I - 1 has reached its slot's tile -- slot (I - 1) % NP is handed back to its producer; block I is
        // computed from registers, and, block I + 1 being staged, its operands are requested into nxt
        // together with the counter of block I + 2.  Past the last block the requests read slots that
        // hold older data; nothing uses it.
        auto step = [&](int I, BlockFrags<P, VAR, DK>& cur, BlockFrags<P, VAR, DK>& nxt) {
            const int sl = I & (NP - 1), sl1 = (I + 1) & (NP - 1), sl2 = (I + 2) & (NP - 1);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            if (I > 0) flag_signal_now(done + ((I - 1) & (NP - 1)));
            if (I + 1 < nblocks && seen < (I + 1) / NP + 1) flag_wait(ready + sl1, (I + 1) / NP + 1, a.status);
            asm volatile("" ::: "memory");
            load_block_frags<P, VAR, DK, DVW, SO>(nxt, smem + (size_t)sl1 * L::bytes, cw, lane);
            seen = flag_peek(ready + sl2);
            consume_block<P, VAR, DK, DVW, SO>(S, cur, out_tile(sl), r, unit);
        };
        if (nblocks > 0) flag_wait(ready, 1, a.status);
        load_block_frags<P, VAR, DK, DVW, SO>(fa, smem, cw, lane);
        seen = flag_peek(ready + (1 & (NP - 1)));
        for (int I = 0; I < nblocks; I += 2) {
            step(I, fa, fb);
            if (I + 1 < nblocks) step(I + 1, fb, fa);
        }
        if (nblocks > 0) {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            flag_signal_now(done + ((nblocks - 1) & (NP - 1)));
        }
    } else {
        // Delta rule: two full sets of operand registers would cost the registers that eight producer waves
        // need.  Only what the block's long dependent chain starts with (k S, the triangular solve's
        // product) is requested a block ahead; the rest (q rows, k^T, scores, gate) at the top of the
        // block itself, where that chain covers its latency.  The slot goes back at the end of the block.
        BlockFrags<P, VAR, DK> fa, fb;
        auto step = [&](int I, BlockFrags<P, VAR, DK>& cur, BlockFrags<P, VAR, DK>& nxt) {
            const int sl = I & (NP - 1), sl1 = (I + 1) & (NP - 1), sl2 = (I + 2) & (NP - 1);
            if (I + 1 < nblocks && seen < (I + 1) / NP + 1) flag_wait(ready + sl1, (I + 1) / NP + 1, a.status);
            asm volatile("" ::: "memory");
            load_block_frags<P, VAR, DK, DVW, SO, 2>(cur, smem + (size_t)sl * L::bytes, cw, lane);
            load_block_frags<P, VAR, DK, DVW, SO, 1>(nxt, smem + (size_t)sl1 * L::bytes, cw, lane);
            seen = flag_peek(ready + sl2);
            consume_block<P, VAR, DK, DVW, SO>(S, cur, out_tile(sl), r, unit);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            flag_signal_now(done + sl);
        };
        if (nblocks > 0) flag_wait(ready, 1, a.status);
        load_block_frags<P, VAR, DK, DVW, SO, 1>(fa, smem, cw, lane);
        seen = flag_peek(ready + (1 & (NP - 1)));
        for (int I = 0; I < nblocks; I += 2) {
            step(I, fa, fb);
            if (I + 1 < nblocks) step(I + 1, fb, fa);
        }
    }

    if (s_out) {
#pragma unroll
        for (int s = 0; s < NTILE; ++s)
#pragma unroll
            for (int i = 0; i < 4; ++i) s_out[(size_t)(16 * s + i) * dv] = S[s][i];
    }
}

// ---------------------------------------------------------------------------------------------
// Launch
// ---------------------------------------------------------------------------------------------
template <class P, int VAR, int DK, int DVW, int HG, bool SO>
static int launch_one(const KArgs& a, hipStream_t stream) {
    typedef Smem<P, VAR, DK, DVW> L;
    auto kern = sla_fwd_kernel<P, VAR, DK, DVW, HG, SO>;
    const size_t lds = L::total;
    static_assert(L::total <= L::limit, "ring slots exceed the LDS of a CU");
    // The dynamic-LDS limit of a kernel is set once per device and instantiation (bit d = done on device d;
    // two threads racing here both set it, which is harmless).
    static std::atomic<uint64_t> configured{0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();
        return SLA_ERR_HIP;
    }
    if (!((configured.load(std::memory_order_acquire) >> dev) & 1u)) {
        if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
            (void)hipGetLastError();
            return SLA_ERR_HIP;
        }
        configured.fetch_or(uint64_t(1) << dev, std::memory_order_release);
    }
    const int pairs = a.B * a.nseg_grid * a.H;
    const int grid = ((pairs + 7) / 8) * 8 * a.nslice;  // see the workgroup mapping in the kernel
    hipLaunchKernelGGL(kern, dim3(grid), dim3(L::threads), lds, stream, a);
    return hipGetLastError() == hipSuccess ? SLA_OK : SLA_ERR_HIP;
}

// Segment combine (between the pre-pass and the main pass of the segment-parallel schedule):
//   E_0 = initial state,  E_{s+1} = diag(D_s) E_s + L_s,
// with L_s the end state of segment s from a zero entry state (the pre-pass left it in slot s + 1) and
// D_s its total decay.  Slot s ends up holding E_s.  One thread per (batch, head, d, 4 value columns).
template <int VAR>
__global__ void sla_segment_combine_kernel(const KArgs a, int dk) {
    const int dv4 = a.dv / 4;
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t per_head = (size_t)dk * dv4;
    if (idx >= (size_t)a.B * a.H * per_head) return;
    const int bh = (int)(idx / per_head), b = bh / a.H, h = bh % a.H;
    const int d = (int)((idx % per_head) / dv4), n = (int)(idx % dv4) * 4;
    const size_t head_sz = (size_t)dk * a.dv, off = (size_t)d * a.dv + n;
    f32x4 E = {0.f, 0.f, 0.f, 0.f};
    if (a.s0) E = *(const f32x4*)(a.s0 + (size_t)bh * head_sz + off);
    *(f32x4*)(a.ws_state + ((size_t)(b * a.nseg) * a.H + h) * head_sz + off) = E;
    for (int s = 0; s + 1 < a.nseg; ++s) {
        float D;
        if constexpr (VAR == SLA_GLA) {
            const float* dp = a.ws_decay + ((size_t)(b * (a.nseg - 1) + s) * a.H + h) * kMaxSlots * dk + d;
            D = 1.f;
            for (int w = 0; w < a.nparts; ++w) D *= dp[w * dk];
        } else {
            D = fast_exp2(((const float*)a.ld)[h] * kLog2e * (float)a.Ls);  // segments before the last are full
        }
        if (a.ws_total && n == 0) a.ws_total[((size_t)(b * (a.nseg - 1) + s) * a.H + h) * dk + d] = D;
        f32x4* Lp = (f32x4*)(a.ws_state + ((size_t)(b * a.nseg + s + 1) * a.H + h) * head_sz + off);
        const f32x4 Lseg = *Lp;
#pragma unroll
        for (int i = 0; i < 4; ++i) E[i] = D * E[i] + Lseg[i];
        *Lp = E;
    }
}

// One call = one fused launch, or (segment-parallel schedule, RetNet and GLA) pre-pass + combine + main pass.
template <class P, int VAR, int DK, int DVW, int HG>
static int launch(const KArgs& a, hipStream_t stream) {
    if (a.nseg <= 1) return launch_one<P, VAR, DK, DVW, HG, false>(a, stream);
    if constexpr (VAR == SLA_GDN) {
        return SLA_ERR_UNSUPPORTED;  // the delta rule's segment transition is a dense matrix; not built
    } else {
        KArgs pre = a;
        pre.nseg_grid = a.nseg - 1;
        KArgs mid = a;
        mid.nparts = Smem<P, VAR, DK, DVW>::slots;
        int rc = launch_one<P, VAR, DK, DVW, HG, true>(pre, stream);
        if (rc != SLA_OK) return rc;
        const size_t n = (size_t)a.B * a.H * DK * (a.dv / 4);
        hipLaunchKernelGGL(sla_segment_combine_kernel<VAR>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, mid, DK);
        if (hipGetLastError() != hipSuccess) return SLA_ERR_HIP;
        if (a.states_only) return SLA_OK;
        return launch_one<P, VAR, DK, DVW, HG, false>(a, stream);
    }
}

template <class P, int VAR, int DK, int DVW>
static int dispatch_heads(const KArgs& a, hipStream_t stream) {
    if (a.H <= 16) return launch<P, VAR, DK, DVW, 4>(a, stream);
    if (a.H <= 32) return launch<P, VAR, DK, DVW, 8>(a, stream);
    return launch<P, VAR, DK, DVW, 16>(a, stream);
}

template <class P, int VAR, int DK>
static int dispatch_dvw(const KArgs& a, int dvw, hipStream_t stream) {
    switch (dvw) {
        case 16: return dispatch_heads<P, VAR, DK, 16>(a, stream);
        case 32: return dispatch_heads<P, VAR, DK, 32>(a, stream);
        case 64: return dispatch_heads<P, VAR, DK, 64>(a, stream);
        default: return SLA_ERR_UNSUPPORTED;
    }
}

template <class P, int VAR>
static int dispatch_dk(const KArgs& a, int dk, int dvw, hipStream_t stream) {
    switch (dk) {
        case 32: return dispatch_dvw<P, VAR, 32>(a, dvw, stream);
        case 64: return dispatch_dvw<P, VAR, 64>(a, dvw, stream);
        case 128: return dispatch_dvw<P, VAR, 128>(a, dvw, stream);
        default: return SLA_ERR_UNSUPPORTED;
    }
}

template <class P>
static int dispatch_variant(const KArgs& a, int variant, int dk, int dvw, hipStream_t stream) {
    switch (variant) {
        case SLA_RETNET: return dispatch_dk<P, SLA_RETNET>(a, dk, dvw, stream);
        case SLA_GLA: return dispatch_dk<P, SLA_GLA>(a, dk, dvw, stream);
        case SLA_GDN: return dispatch_dk<P, SLA_GDN>(a, dk, dvw, stream);
        default: return SLA_ERR_UNSUPPORTED;
    }
}

}  // namespace sla
