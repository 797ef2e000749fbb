// SLA backward pass for gfx950 (MI355X): gradients of the chunkwise forward of Sec. 3.2 ("Chunkwise Parallel
// Training") with the head-softmax gates of Eq. 4-6, for the RetNet and GLA recurrences of Sec. 5.1.
//
// With S_t = diag(alpha_t) S_{t-1} + G^K_t k_t^T v_t and out_t = G^Q_t q_t S_t, and dS_t the gradient with respect
// to S_t (dS_t = G^Q_t q_t^T dout_t + diag(alpha_{t+1}) dS_{t+1}):
//     dq_t = G^Q_t dout_t S_t^T      dG^Q_t = q_t . (dout_t S_t^T)
//     dv_t = G^K_t k_t dS_t          dG^K_t = v_t . (k_t dS_t)
//     dk_t = G^K_t dS_t v_t^T
//     dlog_decay_t = sum_{s >= t} (q_s * dq_s - k_s * dk_s)  [+ rowsum(dS_T * S_T) when the final state has a
//                    cotangent]: every pair (writer j < t <= reader s) crosses token t's decay exactly once.
// dq contracts the state over its value columns, dv over its key rows, dk again over the value columns of dS: each
// is a sweep over the tokens that carries one [dk, dv] tile in registers, sliced over the dimension that is NOT
// contracted, exactly like the forward.  So the pass is three sweeps in 16-token blocks,
//     F  (forward in time,  carries S^T,  64 key columns per workgroup)   -> dq, dG^Q, q*dq
//     R1 (backward in time, carries dS,   64 value columns per workgroup) -> dv, dG^K, d initial state
//     R2 (backward in time, carries dS^T, 64 key columns per workgroup)   -> dk, dlog_decay
// between a small kernel that evaluates the gates (Eq. 4) and one that takes dG through the softmax.
//
// Block algebra (tokens 0..15 of a block, c_t the running sum of log-decay inside it, p_t = e^{c_t}, A = p_15,
// qa = q p, kd = k / p, kb = k A / p, all products on bf16 MFMA with fp32 accumulation, decays in fp32):
//   F : P'[t][j] = dout_t . v_j (j <= t);  dq'_t = p_t * (dout_t S0^T + sum_j P'[t][j] G^K_j kd_j);
//       S^T <- S^T A + v^T (G^K kb)
//   R1: Pq[t][j] = qa_t . kd_j (j <= t);   dv'_j = kb_j dS + sum_t Pq[t][j] G^Q_t dout_t;
//       dS <- diag(A) dS + qa^T (G^Q dout)
//   R2: dk'_j = (1/p_j) * sum_t G^Q_t P'[t][j] qa_t + (A/p_j) * (v_j dS^T);   dS^T <- dS^T A + (G^Q dout)^T qa
// Every workgroup has four consumer waves (16 columns of the slice each, their state tile in registers) and eight
// producer waves in four teams of two; team i stages blocks i, i + 4, ... into slot i of a four-slot LDS ring, so
// four blocks are being staged while the consumers work through the ring.  No barrier after start-up: the
// hand-over is two counters per slot.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "sla.h"

namespace sla {

unsigned int* device_status_word();  // sla_api.hip

namespace {

typedef __attribute__((ext_vector_type(4))) float f4;
typedef __attribute__((ext_vector_type(4))) short s4;
typedef __attribute__((ext_vector_type(8))) short s8;
typedef __attribute__((ext_vector_type(8))) __bf16 bf8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf2;
typedef __attribute__((ext_vector_type(4))) uint32_t u4;
typedef __attribute__((ext_vector_type(2))) uint32_t u2;

constexpr int kTok = 16;        // tokens per block
constexpr int kBwdThreads = 768;  // four consumer waves, eight producer waves
constexpr int kCols = 64;       // columns of the sliced dimension per workgroup
constexpr int kTS = 20;         // token stride (elements) of the transposed [column][token] tiles
constexpr int kFS = 68;         // row stride (elements) of the [token][64 columns] tiles
constexpr float kLog2e = 1.4426950408889634f;

struct BArgs {
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    const uint16_t* dout;
    const uint16_t* ld;      // GLA: [B,T,H,dk] bf16
    const float* ld_head;    // RetNet: [H]
    const float* gq;         // gates, [B,T,H]
    const float* gk;
    const float* s0;         // [B,H,dk,dv] or null
    const float* dsf;        // cotangent of the final state or null
    uint16_t* dq;
    uint16_t* dk;
    uint16_t* dv;
    uint16_t* dld;
    float* ds0;
    float* part_q;           // [dk/16][B,T,H] partial dG^Q
    float* part_k;           // [dk/16][B,T,H] partial dG^K
    float* bsum;             // [blocks][H][dk] fp32: per 16-token block, sum of q * (dq - bf16(dq)) (GLA); block id below
    float* corr;             // [B,H,dk] rowsum(dS_T * S_T) (GLA with a final-state cotangent)
    u4* anchor;              // [anchors][H] states (dk x dv, bf16) entering every kAnchor-th block (GLA); layout below
    int B, T, H;
    size_t rows;             // tokens in all: B * T, or the packed total
    const int* cu;           // packed variable-length batch: sequence b is tokens cu[b] .. cu[b+1]-1 of T; else null
    bool head_major;         // q, k, v, d_out, the GLA decay and their gradients are [B,H,T,d] instead of [B,T,H,d]
    int sweeps;              // which of the three sweeps to launch: 1 = dq, 2 = dv, 4 = dk (all: 7)
    bool dv_state_only;      // the dv sweep writes d_initial_state but not dv (pre-pass of the segment schedule)
    int skip_every;          // > 0: the dv sweep skips every sequence whose index is a multiple of it
    unsigned int* status;    // sticky device status word (SLA_DEVICE_*): a bounded wait that expired is recorded here
};

__device__ __forceinline__ float bf_lo(uint32_t p) { return __uint_as_float(p << 16); }
__device__ __forceinline__ float bf_hi(uint32_t p) { return __uint_as_float(p & 0xffff0000u); }
__device__ __forceinline__ float bf_at(const u4& x, int i) { return (i & 1) ? bf_hi(x[i >> 1]) : bf_lo(x[i >> 1]); }
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    bf2 t;
    t.x = (__bf16)lo;
    t.y = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, t);
}
__device__ __forceinline__ s4 pack4(f4 c) {
    u2 t;
    t.x = pack2(c[0], c[1]);
    t.y = pack2(c[2], c[3]);
    return __builtin_bit_cast(s4, t);
}
__device__ __forceinline__ float ex2(float x) { return __builtin_amdgcn_exp2f(x); }

// 16x16x32: lane (r = lane % 16, g = lane / 16) holds row r of A / column r of B, contraction slots 8g..8g+7.
__device__ __forceinline__ void mma32(f4& c, s8 a, s8 b) {
    c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf8, a), __builtin_bit_cast(bf8, b), c, 0, 0, 0);
}
// 16x16x16: slots 4g..4g+3.  Never issued on an accumulator that the 32-slot opcode also writes.
__device__ __forceinline__ void mma16(f4& c, s4 a, s4 b) { c = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, b, c, 0, 0, 0); }
__device__ __forceinline__ s8 join(s4 a, s4 b) { return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7); }

template <int CTRL>
__device__ __forceinline__ float dpp(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}
// inclusive sums over the 16 lanes of a row (tokens): from lane 0 up / from lane 15 down
__device__ __forceinline__ float row_prefix(float x) {
    x += dpp<0x111>(x);
    x += dpp<0x112>(x);
    x += dpp<0x114>(x);
    x += dpp<0x118>(x);
    return x;
}
__device__ __forceinline__ float row_suffix(float x) {
    x += dpp<0x101>(x);
    x += dpp<0x102>(x);
    x += dpp<0x104>(x);
    x += dpp<0x108>(x);
    return x;
}
__device__ __forceinline__ float row_last(float x) { return dpp<0x15F>(x); }   // lane 15 of the row, to all
__device__ __forceinline__ float row_first(float x) { return dpp<0x150>(x); }  // lane 0 of the row, to all

// Row-major [16][KD + 8] operand tile whose contraction index is permuted in groups of 32 so that the eight slots
// a lane feeds to one 16x16x32 MFMA are adjacent: index 32S + 16u + 4g + i sits at 32S + 8g + 4u + i.  The state
// tiles (two 16-row accumulators per 32 slots) then pair up with it without any shuffle.
template <int KD>
__device__ __forceinline__ void put_perm(uint16_t* tile, int t, int e8, u4 x) {
    const int S = e8 >> 2, u = (e8 >> 1) & 1, g0 = (e8 & 1) * 2;
    uint16_t* row = tile + t * (KD + 8) + 32 * S + 4 * u;
    *(u2*)(row + 8 * g0) = u2{x[0], x[1]};
    *(u2*)(row + 8 * (g0 + 1)) = u2{x[2], x[3]};
}
template <int KD>
__device__ __forceinline__ s8 get_perm(const uint16_t* tile, int r, int g, int c) {
    return *(const s8*)(tile + r * (KD + 8) + 32 * c + 8 * g);
}
// [column][kTS] tile: eight columns of one token
__device__ __forceinline__ void put_T(uint16_t* tile, int col0, int t, u4 x) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        tile[(col0 + 2 * i) * kTS + t] = (uint16_t)(x[i] & 0xffffu);
        tile[(col0 + 2 * i + 1) * kTS + t] = (uint16_t)(x[i] >> 16);
    }
}
__device__ __forceinline__ s4 get_T(const uint16_t* tile, int col, int g) { return *(const s4*)(tile + col * kTS + 4 * g); }

// Producer loads are unconditional (tokens past the end read the last token's row) and are zeroed when they are
// staged: a load under a lane mask would have to complete at the join, which defeats loading blocks ahead.
__device__ __forceinline__ u4 load16(const uint16_t* p) { return *(const u4*)p; }
__device__ __forceinline__ u4 keep(u4 x, bool ok) { return u4{ok ? x[0] : 0u, ok ? x[1] : 0u, ok ? x[2] : 0u, ok ? x[3] : 0u}; }

// Workgroups are dealt to the eight XCDs round-robin by blockIdx, and each XCD has its own L2.  The slices of one
// (batch, head) read the same dout / v (or q / k / decay) rows, so they always share an XCD.  Rectangular batches
// give every XCD a contiguous range of (batch, head) pairs; packed batches deal the pairs round-robin over the
// XCDs, so the heads of one long sequence are spread over all of them.  The grid is 8 * slices * ceil(pairs / 8);
// returns pair * slices + slice, or -1 for the padding.
__device__ __forceinline__ int logical_workgroup(int slices, int pairs, bool packed) {
    const int xcd = blockIdx.x & 7, place = blockIdx.x >> 3;
    if (packed) {
        const int pair = (place / slices) * 8 + xcd;
        return pair < pairs ? pair * slices + place % slices : -1;
    }
    const int wg = xcd * (gridDim.x >> 3) + place;
    return wg < pairs * slices ? wg : -1;
}

// Identity of a 16-token block in the q * dq block-sum array: sequences need not start on a multiple of 16, so
// the sequence index is added; ids are unique and at most rows / 16 + B of them exist.
__device__ __forceinline__ size_t block_id(size_t tok0, int t0, int b) { return (tok0 + (size_t)t0) / kTok + (size_t)b; }

// dlog_decay is a running difference of two sums that nearly cancel, so its rounding error would grow with the
// distance from the end of the sequence.  Every kAnchor blocks the dq sweep keeps the state entering the block and
// the dk sweep replaces its running sum by the exact value there, rowsum(dS * S): the error stays that of one span.
// Anchors sit kAnchor * 16 tokens apart inside a sequence and sequences do not overlap, so the token position
// divided by the span numbers them without collisions; there are fewer than rows / span + 1 of them.
constexpr int kAnchor = 32;
__device__ __forceinline__ bool is_anchor(int blk) { return blk > 0 && (blk & (kAnchor - 1)) == 0; }
__device__ __forceinline__ size_t anchor_id(size_t tok0, int t0) { return (tok0 + (size_t)t0) / (kAnchor * kTok); }

// Sum over the four 16-lane rows of a wave, returned in every lane: two register swaps (odd rows against even
// rows, then the upper half against the lower half) instead of a trip through LDS.
__device__ __forceinline__ float reduce_groups(float x) {
    const uint32_t xi = __float_as_uint(x);
    const u2 a = __builtin_amdgcn_permlane16_swap(xi, xi, false, false);
    const uint32_t yi = __float_as_uint(__uint_as_float(a[0]) + __uint_as_float(a[1]));
    const u2 b = __builtin_amdgcn_permlane32_swap(yi, yi, false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// ------------------------------------------------------------------------------------------------------------
// Hand-over between producer and consumer waves: a ring of kSlots LDS slots, one 16-token block each, and two
// counters per slot.  Block I of a sweep lives in slot I % kSlots and is staged by producer team I % kSlots (two
// waves that fill disjoint tiles of the slot).  ready[s] counts member-fills of slot s (two per block), done[s]
// the consumer waves that have finished a block in it (four per block); both only grow, so a waiter compares with
// the value its own block index implies.  The LDS operations of a wave complete in order: once lgkmcnt has
// drained, what the wave wrote is in LDS and what it read is in registers, and the counter update behind the
// drain is ordered after them.  Every wait is bounded: a block depends only on earlier blocks, so the hand-over
// cannot deadlock, and a wait that exhausts its budget lets the wave go on rather than hang.
// ------------------------------------------------------------------------------------------------------------
constexpr int kSlots = 4;
constexpr int kTeamWaves = 2;
constexpr int kConsumers = 4;
// A kept state is private to the two sweeps, which hold it in the same per-lane tiles: 16-byte piece c of the lane
// (tiles 2c and 2c+1 as eight bf16) of wave w of slice s sits at [state][s][w][c][lane], so a store or load
// instruction of a wave covers 1 KiB without gaps.
template <int DK, int DV>
__device__ __forceinline__ size_t anchor_offset(size_t state, int slice, int wave) {
    return ((state * (DK / kCols) + slice) * kConsumers + wave) * (DV / 32) * 64;
}
constexpr int kSpinLimit = 1 << 22;
typedef __attribute__((address_space(3))) int lds_int;

__device__ __forceinline__ void flag_wait(const lds_int* f, int target, unsigned int* status) {
    int spin = 0;
    while (*(const volatile lds_int*)f < target && ++spin < kSpinLimit) __builtin_amdgcn_s_sleep(1);
    if (spin >= kSpinLimit && (threadIdx.x & 63) == 0) atomicOr(status, (unsigned int)SLA_DEVICE_WAIT_EXPIRED);
    asm volatile("" ::: "memory");
}
// All 64 lanes active on entry; drains the wave's LDS traffic, then lane 0 alone adds one.
__device__ __forceinline__ void flag_signal(lds_int* f) {
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

struct Ring {
    lds_int* ready;
    lds_int* done;
    lds_int* out;          // consumer waves that have left the block's output tile(s) in the slot
    unsigned int* status;  // where an expired wait is recorded
};
// The counters sit behind the slots; zeroed by the first twelve threads before anyone uses them.
__device__ __forceinline__ Ring ring_init(unsigned char* smem, int slot_bytes, int tid, unsigned int* status) {
    lds_int* f = (lds_int*)(smem + kSlots * slot_bytes);
    if (tid < 3 * kSlots) f[tid] = 0;
    __syncthreads();
    return Ring{f, f + kSlots, f + 2 * kSlots, status};
}

// One member wave of a producer team: load(block, regs) issues the global loads of a block, stage(block, regs,
// slot) turns them into LDS tiles.  Two register sets: the loads of the team's next two blocks are in flight while
// a block is staged, and every step issues exactly one set of loads (past the end it re-reads the last block), so
// the wait in front of stage() leaves the newer set in flight on every path.
//
// Output tiles (dk sweep; the dq and dv sweeps are not bound by their stores and ran slower with the extra LDS
// traffic): the consumers leave a block's results in the slot ([16 tokens][64 columns] tiles) and raise ring.out; the
// team member given a `flush` writes the tiles of the block that was in the slot to global memory (whole 128-byte
// rows, streaming stores) before it stages the next one, and the last ones after its loop.
struct NoFlush {
    __device__ __forceinline__ void operator()(int, unsigned char*) const {}
};
template <typename Pre, typename Load, typename Stage, typename Flush = NoFlush>
__device__ __forceinline__ void producer_run(const Ring& ring, unsigned char* smem, int slot_bytes, int team, int nb,
                                             Load load, Stage stage, Flush flush = Flush()) {
    if (team >= nb) return;
    constexpr bool kFlush = !__is_same(Flush, NoFlush);
    Pre ra, rb;
    load(team, ra);
    load(min(team + kSlots, nb - 1), rb);
    unsigned char* buf = smem + team * slot_bytes;
    int I = team, use = 0;
    auto drain = [&]() {  // the output of block I - kSlots, once every consumer wave has left it in the slot
        if constexpr (kFlush) {
            if (use > 0) {
                flag_wait(ring.out + team, kConsumers * use, ring.status);
                flush(I - kSlots, buf);
            }
        }
    };
    while (true) {
        flag_wait(ring.done + team, kConsumers * use, ring.status);  // the consumers have left the block that was here
        drain();
        stage(I, ra, buf);
        load(min(I + 2 * kSlots, nb - 1), ra);
        flag_signal(ring.ready + team);
        I += kSlots, ++use;
        if (I >= nb) break;
        flag_wait(ring.done + team, kConsumers * use, ring.status);
        drain();
        stage(I, rb, buf);
        load(min(I + 2 * kSlots, nb - 1), rb);
        flag_signal(ring.ready + team);
        I += kSlots, ++use;
        if (I >= nb) break;
    }
    drain();
}

// A [16 tokens][64 columns] bf16 output tile.  A row is 16 units of four columns; unit c of token t sits at
// position c ^ t of its row, which spreads the consumers' writes (one unit per lane, 16 tokens apart) and the
// flushing wave's reads (a whole row per 16 lanes) over the banks.
constexpr int kTileBytes = kTok * kCols * 2;
__device__ __forceinline__ void tile_put(unsigned char* tile, int t, int unit, u2 v) {
    *(u2*)(tile + ((t * 16 + (unit ^ t)) << 3)) = v;
}
// Tokens t0 .. t0 + 15 of the sequence (those below T), columns col0 .. col0 + 63 of a tensor of width D whose row of
// token tau is wide0 + tau * wstep.  STREAM: non-temporal stores (the tensor is not read again by this call).
template <bool STREAM>
__device__ __forceinline__ void tile_flush(const unsigned char* tile, uint16_t* dst, size_t wide0, size_t wstep, int D,
                                           int col0, int t0, int T, int lane) {
    const int unit = lane & 15;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = (lane >> 4) + 4 * i;
        const u2 v = *(const u2*)(tile + ((t * 16 + (unit ^ t)) << 3));
        if (t0 + t < T) {
            u2* p = (u2*)(dst + (wide0 + (size_t)(t0 + t) * wstep) * D + col0 + 4 * unit);
            if constexpr (STREAM)
                __builtin_nontemporal_store(v, p);
            else
                *p = v;
        }
    }
}

__device__ __forceinline__ void consumer_acquire(const Ring& ring, int I) {
    flag_wait(ring.ready + (I & (kSlots - 1)), kTeamWaves * (I / kSlots + 1), ring.status);
}
__device__ __forceinline__ void consumer_release(const Ring& ring, int I) { flag_signal(ring.done + (I & (kSlots - 1))); }

// Producer loads are unconditional (tokens past the end read the last token's row) and are zeroed when they are
// staged, so no load sits under a lane mask.
template <int N>
struct PreKeys {  // N groups of eight key columns of one token: decay steps, keys, queries, and the gates
    u4 ld[N], kx[N], qx[N];
    float gq, gk;
};
struct PreKeysE : PreKeys<2> {  // ... and, for the dk sweep of GLA, dq of the same 16 columns and the block's q * dq sums
    u4 dq[2];
    f4 bs[4];
};
template <int N>
struct PreRows {  // N 16-byte pieces of dout and of v
    u4 a[N], b[N];
    float gq[N];
};

// Key-side staging, one key column per lane and the 16 tokens of the block in registers: the decay products along
// the tokens are running multiplications (one exponential per element, one reciprocal per column), and the
// transposed [column][token] tiles are plain row writes.  Loads go through buffer descriptors that span the
// sequence, so tokens past its end read as zero (decay factor 1) without any masking.
constexpr uint32_t kRsrcWord3 = 0x00020000u;  // raw buffer descriptor, 32-bit data format
struct PreCol {
    uint32_t ld[kTok], k[kTok], q[kTok];  // 16-bit values as loaded, in the low halves
    float gq, gk;                         // lane i < 16: the gates of token i of the block
};
struct ColLoader {
    __amdgpu_buffer_rsrc_t rq, rk, rld;
    const float* gq;  // gates of this head, token 0 of the sequence; H floats between tokens
    const float* gk;
    int tstride;      // bytes between tokens of q, k and the decay
    int voff;         // byte offset of this lane's column in token 0
    int T, H, lane;
    // tokens t0 .. t0 + 15 of the sequence
    template <int VAR>
    __device__ __forceinline__ void load(int t0, PreCol& p) const {
        const int base = voff + t0 * tstride;
#pragma unroll
        for (int i = 0; i < kTok; ++i) {
            if constexpr (VAR == SLA_GLA)
                p.ld[i] = (uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rld, base, i * tstride, 0);
            p.k[i] = (uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rk, base, i * tstride, 0);
            p.q[i] = (uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rq, base, i * tstride, 0);
        }
        const size_t tok = (size_t)min(t0 + (lane & 15), T - 1);  // clamped; masked when staged
        p.gq = gq[tok * H];
        p.gk = gk[tok * H];
    }
};
template <int DK>
__device__ __forceinline__ ColLoader make_col_loader(const BArgs& a, size_t tok0, int T, int h, int col, int lane) {
    ColLoader c;
    const int tstride = (a.head_major ? 1 : a.H) * DK * 2;
    const size_t base = a.head_major ? ((tok0 / a.T) * a.H + h) * (size_t)a.T * DK : tok0 * a.H * DK;
    c.rq = __builtin_amdgcn_make_buffer_rsrc((void*)(a.q + base), 0, T * tstride, kRsrcWord3);
    c.rk = __builtin_amdgcn_make_buffer_rsrc((void*)(a.k + base), 0, T * tstride, kRsrcWord3);
    c.rld = __builtin_amdgcn_make_buffer_rsrc((void*)((a.ld ? a.ld : a.q) + base), 0, a.ld ? T * tstride : 0, kRsrcWord3);
    c.gq = a.gq + tok0 * a.H + h;
    c.gk = a.gk + tok0 * a.H + h;
    c.tstride = tstride;
    c.voff = ((a.head_major ? 0 : h * DK) + col) * 2;
    c.T = T;
    c.lane = lane;
    c.H = a.H;
    return c;
}
__device__ __forceinline__ float bf16_low(uint32_t x) { return __uint_as_float(x << 16); }
__device__ __forceinline__ float lane_value(float x, int i) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), i));
}
// decay factors of the 16 tokens of one column: alpha_i, or 1 past the end of the sequence
template <int VAR>
__device__ __forceinline__ void column_decay(const PreCol& p, float head_alpha, int t0, int T, float* al) {
#pragma unroll
    for (int i = 0; i < kTok; ++i) {
        if constexpr (VAR == SLA_GLA)
            al[i] = ex2(bf16_low(p.ld[i]) * kLog2e);
        else
            al[i] = t0 + i < T ? head_alpha : 1.f;
    }
}
// sixteen values of one column as a row of a [column][kTS] bf16 tile
__device__ __forceinline__ void put_row(uint16_t* row, const float* x) {
#pragma unroll
    for (int m = 0; m < 4; ++m)
        *(u2*)(row + 4 * m) = u2{pack2(x[4 * m], x[4 * m + 1]), pack2(x[4 * m + 2], x[4 * m + 3])};
}

// Inclusive running sums c[i] of the log2-domain decay steps of eight key columns over the 16 tokens of the block
// (token = lane % 16), and their totals.
template <int VAR>
__device__ __forceinline__ void block_decay(const u4& ldx, float head_step, bool ok, float* c, float* tot) {
    if constexpr (VAR == SLA_GLA) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            c[i] = row_prefix(bf_at(ldx, i) * kLog2e);  // zero outside the sequence
            tot[i] = row_last(c[i]);
        }
    } else {  // one decay for all columns: one scan, and the exponentials of the eight columns are common too
        const float c0 = row_prefix(ok ? head_step : 0.f), t0 = row_last(c0);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            c[i] = c0;
            tot[i] = t0;
        }
    }
}

// ------------------------------------------------------------------------------------------------------------
// Sweep F: forward in time, state S^T[n][d] (value rows, 16 key columns per wave).
// ------------------------------------------------------------------------------------------------------------
template <int DV>
struct SmemF {
    static constexpr int oDO = 0;
    static constexpr int oV = oDO + kTok * (DV + 8) * 2;
    static constexpr int oVT = oV + kTok * (DV + 8) * 2;
    static constexpr int oKDT = oVT + DV * kTS * 2;
    static constexpr int oKBT = oKDT + kCols * kTS * 2;
    static constexpr int oPF = oKBT + kCols * kTS * 2;   // p_t per token and key column, fp32
    static constexpr int oTOT = oPF + kTok * kFS * 4;    // A = p_15 per key column
    static constexpr int oQS = oTOT + kCols * 4;
    static constexpr int oGQ = oQS + kTok * kFS * 2;
    static constexpr int bytes = oGQ + kTok * 4;
    static constexpr int total = kSlots * bytes + 3 * kSlots * 4;
    static_assert(oV % 16 == 0 && oVT % 16 == 0 && oKDT % 16 == 0 && oPF % 16 == 0 && oTOT % 16 == 0 &&
                      oQS % 16 == 0 && oGQ % 16 == 0 && bytes % 16 == 0,
                  "tiles stay 16-byte aligned");
    static_assert(total <= 160 * 1024, "the ring fits the LDS of a compute unit");
};

template <int VAR, int DK, int DV>
__global__ __launch_bounds__(kBwdThreads) void sla_bwd_dq_kernel(const BArgs a) {
    typedef SmemF<DV> L;
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int NSL = DK / kCols;
    constexpr int R = DV / 32;  // 16-byte pieces of dout (and of v) per lane of the copy wave
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // in a scalar register: role branches are uniform
    const int r = lane & 15, g = lane >> 4;
    const int wg = logical_workgroup(NSL, a.B * a.H, a.cu != nullptr);
    if (wg < 0) return;
    const int slice = wg % NSL, bh = wg / NSL, b = bh / a.H, h = bh % a.H;
    const int sbase = slice * kCols;
    const int H = a.H;
    int T = a.T;                    // tokens of this sequence and the index of its first token
    size_t tok0 = (size_t)b * a.T;
    if (a.cu) {  // packed sequences; offsets are clamped into the tensors whatever cu holds
        const int start = min(max(a.cu[b], 0), a.T), end = min(max(a.cu[b + 1], start), a.T);
        T = end - start;
        tok0 = (size_t)start;
    }
    // rows of the d-wide tensors: token tau of this sequence and head is row wide0 + tau * wstep
    const size_t wide0 = a.head_major ? (size_t)bh * a.T : tok0 * H + h, wstep = a.head_major ? 1 : H;
    const int nb = (T + kTok - 1) / kTok;
    const Ring ring = ring_init(smem, L::bytes, tid, a.status);

    if (wave >= kConsumers) {
        const int team = (wave - kConsumers) >> 1;
        if (((wave - kConsumers) & 1) == 0) {
            // decay, keys and queries of the slice: key column sbase + lane, the 16 tokens in registers
            const float head_alpha = VAR == SLA_RETNET ? ex2(a.ld_head[h] * kLog2e) : 1.f;
            const ColLoader ldr = make_col_loader<DK>(a, tok0, T, h, sbase + lane, lane);
            producer_run<PreCol>(
                ring, smem, L::bytes, team, nb, [&](int blk, PreCol& p) { ldr.template load<VAR>(blk * kTok, p); },
                [&](int blk, const PreCol& p, unsigned char* buf) {
                    const int t0 = blk * kTok;
                    const bool ok = t0 + (lane & 15) < T;
                    const float gk_own = ok ? p.gk : 0.f;
                    float al[kTok];
                    column_decay<VAR>(p, head_alpha, t0, T, al);
                    float* pf = (float*)(buf + L::oPF) + lane;
                    float pre = 1.f;
#pragma unroll
                    for (int i = 0; i < kTok; ++i) {
                        pre *= al[i];
                        pf[i * kFS] = pre;  // p_t
                    }
                    ((float*)(buf + L::oTOT))[lane] = pre;  // A
                    const float invA = __builtin_amdgcn_rcpf(pre);
                    float suf = 1.f, kd[kTok], kb[kTok];
#pragma unroll
                    for (int i = kTok - 1; i >= 0; --i) {
                        const float x = bf16_low(p.k[i]) * lane_value(gk_own, i) * suf;  // G^K k A / p
                        kb[i] = x;
                        kd[i] = x * invA;                                              // G^K k / p
                        suf *= al[i];
                    }
                    put_row((uint16_t*)(buf + L::oKDT) + lane * kTS, kd);
                    put_row((uint16_t*)(buf + L::oKBT) + lane * kTS, kb);
                    uint16_t* qs = (uint16_t*)(buf + L::oQS) + lane;
#pragma unroll
                    for (int i = 0; i < kTok; ++i) qs[i * kFS] = (uint16_t)p.q[i];
                    if (lane < kTok) ((float*)(buf + L::oGQ))[lane] = ok ? p.gq : 0.f;
                });
        } else {  // dout and v, all value columns
            producer_run<PreRows<R>>(
                ring, smem, L::bytes, team, nb,
                [&](int blk, PreRows<R>& p) {
#pragma unroll
                    for (int rep = 0; rep < R; ++rep) {
                        const int t = r, e8 = g + 4 * rep;  // token = lane % 16: the transposed stores of a wave hit disjoint banks
                        const size_t row = wide0 + (size_t)min(blk * kTok + t, T - 1) * wstep;
                        p.a[rep] = load16(a.dout + row * DV + 8 * e8);
                        p.b[rep] = load16(a.v + row * DV + 8 * e8);
                    }
                },
                [&](int blk, const PreRows<R>& p, unsigned char* buf) {
#pragma unroll
                    for (int rep = 0; rep < R; ++rep) {
                        const int t = r, e8 = g + 4 * rep;  // token = lane % 16: the transposed stores of a wave hit disjoint banks
                        const bool ok = blk * kTok + t < T;
                        const u4 dx = keep(p.a[rep], ok), vx = keep(p.b[rep], ok);
                        put_perm<DV>((uint16_t*)(buf + L::oDO), t, e8, dx);
                        put_perm<DV>((uint16_t*)(buf + L::oV), t, e8, vx);
                        put_T((uint16_t*)(buf + L::oVT), 8 * e8, t, vx);
                    }
                });
        }
        return;
    }

    const int cb = 16 * wave;
    __builtin_amdgcn_s_setprio(2);  // the state recurrence is the serial part: let it issue first
    f4 ST[DV / 16];
#pragma unroll
    for (int i = 0; i < DV / 16; ++i) {
        if (a.s0)
            ST[i] = *(const f4*)(a.s0 + ((size_t)bh * DK + sbase + cb + r) * DV + 16 * i + 4 * g);
        else
            ST[i] = f4{0.f, 0.f, 0.f, 0.f};
    }
    for (int blk = 0; blk < nb; ++blk) {
        consumer_acquire(ring, blk);
        unsigned char* buf = smem + (blk & (kSlots - 1)) * L::bytes;
        const int t0 = blk * kTok;
        const uint16_t* DOp = (const uint16_t*)(buf + L::oDO);
        const uint16_t* Vp = (const uint16_t*)(buf + L::oV);
        // P'^T[j][t] = v_j . dout_t, kept for j <= t
        f4 pT = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < DV / 32; ++c) mma32(pT, get_perm<DV>(Vp, r, g, c), get_perm<DV>(DOp, r, g, c));
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (4 * g + i > r) pT[i] = 0.f;
        const s4 fp = pack4(pT);
        // dqa^T[d][t] = sum_n S^T[n][d] dout_t[n] + sum_j kd'_j[d] P'[t][j]
        f4 oS = {0.f, 0.f, 0.f, 0.f}, oP = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < DV / 32; ++c)
            mma32(oS, join(pack4(ST[2 * c]), pack4(ST[2 * c + 1])), get_perm<DV>(DOp, r, g, c));
        const s4 fkd = get_T((const uint16_t*)(buf + L::oKDT), cb + r, g);
        mma16(oP, fkd, fp);
        const f4 pt = *(const f4*)((const float*)(buf + L::oPF) + r * kFS + cb + 4 * g);
        const u2 qx = *(const u2*)((const uint16_t*)(buf + L::oQS) + r * kFS + cb + 4 * g);
        const float gq = ((const float*)(buf + L::oGQ))[r];
        const float Ad = ((const float*)(buf + L::oTOT))[cb + r];
        const s4 fkb = get_T((const uint16_t*)(buf + L::oKBT), cb + r, g);
        const uint16_t* VT = (const uint16_t*)(buf + L::oVT);
        s4 fvt[DV / 16];
#pragma unroll
        for (int i = 0; i < DV / 16; ++i) fvt[i] = get_T(VT, 16 * i + r, g);
        consumer_release(ring, blk);  // every operand of the block is in registers
        // The state update first: it is what the next block waits for, and the vector work below hides its latency.
        if constexpr (VAR == SLA_GLA) {
            if (is_anchor(blk)) {  // the state entering this block, for the dk sweep: bf16, each lane its own tiles
                u4* st = a.anchor + anchor_offset<DK, DV>(anchor_id(tok0, t0) * H + h, slice, wave) + lane;
#pragma unroll
                for (int c = 0; c < DV / 32; ++c) {
                    const s8 x = join(pack4(ST[2 * c]), pack4(ST[2 * c + 1]));
                    st[64 * c] = *(const u4*)&x;
                }
            }
        }
        // S^T <- S^T A + v^T kb'
#pragma unroll
        for (int i = 0; i < DV / 16; ++i) {
            ST[i] = ST[i] * Ad;
            mma16(ST[i], fvt[i], fkb);
        }
        float dqp[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) dqp[i] = (oS[i] + oP[i]) * pt[i];
        const float qf[4] = {bf_lo(qx[0]), bf_hi(qx[0]), bf_lo(qx[1]), bf_hi(qx[1])};
        float part = qf[0] * dqp[0] + qf[1] * dqp[1] + qf[2] * dqp[2] + qf[3] * dqp[3];
        part = reduce_groups(part);
        const int tok = t0 + r;
        if (tok < T) {
            const size_t row = (tok0 + tok) * H + h, wrow = wide0 + (size_t)tok * wstep;
            if (g == 0) a.part_q[((size_t)(slice * 4 + wave) * a.rows * H) + row] = part;
            float dqv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) dqv[i] = gq * dqp[i];
            *(u2*)(a.dq + wrow * DK + sbase + cb + 4 * g) = u2{pack2(dqv[0], dqv[1]), pack2(dqv[2], dqv[3])};
        }
        if constexpr (VAR == SLA_GLA) {
            // The dk sweep forms q * dq per token from the bf16 dq it reads back, but the running sum behind
            // dlog_decay must advance by the block's exact sum: leave the difference, the block's sum of
            // q * (dq - bf16(dq)) in fp32 (the product of two bf16 values is exact in fp32, so the dk sweep's
            // per-token values add up to exactly the other part).
            f4 bs;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float exact = gq * dqp[i], rounded = i & 1 ? bf_hi(pack2(0.f, exact)) : bf_lo(pack2(exact, 0.f));
                bs[i] = row_suffix(tok < T ? qf[i] * (exact - rounded) : 0.f);
            }
            if (r == 0) *(f4*)(a.bsum + (block_id(tok0, t0, b) * H + h) * DK + sbase + cb + 4 * g) = bs;
        }
    }

    if constexpr (VAR == SLA_GLA) {
        if (a.dsf) {  // rowsum(dS_T * S_T) for the key columns of this wave
            float s = 0.f;
#pragma unroll
            for (int i = 0; i < DV / 16; ++i) {
                const f4 x = *(const f4*)(a.dsf + ((size_t)bh * DK + sbase + cb + r) * DV + 16 * i + 4 * g);
                s += x[0] * ST[i][0] + x[1] * ST[i][1] + x[2] * ST[i][2] + x[3] * ST[i][3];
            }
            s = reduce_groups(s);
            if (g == 0) a.corr[(size_t)bh * DK + sbase + cb + r] = s;
        }
    }
}

// ------------------------------------------------------------------------------------------------------------
// Sweep R2: backward in time, state dS^T[n][d] (value rows, 16 key columns per wave) -> dk, dlog_decay.
// ------------------------------------------------------------------------------------------------------------
template <int DV>
struct SmemK {
    static constexpr int oDO = 0;
    static constexpr int oV = oDO + kTok * (DV + 8) * 2;
    static constexpr int oDYT = oV + kTok * (DV + 8) * 2;
    static constexpr int oQAT = oDYT + DV * kTS * 2;
    static constexpr int oCUM = oQAT + kCols * kTS * 2;   // running log2-decay; its last row is the block total
    static constexpr int oQDQ = oCUM + kTok * kFS * 4;    // q * dq in fp32 (GLA), from the dq sweep
    static constexpr int oKS = oQDQ + kTok * kFS * 4;
    static constexpr int oGQ = oKS + kTok * kFS * 2;
    static constexpr int oGK = oGQ + kTok * 4;
    static constexpr int oTILE = oGK + kTok * 4;  // the block's dk and (GLA) dlog_decay tiles, where they fit
    static constexpr bool tiled = kSlots * (oTILE + 2 * kTileBytes) + 3 * kSlots * 4 <= 160 * 1024;
    static constexpr int bytes = oTILE + (tiled ? 2 * kTileBytes : 0);
    // The block's q * dq sums (64 floats, GLA) live in the four padding columns of the 16 rows of the q * dq tile:
    // the sums of key columns 4 m .. 4 m + 3 are floats 64 .. 67 of row m.
    static constexpr int bs_offset(int d) { return oQDQ + ((d >> 2) * kFS + kCols + (d & 3)) * 4; }
    static constexpr int total = kSlots * bytes + 3 * kSlots * 4;
    static_assert(oV % 16 == 0 && oDYT % 16 == 0 && oQAT % 16 == 0 && oCUM % 16 == 0 && oQDQ % 16 == 0 &&
                      oKS % 16 == 0 && oGQ % 16 == 0 && bytes % 16 == 0,
                  "tiles stay 16-byte aligned");
    static_assert(total <= 160 * 1024, "the ring fits the LDS of a compute unit");
};

template <int VAR, int DK, int DV>
__global__ __launch_bounds__(kBwdThreads) void sla_bwd_dk_kernel(const BArgs a) {
    typedef SmemK<DV> L;
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int NSL = DK / kCols;
    constexpr int R = DV / 32;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, g = lane >> 4;
    const int wg = logical_workgroup(NSL, a.B * a.H, a.cu != nullptr);
    if (wg < 0) return;
    const int slice = wg % NSL, bh = wg / NSL, b = bh / a.H, h = bh % a.H;
    const int sbase = slice * kCols;
    const int H = a.H;
    int T = a.T;                    // tokens of this sequence and the index of its first token
    size_t tok0 = (size_t)b * a.T;
    if (a.cu) {  // packed sequences; offsets are clamped into the tensors whatever cu holds
        const int start = min(max(a.cu[b], 0), a.T), end = min(max(a.cu[b + 1], start), a.T);
        T = end - start;
        tok0 = (size_t)start;
    }
    // rows of the d-wide tensors: token tau of this sequence and head is row wide0 + tau * wstep
    const size_t wide0 = a.head_major ? (size_t)bh * a.T : tok0 * H + h, wstep = a.head_major ? 1 : H;
    const int nb = (T + kTok - 1) / kTok;
    const Ring ring = ring_init(smem, L::bytes, tid, a.status);

    if (wave >= kConsumers) {  // block number I of the sweep covers tokens (nb - 1 - I) * 16 ...
        const int team = (wave - kConsumers) >> 1;
        if (((wave - kConsumers) & 1) == 0) {
            const int t = r, d0 = sbase + 8 * g;  // piece j adds 32 columns: a store instruction's four lane groups sit 8 columns apart, on disjoint banks
            const float head_step = VAR == SLA_RETNET ? a.ld_head[h] * kLog2e : 0.f;
            producer_run<PreKeysE>(
                ring, smem, L::bytes, team, nb,
                [&](int I, PreKeysE& p) {
                    const int tau = min((nb - 1 - I) * kTok + t, T - 1);
                    const size_t row = (tok0 + tau) * H + h, wrow = wide0 + (size_t)tau * wstep;
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        if constexpr (VAR == SLA_GLA) p.ld[j] = load16(a.ld + wrow * DK + d0 + 32 * j);
                        p.kx[j] = load16(a.k + wrow * DK + d0 + 32 * j);
                        p.qx[j] = load16(a.q + wrow * DK + d0 + 32 * j);
                    }
                    if constexpr (VAR == SLA_GLA) {
                        const float* bs = a.bsum + (block_id(tok0, (nb - 1 - I) * kTok, b) * H + h) * DK + d0;
#pragma unroll
                        for (int j = 0; j < 2; ++j) {
                            p.dq[j] = load16(a.dq + wrow * DK + d0 + 32 * j);
                            p.bs[2 * j] = *(const f4*)(bs + 32 * j);  // the same address in all 16 token lanes
                            p.bs[2 * j + 1] = *(const f4*)(bs + 32 * j + 4);
                        }
                    }
                    p.gk = a.gk[row];
                    p.gq = a.gq[row];
                },
                [&](int I, const PreKeysE& p, unsigned char* buf) {
                    const bool ok = (nb - 1 - I) * kTok + t < T;
                    if constexpr (VAR == SLA_GLA) {  // q * dq per token from the bf16 dq; the block's correction to the exact sum
                        float* qd = (float*)(buf + L::oQDQ) + t * kFS + 8 * g;
#pragma unroll
                        for (int j = 0; j < 2; ++j) {
                            const u4 qx = keep(p.qx[j], ok), dx = keep(p.dq[j], ok);
                            *(f4*)(qd + 32 * j) = f4{bf_lo(qx[0]) * bf_lo(dx[0]), bf_hi(qx[0]) * bf_hi(dx[0]),
                                                     bf_lo(qx[1]) * bf_lo(dx[1]), bf_hi(qx[1]) * bf_hi(dx[1])};
                            *(f4*)(qd + 32 * j + 4) = f4{bf_lo(qx[2]) * bf_lo(dx[2]), bf_hi(qx[2]) * bf_hi(dx[2]),
                                                         bf_lo(qx[3]) * bf_lo(dx[3]), bf_hi(qx[3]) * bf_hi(dx[3])};
                            if (t == 0) {
                                *(f4*)(buf + L::bs_offset(8 * g + 32 * j)) = p.bs[2 * j];
                                *(f4*)(buf + L::bs_offset(8 * g + 32 * j + 4)) = p.bs[2 * j + 1];
                            }
                        }
                    }
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        const int c0 = 8 * g + 32 * j;
                        float c[8], tot[8];
                        block_decay<VAR>(keep(p.ld[j], ok), head_step, ok, c, tot);
                        float* cum = (float*)(buf + L::oCUM) + t * kFS + c0;
                        *(f4*)cum = f4{c[0], c[1], c[2], c[3]};
                        *(f4*)(cum + 4) = f4{c[4], c[5], c[6], c[7]};
                        const u4 qx = keep(p.qx[j], ok), kx = keep(p.kx[j], ok);
                        u4 qa;
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            qa[i] = pack2(bf_lo(qx[i]) * ex2(c[2 * i]), bf_hi(qx[i]) * ex2(c[2 * i + 1]));
                        put_T((uint16_t*)(buf + L::oQAT), c0, t, qa);
                        uint16_t* ks = (uint16_t*)(buf + L::oKS) + t * kFS + c0;
                        *(u2*)ks = u2{kx[0], kx[1]};
                        *(u2*)(ks + 4) = u2{kx[2], kx[3]};
                    }
                    if (g == 0) {
                        ((float*)(buf + L::oGQ))[t] = ok ? p.gq : 0.f;
                        ((float*)(buf + L::oGK))[t] = ok ? p.gk : 0.f;
                    }
                });
        } else {  // dout and v; this member also writes the finished dk (and dlog_decay) tiles out
            auto load_rows = [&](int I, PreRows<R>& p) {
#pragma unroll
                for (int rep = 0; rep < R; ++rep) {
                    const int t = r, e8 = g + 4 * rep;  // token = lane % 16: the transposed stores of a wave hit disjoint banks
                    const int tau = min((nb - 1 - I) * kTok + t, T - 1);
                    const size_t row = (tok0 + tau) * H + h, wrow = wide0 + (size_t)tau * wstep;
                    p.a[rep] = load16(a.dout + wrow * DV + 8 * e8);
                    p.b[rep] = load16(a.v + wrow * DV + 8 * e8);
                    p.gq[rep] = a.gq[row];
                }
            };
            auto stage_rows = [&](int I, const PreRows<R>& p, unsigned char* buf) {
#pragma unroll
                for (int rep = 0; rep < R; ++rep) {
                    const int t = r, e8 = g + 4 * rep;  // token = lane % 16: the transposed stores of a wave hit disjoint banks
                    const bool ok = (nb - 1 - I) * kTok + t < T;
                    const u4 dx = keep(p.a[rep], ok), vx = keep(p.b[rep], ok);
                    put_perm<DV>((uint16_t*)(buf + L::oDO), t, e8, dx);
                    put_perm<DV>((uint16_t*)(buf + L::oV), t, e8, vx);
                    u4 dy;
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        dy[j] = pack2(p.gq[rep] * bf_lo(dx[j]), p.gq[rep] * bf_hi(dx[j]));
                    put_T((uint16_t*)(buf + L::oDYT), 8 * e8, t, dy);
                }
            };
            if constexpr (L::tiled) {
                producer_run<PreRows<R>>(ring, smem, L::bytes, team, nb, load_rows, stage_rows,
                                         [&](int I, unsigned char* buf) {
                                             const int t0 = (nb - 1 - I) * kTok;
                                             tile_flush<true>(buf + L::oTILE, a.dk, wide0, wstep, DK, sbase, t0, T, lane);
                                             if constexpr (VAR == SLA_GLA)
                                                 tile_flush<true>(buf + L::oTILE + kTileBytes, a.dld, wide0, wstep, DK,
                                                                  sbase, t0, T, lane);
                                         });
            } else {
                producer_run<PreRows<R>>(ring, smem, L::bytes, team, nb, load_rows, stage_rows);
            }
        }
        return;
    }

    const int cb = 16 * wave;
    __builtin_amdgcn_s_setprio(2);  // the state recurrence is the serial part: let it issue first
    f4 DST[DV / 16];
    float run[4] = {0.f, 0.f, 0.f, 0.f};  // sum over later tokens of q*dq - k*dk, for key columns cb + 4g + i
#pragma unroll
    for (int i = 0; i < DV / 16; ++i) {
        if (a.dsf)
            DST[i] = *(const f4*)(a.dsf + ((size_t)bh * DK + sbase + cb + r) * DV + 16 * i + 4 * g);
        else
            DST[i] = f4{0.f, 0.f, 0.f, 0.f};
    }
    if constexpr (VAR == SLA_GLA) {
        if (a.dsf) {
#pragma unroll
            for (int i = 0; i < 4; ++i) run[i] = a.corr[(size_t)bh * DK + sbase + cb + 4 * g + i];
        }
    }
    for (int blk = 0; blk < nb; ++blk) {
        consumer_acquire(ring, blk);
        unsigned char* buf = smem + (blk & (kSlots - 1)) * L::bytes;
        const int t0 = (nb - 1 - blk) * kTok;
        const bool anchored = VAR == SLA_GLA && is_anchor(nb - 1 - blk);
        // The state entering this block, kept by the dq sweep: asked for here and used after the update, where the
        // registers allow it (the widest value dimension reads it at the point of use instead).
        constexpr bool kEarly = DV <= 128;
        u4 SA[kEarly ? DV / 32 : 1];
        const u4* st = a.anchor;
        if (anchored) {
            st += anchor_offset<DK, DV>(anchor_id(tok0, t0) * H + h, slice, wave) + lane;
            if constexpr (kEarly) {
#pragma unroll
                for (int c = 0; c < DV / 32; ++c) SA[c] = st[64 * c];
            }
        }
        const uint16_t* DOp = (const uint16_t*)(buf + L::oDO);
        const uint16_t* Vp = (const uint16_t*)(buf + L::oV);
        const float* GQ = (const float*)(buf + L::oGQ);
        // dP[t][j] = G^Q_t (dout_t . v_j), kept for j <= t
        f4 dP = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < DV / 32; ++c) mma32(dP, get_perm<DV>(DOp, r, g, c), get_perm<DV>(Vp, r, g, c));
        const f4 gq4 = *(const f4*)(GQ + 4 * g);
#pragma unroll
        for (int i = 0; i < 4; ++i) dP[i] = (r > 4 * g + i) ? 0.f : dP[i] * gq4[i];
        const s4 fp = pack4(dP);
        // Xs^T[d][j] = sum_n dS^T[n][d] v_j[n];  Xi^T[d][j] = sum_t qa_t[d] dP[t][j]
        f4 Xs = {0.f, 0.f, 0.f, 0.f}, Xi = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < DV / 32; ++c)
            mma32(Xs, join(pack4(DST[2 * c]), pack4(DST[2 * c + 1])), get_perm<DV>(Vp, r, g, c));
        const s4 fqa = get_T((const uint16_t*)(buf + L::oQAT), cb + r, g);
        mma16(Xi, fqa, fp);
        const f4 cum = *(const f4*)((const float*)(buf + L::oCUM) + r * kFS + cb + 4 * g);
        const f4 tot = *(const f4*)((const float*)(buf + L::oCUM) + (kTok - 1) * kFS + cb + 4 * g);
        f4 e = {0.f, 0.f, 0.f, 0.f}, bs4 = {0.f, 0.f, 0.f, 0.f};
        if constexpr (VAR == SLA_GLA) {
            e = *(const f4*)((const float*)(buf + L::oQDQ) + r * kFS + cb + 4 * g);
            bs4 = *(const f4*)(buf + L::bs_offset(cb + 4 * g));
        }
        const float gk = ((const float*)(buf + L::oGK))[r];
        const u2 kx = *(const u2*)((const uint16_t*)(buf + L::oKS) + r * kFS + cb + 4 * g);
        const float Ad = ex2(((const float*)(buf + L::oCUM))[(kTok - 1) * kFS + cb + r]);
        const uint16_t* DYT = (const uint16_t*)(buf + L::oDYT);
        s4 fdy[DV / 16];
#pragma unroll
        for (int i = 0; i < DV / 16; ++i) fdy[i] = get_T(DYT, 16 * i + r, g);
        consumer_release(ring, blk);  // every operand of the block is in registers
        // dS^T <- dS^T A + dy^T qa.  It is what the next block waits for: issued first where nothing else is kept alive
        // across it (RetNet: 109 -> 101 us per sweep); GLA's decay-gradient work holds too many registers for that
        // and ran 2 us slower, so there it stays last.
        auto update_state = [&]() {
#pragma unroll
            for (int i = 0; i < DV / 16; ++i) {
                DST[i] = DST[i] * Ad;
                mma16(DST[i], fdy[i], fqa);
            }
        };
        if constexpr (VAR != SLA_GLA) update_state();
        float dkp[4], dkv[4];  // before and after the write gate
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            dkp[i] = Xi[i] * ex2(-cum[i]) + Xs[i] * ex2(tot[i] - cum[i]);
            dkv[i] = gk * dkp[i];
        }
        const float kf[4] = {bf_lo(kx[0]), bf_hi(kx[0]), bf_lo(kx[1]), bf_hi(kx[1])};
        float part = kf[0] * dkp[0] + kf[1] * dkp[1] + kf[2] * dkp[2] + kf[3] * dkp[3];  // dG^K = k . dk'
        part = reduce_groups(part);
        const int tok = t0 + r;
        const bool ok = tok < T;
        const size_t row = (tok0 + (ok ? tok : 0)) * H + h, wrow = wide0 + (size_t)(ok ? tok : 0) * wstep;
        const u2 dk4 = u2{pack2(dkv[0], dkv[1]), pack2(dkv[2], dkv[3])};
        if constexpr (L::tiled) tile_put(buf + L::oTILE, r, 4 * wave + g, dk4);
        if (ok) {
            if (g == 0) a.part_k[((size_t)(slice * 4 + wave) * a.rows * H) + row] = part;
            if constexpr (!L::tiled) *(u2*)(a.dk + wrow * DK + sbase + cb + 4 * g) = dk4;
        }
        if constexpr (VAR == SLA_GLA) {
            // dlog_decay_t = sum_{s >= t} (q_s dq_s - k_s dk_s): inside the block one suffix scan of the per-token
            // differences, beyond it the running sum, which advances by the block's total plus the dq sweep's
            // correction of the bf16-derived q * dq values to their exact sum
            float dl[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float s = row_suffix(e[i] - kf[i] * dkv[i]);
                dl[i] = s + run[i];
                run[i] += bs4[i] + row_first(s);
            }
            const u2 dl4 = u2{pack2(dl[0], dl[1]), pack2(dl[2], dl[3])};
            if constexpr (L::tiled)
                tile_put(buf + L::oTILE + kTileBytes, r, 4 * wave + g, dl4);
            else if (ok)
                *(u2*)(a.dld + wrow * DK + sbase + cb + 4 * g) = dl4;
        }
        if constexpr (L::tiled) flag_signal(ring.out + (blk & (kSlots - 1)));
        if constexpr (VAR == SLA_GLA) update_state();
        if (anchored) {  // the sum over all later tokens equals rowsum(dS * S) at this boundary: take it from there
            float z = 0.f;
#pragma unroll
            for (int c = 0; c < DV / 32; ++c) {
                const u4 x = kEarly ? SA[kEarly ? c : 0] : st[64 * c];
                z += DST[2 * c][0] * bf_lo(x[0]) + DST[2 * c][1] * bf_hi(x[0]) + DST[2 * c][2] * bf_lo(x[1]) +
                     DST[2 * c][3] * bf_hi(x[1]) + DST[2 * c + 1][0] * bf_lo(x[2]) + DST[2 * c + 1][1] * bf_hi(x[2]) +
                     DST[2 * c + 1][2] * bf_lo(x[3]) + DST[2 * c + 1][3] * bf_hi(x[3]);
            }
            z = reduce_groups(z);  // every lane: the value of key column cb + lane % 16
#pragma unroll
            for (int i = 0; i < 4; ++i) run[i] = __shfl(z, 4 * g + i);
        }
    }
}

// ------------------------------------------------------------------------------------------------------------
// Sweep R1: backward in time, state dS[d][n] (key rows, 16 value columns per wave) -> dv, dG^K, d initial state.
// ------------------------------------------------------------------------------------------------------------
template <int DK>
struct SmemV {
    static constexpr int oQA = 0;
    static constexpr int oKD = oQA + kTok * (DK + 8) * 2;
    static constexpr int oKB = oKD + kTok * (DK + 8) * 2;
    static constexpr int oQAT = oKB + kTok * (DK + 8) * 2;
    static constexpr int oDYT = oQAT + DK * kTS * 2;
    static constexpr int oAT = oDYT + kCols * kTS * 2;
    static constexpr int oGK = oAT + DK * 4;
    static constexpr int bytes = oGK + kTok * 4;
    static constexpr int total = kSlots * bytes + 3 * kSlots * 4;
    static_assert(oKD % 16 == 0 && oKB % 16 == 0 && oQAT % 16 == 0 && oDYT % 16 == 0 &&
                      oAT % 16 == 0 && oGK % 16 == 0 && bytes % 16 == 0,
                  "tiles stay 16-byte aligned");
    static_assert(total <= 160 * 1024, "the ring fits the LDS of a compute unit");
};

template <int N>
struct PreVals {  // N groups of eight key columns of one token, and (member 0) two pieces of the dout slice
    u4 ld[N], kx[N], qx[N];
    u4 sl[2];
    float gq[2], gk;
};

template <int VAR, int DK, int DV>
__global__ __launch_bounds__(kBwdThreads) void sla_bwd_dv_kernel(const BArgs a) {
    typedef SmemV<DK> L;
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int NSL = DV / kCols;
    constexpr int N = DK / 64;  // each member wave stages half of the key columns: DK / 8 per lane
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, g = lane >> 4;
    const int wg = logical_workgroup(NSL, a.B * a.H, a.cu != nullptr);
    if (wg < 0) return;
    const int slice = wg % NSL, bh = wg / NSL, b = bh / a.H, h = bh % a.H;
    if (a.skip_every > 0 && b % a.skip_every == 0) return;  // pre-pass: the first segment of a row is not needed
    const int sbase = slice * kCols;
    const int H = a.H;
    int T = a.T;                    // tokens of this sequence and the index of its first token
    size_t tok0 = (size_t)b * a.T;
    if (a.cu) {  // packed sequences; offsets are clamped into the tensors whatever cu holds
        const int start = min(max(a.cu[b], 0), a.T), end = min(max(a.cu[b + 1], start), a.T);
        T = end - start;
        tok0 = (size_t)start;
    }
    // rows of the d-wide tensors: token tau of this sequence and head is row wide0 + tau * wstep
    const size_t wide0 = a.head_major ? (size_t)bh * a.T : tok0 * H + h, wstep = a.head_major ? 1 : H;
    const int nb = (T + kTok - 1) / kTok;
    const Ring ring = ring_init(smem, L::bytes, tid, a.status);

    if (wave >= kConsumers) {
        // member m: key columns m DK/2 + 8 (lane / 16) + 32 j ..., token lane % 16; member 0 also stages the slice of
        // dout (gated, transposed): two 16-byte pieces per lane
        const int team = (wave - kConsumers) >> 1, m = (wave - kConsumers) & 1;
        const int t = r, d0 = m * (DK / 2) + 8 * g;  // piece j adds 32 columns
        const uint16_t* slice_src = a.dout + sbase;
        const float head_step = VAR == SLA_RETNET ? a.ld_head[h] * kLog2e : 0.f;
        producer_run<PreVals<N>>(
            ring, smem, L::bytes, team, nb,
            [&](int I, PreVals<N>& p) {
                const int t0 = (nb - 1 - I) * kTok;
                const int tau = min(t0 + t, T - 1);
                const size_t row = (tok0 + tau) * H + h, wrow = wide0 + (size_t)tau * wstep;
#pragma unroll
                for (int j = 0; j < N; ++j) {
                    if constexpr (VAR == SLA_GLA) p.ld[j] = load16(a.ld + wrow * DK + d0 + 32 * j);
                    p.kx[j] = load16(a.k + wrow * DK + d0 + 32 * j);
                    p.qx[j] = load16(a.q + wrow * DK + d0 + 32 * j);
                }
                p.gk = a.gk[row];
                if (m == 0) {  // uniform over the wave
#pragma unroll
                    for (int rep = 0; rep < 2; ++rep) {
                        const int st = r, se8 = g + 4 * rep;
                        const int stau = min(t0 + st, T - 1);
                        const size_t srow = (tok0 + stau) * H + h;
                        p.sl[rep] = load16(slice_src + (wide0 + (size_t)stau * wstep) * DV + 8 * se8);
                        p.gq[rep] = a.gq[srow];
                    }
                }
            },
            [&](int I, const PreVals<N>& p, unsigned char* buf) {
                const int t0 = (nb - 1 - I) * kTok;
                const bool ok = t0 + t < T;
#pragma unroll
                for (int j = 0; j < N; ++j) {
                    const int c0 = d0 + 32 * j;
                    float c[8], tot[8];
                    block_decay<VAR>(keep(p.ld[j], ok), head_step, ok, c, tot);
                    const u4 qx = keep(p.qx[j], ok), kx = keep(p.kx[j], ok);
                    // kb = k A / p as (k / p) A: the block's decay A is one exponential per column, which the state
                    // update wants anyway, instead of one more per element (the quarter-rate unit is the busiest)
                    float A[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) A[i] = ex2(tot[i]);
                    u4 qa, kd, kb;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float kl = bf_lo(kx[i]) * ex2(-c[2 * i]), kh = bf_hi(kx[i]) * ex2(-c[2 * i + 1]);
                        qa[i] = pack2(bf_lo(qx[i]) * ex2(c[2 * i]), bf_hi(qx[i]) * ex2(c[2 * i + 1]));
                        kd[i] = pack2(kl, kh);
                        kb[i] = pack2(kl * A[2 * i], kh * A[2 * i + 1]);
                    }
                    put_perm<DK>((uint16_t*)(buf + L::oQA), t, c0 >> 3, qa);
                    put_perm<DK>((uint16_t*)(buf + L::oKD), t, c0 >> 3, kd);
                    put_perm<DK>((uint16_t*)(buf + L::oKB), t, c0 >> 3, kb);
                    put_T((uint16_t*)(buf + L::oQAT), c0, t, qa);
                    if (t == 0) {
                        float* at = (float*)(buf + L::oAT) + c0;
                        *(f4*)at = f4{A[0], A[1], A[2], A[3]};
                        *(f4*)(at + 4) = f4{A[4], A[5], A[6], A[7]};
                    }
                }
                if (m == 0 && g == 0) ((float*)(buf + L::oGK))[t] = ok ? p.gk : 0.f;
                if (m == 0) {
#pragma unroll
                    for (int rep = 0; rep < 2; ++rep) {
                        const int st = r, se8 = g + 4 * rep;
                        const u4 sl = keep(p.sl[rep], t0 + st < T);
                        u4 dy;
#pragma unroll
                        for (int j = 0; j < 4; ++j) dy[j] = pack2(p.gq[rep] * bf_lo(sl[j]), p.gq[rep] * bf_hi(sl[j]));
                        put_T((uint16_t*)(buf + L::oDYT), 8 * se8, st, dy);
                    }
                }
            });
        return;
    }

    const int cb = 16 * wave;
    __builtin_amdgcn_s_setprio(2);  // the state recurrence is the serial part: let it issue first
    f4 DS[DK / 16];  // rows d = 16 i + 4 g + (0..3), column n = sbase + cb + r
#pragma unroll
    for (int i = 0; i < DK / 16; ++i) {
        DS[i] = f4{0.f, 0.f, 0.f, 0.f};
        if (a.dsf) {
#pragma unroll
            for (int j = 0; j < 4; ++j) DS[i][j] = a.dsf[((size_t)bh * DK + 16 * i + 4 * g + j) * DV + sbase + cb + r];
        }
    }
    for (int blk = 0; blk < nb; ++blk) {
        consumer_acquire(ring, blk);
        unsigned char* buf = smem + (blk & (kSlots - 1)) * L::bytes;
        const int t0 = (nb - 1 - blk) * kTok;
        const uint16_t* QAp = (const uint16_t*)(buf + L::oQA);
        const uint16_t* KDp = (const uint16_t*)(buf + L::oKD);
        const uint16_t* KBp = (const uint16_t*)(buf + L::oKB);
        f4 Ys = {0.f, 0.f, 0.f, 0.f}, Yi = {0.f, 0.f, 0.f, 0.f};
        const s4 fdy = get_T((const uint16_t*)(buf + L::oDYT), cb + r, g);
        if (!a.dv_state_only) {  // the pre-pass of the segment schedule wants the state recurrence alone
            // Pq[t][j] = qa_t . kd_j, kept for j <= t
            f4 Pq = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < DK / 32; ++c) mma32(Pq, get_perm<DK>(QAp, r, g, c), get_perm<DK>(KDp, r, g, c));
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (r > 4 * g + i) Pq[i] = 0.f;
            const s4 fp = pack4(Pq);
            // dv'^T[n][j] = sum_d dS[d][n] kb_j[d] + sum_t dy_t[n] Pq[t][j]
#pragma unroll
            for (int c = 0; c < DK / 32; ++c)
                mma32(Ys, join(pack4(DS[2 * c]), pack4(DS[2 * c + 1])), get_perm<DK>(KBp, r, g, c));
            mma16(Yi, fdy, fp);
        }
        const float gk = ((const float*)(buf + L::oGK))[r];
        const uint16_t* QAT = (const uint16_t*)(buf + L::oQAT);
        const float* AT = (const float*)(buf + L::oAT);
        s4 fqat[DK / 16];
        f4 Ad[DK / 16];
#pragma unroll
        for (int i = 0; i < DK / 16; ++i) {
            fqat[i] = get_T(QAT, 16 * i + r, g);
            Ad[i] = *(const f4*)(AT + 16 * i + 4 * g);
        }
        consumer_release(ring, blk);  // every operand of the block is in registers
        const int tok = t0 + r;
        if (tok < T && !a.dv_state_only) {
            *(u2*)(a.dv + (wide0 + (size_t)tok * wstep) * DV + sbase + cb + 4 * g) =
                u2{pack2(gk * (Ys[0] + Yi[0]), gk * (Ys[1] + Yi[1])), pack2(gk * (Ys[2] + Yi[2]), gk * (Ys[3] + Yi[3]))};
        }
        // dS <- diag(A) dS + qa^T dy
#pragma unroll
        for (int i = 0; i < DK / 16; ++i) {
            DS[i] = DS[i] * Ad[i];
            mma16(DS[i], fqat[i], fdy);
        }
    }

    if (a.ds0) {
#pragma unroll
        for (int i = 0; i < DK / 16; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) a.ds0[((size_t)bh * DK + 16 * i + 4 * g + j) * DV + sbase + cb + r] = DS[i][j];
    }
}

// ------------------------------------------------------------------------------------------------------------
// Gates (Eq. 4) and their backward.
// ------------------------------------------------------------------------------------------------------------
// One thread per (token, head); the 256-thread block covers whole tokens (256 / H of them) and the sums over the
// heads of a token go through LDS.
constexpr int kEwThreads = 256;

__global__ __launch_bounds__(kEwThreads) void sla_bwd_gates_kernel(const float* ql, const float* kl, float* gq,
                                                                    float* gk, size_t rows, int H) {
    __shared__ float sx[kEwThreads];
    const int per = kEwThreads / H, tid = threadIdx.x, lr = tid / H, h = tid - lr * H;
    const size_t row = (size_t)blockIdx.x * per + lr;
    const bool ok = lr < per && row < rows;
    for (int which = 0; which < 2; ++which) {
        const float* x = which ? kl : ql;
        float* g = which ? gk : gq;
        if (!x) {  // uniform: G = 1
            if (ok) g[row * H + h] = 1.f;
            continue;
        }
        const float v = ok ? x[row * H + h] : 0.f;
        sx[tid] = v;
        __syncthreads();
        float m = -INFINITY;
        if (ok)
            for (int i = 0; i < H; ++i) m = fmaxf(m, sx[lr * H + i]);
        __syncthreads();
        const float e = ok ? ex2((v - m) * kLog2e) : 0.f;
        sx[tid] = e;
        __syncthreads();
        float s = 0.f;
        if (ok)
            for (int i = 0; i < H; ++i) s += sx[lr * H + i];
        if (ok) g[row * H + h] = e / s;
        __syncthreads();
    }
}

// dlogits = G * (dG - sum_h G dG), dG summed over its partial planes
// Packed batches (cu != null): rows outside [cu[0], cu[B]) belong to no sequence; the sweeps never wrote their
// partial planes, and their gradients are not written either.
__global__ __launch_bounds__(kEwThreads) void sla_bwd_logits_kernel(const float* g, const float* part, int planes,
                                                                     size_t plane, float* dl, size_t rows, int H,
                                                                     const int* cu, int B) {
    __shared__ float sx[kEwThreads];
    const int per = kEwThreads / H, tid = threadIdx.x, lr = tid / H, h = tid - lr * H;
    const size_t row = (size_t)blockIdx.x * per + lr;
    bool ok = lr < per && row < rows;
    if (cu) {
        const int total = (int)rows, lo = min(max(cu[0], 0), total), hi = min(max(cu[B], lo), total);
        ok = ok && row >= (size_t)lo && row < (size_t)hi;
    }
    float dg = 0.f, gv = 0.f;
    if (ok) {
        for (int p = 0; p < planes; ++p) dg += part[(size_t)p * plane + row * H + h];
        gv = g[row * H + h];
    }
    sx[tid] = gv * dg;
    __syncthreads();
    if (ok) {
        float dot = 0.f;
        for (int i = 0; i < H; ++i) dot += sx[lr * H + i];
        dl[row * H + h] = gv * (dg - dot);
    }
}

size_t round4(size_t n) { return (n + 3) & ~(size_t)3; }

template <typename K>
bool allow_lds(K kernel, int lds) {
    if (hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds) == hipSuccess)
        return true;
    (void)hipGetLastError();
    return false;
}

template <int VAR, int DK, int DV>
int launch_sweeps(const BArgs& a, hipStream_t stream) {
    constexpr int ldsF = SmemF<DV>::total, ldsV = SmemV<DK>::total, ldsK = SmemK<DV>::total;
    // once per device and instantiation (bit d = done on device d); not a stream operation
    static std::atomic<uint64_t> configured{0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();
        return SLA_ERR_HIP;
    }
    if (!((configured.load(std::memory_order_acquire) >> dev) & 1u)) {
        if (!allow_lds(sla_bwd_dq_kernel<VAR, DK, DV>, ldsF) || !allow_lds(sla_bwd_dv_kernel<VAR, DK, DV>, ldsV) ||
            !allow_lds(sla_bwd_dk_kernel<VAR, DK, DV>, ldsK))
            return SLA_ERR_HIP;
        configured.fetch_or(uint64_t(1) << dev, std::memory_order_release);
    }
    const unsigned bh = (unsigned)(a.B * a.H);
    const dim3 block(kBwdThreads);
    auto grid = [bh](unsigned slices) { return dim3(((bh + 7u) / 8u) * 8u * slices); };  // see logical_workgroup()
    if (a.sweeps & 1)
        hipLaunchKernelGGL((sla_bwd_dq_kernel<VAR, DK, DV>), grid(DK / kCols), block, (size_t)ldsF, stream, a);
    if (a.sweeps & 2)
        hipLaunchKernelGGL((sla_bwd_dv_kernel<VAR, DK, DV>), grid(DV / kCols), block, (size_t)ldsV, stream, a);
    if (a.sweeps & 4)
        hipLaunchKernelGGL((sla_bwd_dk_kernel<VAR, DK, DV>), grid(DK / kCols), block, (size_t)ldsK, stream, a);
    return hipGetLastError() == hipSuccess ? SLA_OK : SLA_ERR_HIP;
}

template <int VAR, int DK>
int launch_dv(const BArgs& a, int dv, hipStream_t stream) {
    switch (dv) {
        case 64: return launch_sweeps<VAR, DK, 64>(a, stream);
        case 128: return launch_sweeps<VAR, DK, 128>(a, stream);
        case 256: return launch_sweeps<VAR, DK, 256>(a, stream);
        default: return SLA_ERR_UNSUPPORTED;
    }
}

template <int VAR>
int launch_dk(const BArgs& a, int dk, int dv, hipStream_t stream) {
    switch (dk) {
        case 64: return launch_dv<VAR, 64>(a, dv, stream);
        case 128: return launch_dv<VAR, 128>(a, dv, stream);
        default: return SLA_ERR_UNSUPPORTED;
    }
}

}  // namespace

// Eq. 4 for both gates (G^K = 1 when kl is null), shared with the delta rule's backward.
int launch_bwd_gates(const float* ql, const float* kl, float* gq, float* gk, size_t rows, int H, hipStream_t stream) {
    if (rows == 0) return SLA_OK;
    const unsigned per = kEwThreads / (unsigned)H, eg = (unsigned)((rows + per - 1) / per);
    hipLaunchKernelGGL(sla_bwd_gates_kernel, dim3(eg), dim3(kEwThreads), 0, stream, ql, kl, gq, gk, rows, H);
    return hipGetLastError() == hipSuccess ? SLA_OK : SLA_ERR_HIP;
}

// dlogits = G * (dG - sum_h G dG) with dG the sum of `planes` partial planes, `plane` floats apart (shared with the
// fp32 path).
int launch_bwd_logits(const float* g, const float* part, int planes, size_t plane, float* dl, size_t rows, int H,
                      const int* cu, int B, hipStream_t stream) {
    if (rows == 0) return SLA_OK;
    const unsigned per = kEwThreads / (unsigned)H, eg = (unsigned)((rows + per - 1) / per);
    hipLaunchKernelGGL(sla_bwd_logits_kernel, dim3(eg), dim3(kEwThreads), 0, stream, g, part, planes, plane, dl, rows,
                       H, cu, B);
    return hipGetLastError() == hipSuccess ? SLA_OK : SLA_ERR_HIP;
}

size_t backward_f32_workspace_floats(const sla_params& p, bool packed);  // sla_backward_f32.hip
int launch_backward_f32(const sla_params& p, const void* q, const void* k, const void* v, const float* ql,
                        const float* kl, const void* ld, const float* s0, const void* dout, const float* dsf, void* dq,
                        void* dk, void* dv, float* dql, float* dkl, void* dld, float* ds0, float* ws, const int* cu,
                        hipStream_t stream);

// Workspace, in floats: gates G^Q, G^K [B,T,H]; partial dG^Q and dG^K (dk/16 planes each); for GLA the sums of
// q * dq over every 16-token block [rows/16 + B + 1][H,dk], the final-state term of dlog_decay [B,H,dk] and the
// states kept every 512 tokens [rows/512 + 1][H,dk,dv] in bf16.
size_t backward_workspace_floats(const sla_params& p, bool packed) {
    if (p.dtype == SLA_F32) return backward_f32_workspace_floats(p, packed);
    const size_t rows = packed ? (size_t)p.T : (size_t)p.B * p.T;
    const size_t n = round4(rows * p.H);
    size_t total = n * (2 + 2 * (p.dk / 16));
    if (p.variant == SLA_GLA)
        total += round4((rows / kTok + p.B + 1) * p.H * p.dk) + round4((size_t)p.B * p.H * p.dk) +
                 round4((rows / (kAnchor * kTok) + 1) * p.H * p.dk * p.dv / 2);
    return total;
}

namespace {

// Segment schedule of the backward pass (rectangular batch with few sequences): see launch_backward_segments.
__global__ __launch_bounds__(kEwThreads) void sla_bwd_segment_offsets_kernel(int* cu, int B, int T, int nseg, int len) {
    const int i = blockIdx.x * kEwThreads + threadIdx.x;
    if (i > B * nseg) return;
    const int b = i / nseg, s = i - b * nseg;
    cu[i] = i == B * nseg ? B * T : b * T + min(s * len, T);
}

// dsf[b][s] = the caller's final-state cotangent for the last segment of a batch row, zero for the others.
__global__ __launch_bounds__(kEwThreads) void sla_bwd_segment_seed_kernel(const f4* dsf_user, f4* dsf, int nseg,
                                                                          size_t per_row, size_t count) {
    const size_t i = (size_t)blockIdx.x * kEwThreads + threadIdx.x;
    if (i >= count) return;
    const size_t bs = i / per_row, b = bs / nseg, s = bs - b * nseg;
    dsf[i] = (dsf_user && s == (size_t)nseg - 1) ? dsf_user[b * per_row + (i - bs * per_row)] : f4{0.f, 0.f, 0.f, 0.f};
}

// part[b][s] holds the state cotangent at the START of segment s when the cotangent at its end is zero (the last
// segment: the caller's).  By linearity the true one is T_s = part_s + diag(D_s) T_{s+1}, and the cotangent at the
// END of segment s is T_{s+1}: written to dsf[b][s] (s < nseg - 1; the last keeps the caller's).  T_0 is the gradient
// with respect to the initial state.  One thread per (batch, head, key row, 4 value columns).
template <int VAR>
__global__ __launch_bounds__(kEwThreads) void sla_bwd_segment_combine_kernel(const float* part, const float* totals,
                                                                             const float* ld_head, float* dsf,
                                                                             float* ds0_user, int B, int H, int dk,
                                                                             int dv, int nseg, int len) {
    const int dv4 = dv / 4;
    const size_t per_head = (size_t)dk * dv4, idx = (size_t)blockIdx.x * kEwThreads + threadIdx.x;
    if (idx >= (size_t)B * H * per_head) return;
    const int bh = (int)(idx / per_head), b = bh / H, h = bh % H;
    const int d = (int)((idx % per_head) / dv4), n = (int)(idx % dv4) * 4;
    const size_t head_sz = (size_t)dk * dv, off = (size_t)d * dv + n;
    auto at = [&](int s) { return ((size_t)(b * nseg + s) * H + h) * head_sz + off; };
    f4 t = *(const f4*)(part + at(nseg - 1));
    for (int s = nseg - 2; s >= 0; --s) {
        *(f4*)(dsf + at(s)) = t;
        const float D = VAR == SLA_GLA ? totals[((size_t)(b * (nseg - 1) + s) * H + h) * dk + d]
                                       : ex2(ld_head[h] * kLog2e * (float)len);  // segments before the last are full
        const f4 x = *(const f4*)(part + at(s));
#pragma unroll
        for (int i = 0; i < 4; ++i) t[i] = x[i] + D * t[i];
    }
    if (ds0_user) *(f4*)(ds0_user + (size_t)bh * head_sz + off) = t;
}

}  // namespace

int launch_segment_states(const sla_params& p, int dvw, int nseg, int seg_len, const void* q, const void* k,
                          const void* v, const float* ql, const float* kl, const void* ld, const float* s0,
                          float* workspace, float* totals, hipStream_t stream);
size_t segment_workspace_floats(const sla_params& p, int nseg);

// Floats the segment schedule adds to the workspace of the packed backward over B * nseg sequences: the forward
// pre-pass's own workspace, segment decay totals, two state-sized arrays per segment and the segment offsets.
size_t backward_segment_extra_floats(const sla_params& p, int nseg) {
    const size_t states = (size_t)p.B * nseg * p.H * p.dk * p.dv;
    return round4(segment_workspace_floats(p, nseg)) + round4((size_t)p.B * (nseg - 1) * p.H * p.dk) + 2 * states +
           round4((size_t)p.B * nseg + 1);
}

sla_params packed_segments(const sla_params& p, int nseg) {
    sla_params pk = p;
    pk.B = p.B * nseg;
    pk.T = p.B * p.T;
    pk.segments = 1;
    return pk;
}

int launch_backward_some(const sla_params& p, const void* q, const void* k, const void* v, const float* ql,
                         const float* kl, const void* ld, const float* s0, const void* dout, const float* dsf, void* dq,
                         void* dk, void* dv, float* dql, float* dkl, void* dld, float* ds0, float* ws, const int* cu,
                         hipStream_t stream, int sweeps, bool dv_state_only, int skip_every = 0);

// Few sequences (B * H * slices below the number of compute units): every batch row is cut into nseg segments of
// seg_len tokens, which then run as B * nseg packed sequences, each with its own entry state and end cotangent:
//   1. entry states of the segments: the forward pass's pre-pass and combine kernel;
//   2. the dv sweep alone over the segments with zero end cotangents (the last segment: the caller's), which leaves
//      each segment's start cotangent; 3. a combine kernel turns those into the true end cotangents;
//   4. the packed backward pass over the segments.
int launch_backward_segments(const sla_params& p, int nseg, int seg_len, int dvw, const void* q, const void* k,
                             const void* v, const float* ql, const float* kl, const void* ld, const float* s0,
                             const void* dout, const float* dsf, void* dq, void* dk, void* dv, float* dql, float* dkl,
                             void* dld, float* ds0, float* ws, hipStream_t stream) {
    const sla_params pk = packed_segments(p, nseg);
    const size_t states = (size_t)pk.B * p.H * p.dk * p.dv;
    float* w = ws + backward_workspace_floats(pk, true);
    float* fwd = w; w += round4(segment_workspace_floats(p, nseg));  // entry states first
    float* totals = w; w += round4((size_t)p.B * (nseg - 1) * p.H * p.dk);
    float* part = w; w += states;
    float* seg_dsf = w; w += states;
    int* cu = (int*)w;
    const unsigned eb = kEwThreads;
    hipLaunchKernelGGL(sla_bwd_segment_offsets_kernel, dim3((unsigned)(pk.B + eb) / eb), dim3(eb), 0, stream, cu, p.B,
                       p.T, nseg, seg_len);
    hipLaunchKernelGGL(sla_bwd_segment_seed_kernel, dim3((unsigned)((states / 4 + eb - 1) / eb)), dim3(eb), 0, stream,
                       (const f4*)dsf, (f4*)seg_dsf, nseg, (size_t)p.H * p.dk * p.dv / 4, states / 4);
    if (hipGetLastError() != hipSuccess) return SLA_ERR_HIP;
    int rc = launch_segment_states(p, dvw, nseg, seg_len, q, k, v, ql, kl, ld, s0, fwd, totals, stream);
    if (rc != SLA_OK) return rc;
    // the start cotangent of a row's first segment is wanted only as the gradient of the initial state
    rc = launch_backward_some(pk, q, k, v, ql, kl, ld, nullptr, dout, seg_dsf, dq, dk, dv, dql, dkl, dld, part, ws, cu,
                              stream, 2, true, ds0 ? 0 : nseg);
    if (rc != SLA_OK) return rc;
    const size_t n = (size_t)p.B * p.H * p.dk * (p.dv / 4);
    if (p.variant == SLA_GLA)
        hipLaunchKernelGGL(sla_bwd_segment_combine_kernel<SLA_GLA>, dim3((unsigned)((n + eb - 1) / eb)), dim3(eb), 0,
                           stream, (const float*)part, (const float*)totals, (const float*)nullptr, seg_dsf, ds0, p.B,
                           p.H, p.dk, p.dv, nseg, seg_len);
    else
        hipLaunchKernelGGL(sla_bwd_segment_combine_kernel<SLA_RETNET>, dim3((unsigned)((n + eb - 1) / eb)), dim3(eb), 0,
                           stream, (const float*)part, (const float*)nullptr, (const float*)ld, seg_dsf, ds0, p.B, p.H,
                           p.dk, p.dv, nseg, seg_len);
    if (hipGetLastError() != hipSuccess) return SLA_ERR_HIP;
    return launch_backward_some(pk, q, k, v, ql, kl, ld, fwd, dout, seg_dsf, dq, dk, dv, dql, dkl, dld, nullptr, ws, cu,
                                stream, 7, false);
}

int launch_backward(const sla_params& p, const void* q, const void* k, const void* v, const float* ql, const float* kl,
                    const void* ld, const float* s0, const void* dout, const float* dsf, void* dq, void* dk, void* dv,
                    float* dql, float* dkl, void* dld, float* ds0, float* ws, const int* cu, hipStream_t stream) {
    if (p.dtype == SLA_F32)  // fp32 tensors: token by token in fp32 vector arithmetic
        return launch_backward_f32(p, q, k, v, ql, kl, ld, s0, dout, dsf, dq, dk, dv, dql, dkl, dld, ds0, ws, cu, stream);
    return launch_backward_some(p, q, k, v, ql, kl, ld, s0, dout, dsf, dq, dk, dv, dql, dkl, dld, ds0, ws, cu, stream, 7,
                                false);
}

int launch_backward_some(const sla_params& p, const void* q, const void* k, const void* v, const float* ql,
                         const float* kl, const void* ld, const float* s0, const void* dout, const float* dsf, void* dq,
                         void* dk, void* dv, float* dql, float* dkl, void* dld, float* ds0, float* ws, const int* cu,
                         hipStream_t stream, int sweeps, bool dv_state_only, int skip_every) {
    const size_t rows = cu ? (size_t)p.T : (size_t)p.B * p.T, n = round4(rows * p.H);
    BArgs a;
    a.sweeps = sweeps;
    a.dv_state_only = dv_state_only;
    a.skip_every = skip_every;
    a.status = device_status_word();
    if (!a.status) return SLA_ERR_HIP;
    a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v; a.dout = (const uint16_t*)dout;
    a.ld = p.variant == SLA_GLA ? (const uint16_t*)ld : nullptr;
    a.ld_head = p.variant == SLA_RETNET ? (const float*)ld : nullptr;
    float* w = ws;
    float* gq = w; w += n;
    float* gk = w; w += n;
    a.gq = gq; a.gk = gk;
    a.part_q = w; w += n * (p.dk / 16);
    a.part_k = w; w += n * (p.dk / 16);
    a.bsum = nullptr; a.corr = nullptr; a.anchor = nullptr;
    if (p.variant == SLA_GLA) {
        a.bsum = w; w += round4((rows / kTok + p.B + 1) * p.H * p.dk);
        a.corr = w; w += round4((size_t)p.B * p.H * p.dk);
        a.anchor = (u4*)w;  // 16-byte aligned: every part before it is a multiple of four floats
    }
    a.s0 = s0; a.dsf = dsf;
    a.dq = (uint16_t*)dq; a.dk = (uint16_t*)dk; a.dv = (uint16_t*)dv; a.dld = (uint16_t*)dld; a.ds0 = ds0;
    a.B = p.B; a.T = p.T; a.H = p.H; a.rows = rows; a.cu = cu;
    a.head_major = (p.flags & SLA_FLAG_HEAD_MAJOR) != 0;

    const unsigned eb = kEwThreads, per = eb / (unsigned)p.H, eg = (unsigned)((rows + per - 1) / per);
    if (rows > 0) {
        hipLaunchKernelGGL(sla_bwd_gates_kernel, dim3(eg), dim3(eb), 0, stream, ql, kl, gq, gk, rows, p.H);
        if (hipGetLastError() != hipSuccess) return SLA_ERR_HIP;
    }
    const int rc = p.variant == SLA_GLA ? launch_dk<SLA_GLA>(a, p.dk, p.dv, stream)
                                        : launch_dk<SLA_RETNET>(a, p.dk, p.dv, stream);
    if (rc != SLA_OK || rows == 0 || sweeps != 7) return rc;
    // the sweeps write the planes of one gate rows * H floats apart (the space reserved per plane is n >= rows * H)
    int rl = launch_bwd_logits(gq, a.part_q, p.dk / 16, rows * p.H, dql, rows, p.H, cu, p.B, stream);
    if (rl == SLA_OK && kl) rl = launch_bwd_logits(gk, a.part_k, p.dk / 16, rows * p.H, dkl, rows, p.H, cu, p.B, stream);
    return rl;
}

}  // namespace sla
