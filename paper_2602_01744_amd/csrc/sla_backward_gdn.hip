// Backward pass of the gated delta rule with SLA's head gates (Softmax-GatedDeltaNet, Sec. 5.1), bf16 or fp32 tensors.
//
// Forward step, per head, with a scalar decay a_t = exp(log_decay_t) and write strength beta_t:
//     Sb = a_t S_{t-1}      res_t = G^K_t v_t - k_t Sb      u_t = beta_t res_t      S_t = Sb + k_t^T u_t
//     out_t = G^Q_t q_t S_t
// and, walking back with X_t the gradient with respect to S_t (including token t's own read-out term):
//     X_t = dS + q_t^T dy_t (dy = G^Q dout)      du_t = k_t X_t       w_t = beta_t du_t
//     dv_t = G^K_t w_t     dG^K_t = beta_t du_t . v_t     dbeta_t = du_t . res_t
//     dk_t = X_t u_t - a_t w_t S_{t-1}^T          dq_t = dy_t S_t^T   dG^Q_t = dout_t . (q_t S_t)
//     dS   = a_t (X_t - k_t^T w_t)
//     dlog_decay_t = <d_final, S_T> + sum_{s >= t} (G^Q_s dG^Q_s - G^K_s dG^K_s)
// (the last line: <X_t, S_t> changes by exactly these token-local scalars from one token to the next).
//
// Only two quantities depend on a state through the delta rule's own feedback: res_t (forward) and w_t (backward).
// Once they are known every state recurrence is linear, so the pass is four sweeps that each carry one state tile in
// registers, token by token, in plain fp32 vector arithmetic (the feedback makes tokens of a block depend on each
// other; no matrix-core block form is used here):
//   1. state sweep, forward in time, state tile [dk rows, 8 value columns] per wave: res_t;
//   2. cotangent sweep, backward in time, same tile shape: w_t, dv, partial dG^K and dbeta, d_initial_state;
//   3. key sweep, backward in time, tile [dv rows, 8 key columns] of X^T: the first part of dk, X_t u_t;
//   4. query sweep, forward in time, tile [dv rows, 8 key columns] of S^T: dq, partial dG^Q, dk completed,
//      <d_final, S_T>.
// A finishing kernel sums the partial planes, takes the gate gradients through the head softmax of Eq. 4 and writes
// dbeta; a scan kernel forms dlog_decay.
//
// Tile layout of a wave (all four sweeps): lane = 16 * (column group) + (row group); a lane holds ROWS/16 rows by
// 2 columns of the tile, a wave 8 columns.  A product that contracts the rows is a per-lane partial sum followed by
// a rotate-and-add over the 16 lanes of a DPP row, which leaves the total in every lane.  A workgroup is eight such
// waves (64 columns, two waves per SIMD so that one computes while the other waits for the LDS) plus four loader
// waves that stage the next 16 tokens (as fp32) into the other half of a double-buffered LDS area while the compute
// waves work; one barrier per 16 tokens.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "sla.h"
#include "sla_gdn_block.h"
#include "sla_token_sweep.h"

namespace sla {

int launch_bwd_gates(const float* ql, const float* kl, float* gq, float* gk, size_t rows, int H, hipStream_t stream);

namespace {

using namespace tok;


struct GArgs {
    const void* q;          // [B,T,H,dk], bf16 or fp32 (the kernels' element type E)
    const void* k;
    const void* v;          // [B,T,H,dv]
    const void* dout;
    const float* ld;        // [B,T,H]
    const float* beta;
    const float* gq;        // gates [B,T,H]
    const float* gk;
    const float* s0;        // [B,H,dk,dv] or null
    const float* dsf;
    void* dq;
    void* dk;
    void* dv;
    float* ds0;
    float* res;             // [B,T,H,dv] fp32: G^K v - k Sb
    float* w;               // [B,T,H,dv] fp32: beta * (k X)
    float* dk1;             // [B,T,H,dk] fp32: X u
    float* part_q;          // [dk/8][plane]: partial q . (dout S^T)
    float* part_k;          // [dv/8][plane]: partial beta du . v
    float* part_b;          // [dv/8][plane]: partial du . res
    float* corr;            // [dk/8][B*H]: partial <d_final, S_T>
    size_t plane;           // floats between partial planes (>= rows * H)
    size_t rows;            // tokens in all: B * T, or the packed total T
    const int* cu;          // packed batch: sequence b is tokens cu[b] .. cu[b+1]-1 of the T in all; else null
    int B, T, H;
};



// Per-token scalars {a, beta, G^Q, G^K, F, 1/F, R, 1/R}; a token past the end leaves every state unchanged (a = 1,
// the gates and beta 0).  The sweeps keep their state tile divided by a running decay product so that the decay costs
// no multiplication per tile element: inside a group of kNorm tokens a forward sweep holds S / F_t with
// F_t = product of a over the group's tokens up to t, a backward sweep holds X / R_t with R_t = product of a over the
// group's tokens after t; at the end of a group the tile is multiplied out.  With log_decay >= -20 per token the
// products stay above e^-80, inside fp32's range.
constexpr int kNorm = 4;
constexpr int kScal = 8;
struct RegsS {
    float ld, be, gq, gk;
    __device__ __forceinline__ void load(const GArgs& a, size_t tok0, int h, int t0, int T, int lt) {
        const size_t i = (tok0 + (size_t)min(t0 + (lt & (kChunk - 1)), T - 1)) * a.H + h;
        ld = a.ld[i]; be = a.beta[i]; gq = a.gq[i]; gk = a.gk[i];
    }
    __device__ __forceinline__ void put(float* dst, int t0, int T, int lt) const {
        const bool ok = t0 + (lt & (kChunk - 1)) < T;
        const float al = ok ? __builtin_amdgcn_exp2f(ld * kLog2e) : 1.f;
        float F = 1.f, R = 1.f;  // lanes 0..15 of the first loader wave hold the chunk's 16 tokens
#pragma unroll
        for (int j = 0; j < kNorm; ++j) {
            const float x = __shfl(al, (lt & (kChunk - kNorm)) + j);
            if (j <= (lt & (kNorm - 1))) F *= x;
            else R *= x;
        }
        if (lt < kChunk) {
            float* d = dst + kScal * lt;
            *(f4*)d = ok ? f4{al, be, gq, gk} : f4{1.f, 0.f, 0.f, 0.f};
            *(f4*)(d + 4) = f4{F, __builtin_amdgcn_rcpf(F), R, __builtin_amdgcn_rcpf(R)};
        }
    }
};


// ------------------------------------------------------------------------------------------------------------
// Sweep 1: forward in time, S[dk rows, value columns] -> res.
// ------------------------------------------------------------------------------------------------------------
template <class E, int DK, int DV>
__global__ __launch_bounds__(kThreads) void gdn_bwd_state_kernel(const GArgs a) {
    constexpr int RT = DK / 16;
    constexpr int oK = 0, oV = oK + kChunk * DK, oSC = oV + kChunk * kSlice, kBuf = oSC + kScal * kChunk;
    extern __shared__ __align__(16) unsigned char smem[];
    float* lds = (float*)smem;
    const Where me = where(a, DV / kSlice);
    if (me.bh < 0) return;
    const int T = me.T, H = a.H, nch = (T + kChunk - 1) / kChunk;
    const size_t sk = (size_t)H * DK, sv = (size_t)H * DV;
    if (me.wave >= kWaves) {
        const int lt = me.tid - 64 * kWaves;
        const E* kb = (const E*)a.k + (me.tok0 * H + me.h) * DK;
        const E* vb = (const E*)a.v + (me.tok0 * H + me.h) * DV + me.slice * kSlice;
        for (int c = 0; c <= nch; ++c) {
            if (c < nch) {
                const int t0 = c * kChunk;
                float* buf = lds + (c & 1) * kBuf;
                RegsIn<E, DK> rk;
                RegsIn<E, kSlice> rv;
                RegsS rs;
                rk.load(kb, sk, t0, T, lt);
                rv.load(vb, sv, t0, T, lt);
                rs.load(a, me.tok0, me.h, t0, T, lt);
                rk.put_rows(buf + oK, t0, T, lt);
                rv.put(buf + oV, t0, T, lt);
                rs.put(buf + oSC, t0, T, lt);
            }
            __syncthreads();
        }
        return;
    }
    float M[RT][CW];
#pragma unroll
    for (int r = 0; r < RT; ++r) {
        const fc x = a.s0 ? *(const fc*)(a.s0 + ((size_t)me.bh * DK + me.rg * RT + r) * DV + me.col) : fc{0.f, 0.f};
#pragma unroll
        for (int j = 0; j < CW; ++j) M[r][j] = x[j];
    }
    __syncthreads();  // chunk 0 staged
    for (int c = 0; c < nch; ++c) {
        const float* buf = lds + (c & 1) * kBuf;
#pragma unroll kNorm
        for (int i = 0; i < kChunk; ++i) {
            const f4 sc = *(const f4*)(buf + oSC + kScal * i), sn = *(const f4*)(buf + oSC + kScal * i + 4);
            const float be = sc[1], gk = sc[3], F = sn[0], Fi = sn[1];  // M holds S / F
            float kf[RT];
            get_rows<RT>(kf, buf + oK + i * DK + me.rg * 4);
            const fc vv = *(const fc*)(buf + oV + i * kSlice + me.lcol);
            float p[CW] = {};
#pragma unroll
            for (int r = 0; r < RT; ++r)
#pragma unroll
                for (int j = 0; j < CW; ++j) p[j] += kf[r] * M[r][j];
            fc res;
            float u[CW];
#pragma unroll
            for (int j = 0; j < CW; ++j) {
                res[j] = gk * vv[j] - F * row_all(p[j]);  // k Sb = a k S_{t-1} = F_t k (S_{t-1} / F_{t-1})
                u[j] = be * res[j] * Fi;
            }
#pragma unroll
            for (int r = 0; r < RT; ++r)
#pragma unroll
                for (int j = 0; j < CW; ++j) M[r][j] += kf[r] * u[j];
            if ((i & (kNorm - 1)) == kNorm - 1) {
#pragma unroll
                for (int r = 0; r < RT; ++r)
#pragma unroll
                    for (int j = 0; j < CW; ++j) M[r][j] *= F;
            }
            const int t = c * kChunk + i;
            if (t < T) {
                const size_t row = (me.tok0 + t) * H + me.h;
                if (me.rg == 0) *(fc*)(a.res + row * DV + me.col) = res;
            }
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------------------------
// Sweep 2: backward in time, X[dk rows, value columns] -> w, dv, partial dG^K and dbeta, d_initial_state.
// ------------------------------------------------------------------------------------------------------------
template <class E, int DK, int DV>
__global__ __launch_bounds__(kThreads) void gdn_bwd_cotangent_kernel(const GArgs a) {
    constexpr int RT = DK / 16;
    constexpr int oK = 0, oQ = oK + kChunk * DK, oV = oQ + kChunk * DK, oDO = oV + kChunk * kSlice,
                  oR = oDO + kChunk * kSlice, oSC = oR + kChunk * kSlice, kBuf = oSC + kScal * kChunk;
    extern __shared__ __align__(16) unsigned char smem[];
    float* lds = (float*)smem;
    const Where me = where(a, DV / kSlice);
    if (me.bh < 0) return;
    const int T = me.T, H = a.H, nch = (T + kChunk - 1) / kChunk;
    const size_t sk = (size_t)H * DK, sv = (size_t)H * DV;
    if (me.wave >= kWaves) {  // step c of the sweep covers tokens (nch - 1 - c) * 16 ...
        const int lt = me.tid - 64 * kWaves;
        const E* kb = (const E*)a.k + (me.tok0 * H + me.h) * DK;
        const E* qb = (const E*)a.q + (me.tok0 * H + me.h) * DK;
        const E* vb = (const E*)a.v + (me.tok0 * H + me.h) * DV + me.slice * kSlice;
        const E* db = (const E*)a.dout + (me.tok0 * H + me.h) * DV + me.slice * kSlice;
        const float* rb = a.res + (me.tok0 * H + me.h) * DV + me.slice * kSlice;
        for (int c = 0; c <= nch; ++c) {
            if (c < nch) {
                const int t0 = (nch - 1 - c) * kChunk;
                float* buf = lds + (c & 1) * kBuf;
                RegsIn<E, DK> rk, rq;
                RegsIn<E, kSlice> rv, rd;
                RegsF<kSlice> rr;
                RegsS rs;
                rk.load(kb, sk, t0, T, lt); rq.load(qb, sk, t0, T, lt);
                rv.load(vb, sv, t0, T, lt); rd.load(db, sv, t0, T, lt);
                rr.load(rb, sv, t0, T, lt);
                rs.load(a, me.tok0, me.h, t0, T, lt);
                rk.put_rows(buf + oK, t0, T, lt); rq.put_rows(buf + oQ, t0, T, lt);
                rv.put(buf + oV, t0, T, lt); rd.put(buf + oDO, t0, T, lt);
                rr.put(buf + oR, t0, T, lt);
                rs.put(buf + oSC, t0, T, lt);
            }
            __syncthreads();
        }
        return;
    }
    float X[RT][CW];
#pragma unroll
    for (int r = 0; r < RT; ++r) {
        const fc x = a.dsf ? *(const fc*)(a.dsf + ((size_t)me.bh * DK + me.rg * RT + r) * DV + me.col) : fc{0.f, 0.f};
#pragma unroll
        for (int j = 0; j < CW; ++j) X[r][j] = x[j];
    }
    __syncthreads();
    for (int c = 0; c < nch; ++c) {
        const float* buf = lds + (c & 1) * kBuf;
#pragma unroll kNorm
        for (int i = kChunk - 1; i >= 0; --i) {
            const f4 sc = *(const f4*)(buf + oSC + kScal * i), sn = *(const f4*)(buf + oSC + kScal * i + 4);
            const float al = sc[0], be = sc[1], gq = sc[2], gk = sc[3], R = sn[2], Ri = sn[3];  // X holds X_t / R
            float kf[RT], qf[RT];
            get_rows<RT>(kf, buf + oK + i * DK + me.rg * 4);
            get_rows<RT>(qf, buf + oQ + i * DK + me.rg * 4);
            const int lc = i * kSlice + me.lcol;
            const fc vv = *(const fc*)(buf + oV + lc), dd = *(const fc*)(buf + oDO + lc), rr = *(const fc*)(buf + oR + lc);
            float du[CW] = {};
#pragma unroll
            for (int r = 0; r < RT; ++r)
#pragma unroll
                for (int j = 0; j < CW; ++j) {
                    X[r][j] += qf[r] * (gq * Ri * dd[j]);
                    du[j] += kf[r] * X[r][j];
                }
            fc w;
            float pk = 0.f, pb = 0.f, wr[CW];
#pragma unroll
            for (int j = 0; j < CW; ++j) {
                du[j] = R * row_all(du[j]);
                w[j] = be * du[j];
                wr[j] = w[j] * Ri;
                pk += du[j] * vv[j];
                pb += du[j] * rr[j];
            }
            const bool out_of_group = (i & (kNorm - 1)) == 0;  // then multiply out: X_{t-1} = a R (X/R - k w/R)
            const float mul = R * al;
#pragma unroll
            for (int r = 0; r < RT; ++r)
#pragma unroll
                for (int j = 0; j < CW; ++j) {
                    X[r][j] -= kf[r] * wr[j];
                    if (out_of_group) X[r][j] *= mul;
                }
            pk = all_groups(pk) * be;
            pb = all_groups(pb);
            const int t = (nch - 1 - c) * kChunk + i;
            if (t < T) {
                const size_t row = (me.tok0 + t) * H + me.h;
                if (me.lane == 0) {
                    a.part_k[(size_t)(me.slice * kWaves + me.wave) * a.plane + row] = pk;
                    a.part_b[(size_t)(me.slice * kWaves + me.wave) * a.plane + row] = pb;
                }
                if (me.rg == 0) {
                    *(fc*)(a.w + row * DV + me.col) = w;
                    store2((E*)a.dv + row * DV + me.col, gk * w[0], gk * w[1]);
                }
            }
        }
        __syncthreads();
    }
    if (a.ds0) {
#pragma unroll
        for (int r = 0; r < RT; ++r)
            *(fc*)(a.ds0 + ((size_t)me.bh * DK + me.rg * RT + r) * DV + me.col) = fc{X[r][0], X[r][1]};
    }
}

// ------------------------------------------------------------------------------------------------------------
// Sweeps 3 and 4 carry the transposed tiles: rows are the dv value columns, a workgroup owns 64 key columns.
//   FWD = false (sweep 3, backward in time):  X^T += dy^T q;  dk1 = u X^T;   X^T = a (X^T - w^T k)
//   FWD = true  (sweep 4, forward in time):   pk = w S^T;     S^T = a S^T + u^T k;   dq = G^Q dout S^T;
//                                             dk = dk1 - a pk
// ------------------------------------------------------------------------------------------------------------
template <class E, int DK, int DV, bool FWD>
__global__ __launch_bounds__(kThreads) void gdn_bwd_key_kernel(const GArgs a) {
    constexpr int RT = DV / 16;
    constexpr int oDO = 0, oR = oDO + kChunk * DV, oW = oR + kChunk * DV, oK = oW + kChunk * DV,
                  oX = oK + kChunk * kSlice,  // sweep 3: q slice; sweep 4: dk1 slice
        oQ = oX + kChunk * kSlice,              // sweep 4: q slice (for dG^Q = q . dq')
        oSC = oQ + kChunk * kSlice, kBuf = oSC + kScal * kChunk;
    extern __shared__ __align__(16) unsigned char smem[];
    float* lds = (float*)smem;
    const Where me = where(a, DK / kSlice);
    if (me.bh < 0) return;
    const int T = me.T, H = a.H, nch = (T + kChunk - 1) / kChunk;
    const size_t sk = (size_t)H * DK, sv = (size_t)H * DV;
    if (me.wave >= kWaves) {
        const int lt = me.tid - 64 * kWaves;
        const E* db = (const E*)a.dout + (me.tok0 * H + me.h) * DV;
        const float* rb = a.res + (me.tok0 * H + me.h) * DV;
        const float* wb = a.w + (me.tok0 * H + me.h) * DV;
        const E* kb = (const E*)a.k + (me.tok0 * H + me.h) * DK + me.slice * kSlice;
        const E* qb = (const E*)a.q + (me.tok0 * H + me.h) * DK + me.slice * kSlice;
        const float* d1 = a.dk1 + (me.tok0 * H + me.h) * DK + me.slice * kSlice;
        for (int c = 0; c <= nch; ++c) {
            if (c < nch) {
                const int t0 = (FWD ? c : nch - 1 - c) * kChunk;
                float* buf = lds + (c & 1) * kBuf;
                RegsIn<E, DV> rd;
                RegsF<DV> rr, rw;
                RegsIn<E, kSlice> rk, rq;
                RegsF<kSlice> r1;
                RegsS rs;
                rd.load(db, sv, t0, T, lt); rr.load(rb, sv, t0, T, lt); rw.load(wb, sv, t0, T, lt);
                rk.load(kb, sk, t0, T, lt);
                rq.load(qb, sk, t0, T, lt);
                if constexpr (FWD) r1.load(d1, sk, t0, T, lt);
                rs.load(a, me.tok0, me.h, t0, T, lt);
                rd.put_rows(buf + oDO, t0, T, lt); rr.put_rows(buf + oR, t0, T, lt); rw.put_rows(buf + oW, t0, T, lt);
                rk.put(buf + oK, t0, T, lt);
                if constexpr (FWD) {
                    r1.put(buf + oX, t0, T, lt);
                    rq.put(buf + oQ, t0, T, lt);
                } else {
                    rq.put(buf + oX, t0, T, lt);
                }
                rs.put(buf + oSC, t0, T, lt);
            }
            __syncthreads();
        }
        return;
    }
    // tile element [r][j]: value column n = rg * RT + r, key column d = col + j
    float M[RT][CW];
    const float* init = FWD ? a.s0 : a.dsf;
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int j = 0; j < CW; ++j)
            M[r][j] = init ? init[((size_t)me.bh * DK + me.col + j) * DV + me.rg * RT + r] : 0.f;
    __syncthreads();
    for (int c = 0; c < nch; ++c) {
        const float* buf = lds + (c & 1) * kBuf;
#pragma unroll kNorm
        for (int ii = 0; ii < kChunk; ++ii) {
            const int i = FWD ? ii : kChunk - 1 - ii;
            const f4 sc = *(const f4*)(buf + oSC + kScal * i), sn = *(const f4*)(buf + oSC + kScal * i + 4);
            const float al = sc[0], be = sc[1], gq = sc[2];
            const float N = FWD ? sn[0] : sn[2], Ni = FWD ? sn[1] : sn[3];  // M holds S^T / F or X^T / R
            float dd[RT], rr[RT], ww[RT];
            get_rows<RT>(dd, buf + oDO + i * DV + me.rg * 4);
            get_rows<RT>(rr, buf + oR + i * DV + me.rg * 4);
            get_rows<RT>(ww, buf + oW + i * DV + me.rg * 4);
            const int lc = i * kSlice + me.lcol;
            const fc kf = *(const fc*)(buf + oK + lc), xf = *(const fc*)(buf + oX + lc);
            const int t = (FWD ? c : nch - 1 - c) * kChunk + i;
            const size_t row = (me.tok0 + min(t, T - 1)) * H + me.h;
            if constexpr (FWD) {
                float pk[CW] = {}, y[CW] = {};
#pragma unroll
                for (int r = 0; r < RT; ++r)
#pragma unroll
                    for (int j = 0; j < CW; ++j) {
                        pk[j] += ww[r] * M[r][j];
                        M[r][j] += (be * Ni * rr[r]) * kf[j];
                        y[j] += dd[r] * M[r][j];
                    }
                const fc qf = *(const fc*)(buf + oQ + lc);
                float dq[CW], dk[CW], pq = 0.f;
#pragma unroll
                for (int j = 0; j < CW; ++j) {
                    const float dqp = N * row_all(y[j]);  // before the read gate: dG^Q = q . dq'
                    pq += qf[j] * dqp;
                    dq[j] = gq * dqp;
                    dk[j] = xf[j] - N * row_all(pk[j]);  // a w S_{t-1}^T = F_t w (S_{t-1} / F_{t-1})^T
                }
                pq = all_groups(pq);
                if (t < T && me.lane == 0) a.part_q[(size_t)(me.slice * kWaves + me.wave) * a.plane + row] = pq;
                if ((i & (kNorm - 1)) == kNorm - 1) {
#pragma unroll
                    for (int r = 0; r < RT; ++r)
#pragma unroll
                        for (int j = 0; j < CW; ++j) M[r][j] *= N;
                }
                if (t < T && me.rg == 0) {
                    store2((E*)a.dq + row * DK + me.col, dq[0], dq[1]);
                    store2((E*)a.dk + row * DK + me.col, dk[0], dk[1]);
                }
            } else {
                float d1[CW] = {};
#pragma unroll
                for (int r = 0; r < RT; ++r)
#pragma unroll
                    for (int j = 0; j < CW; ++j) {
                        M[r][j] += (gq * Ni * dd[r]) * xf[j];
                        d1[j] += (be * rr[r]) * M[r][j];
                        M[r][j] -= (Ni * ww[r]) * kf[j];
                    }
                fc o;
#pragma unroll
                for (int j = 0; j < CW; ++j) o[j] = N * row_all(d1[j]);
                if ((i & (kNorm - 1)) == 0) {
                    const float mul = N * al;
#pragma unroll
                    for (int r = 0; r < RT; ++r)
#pragma unroll
                        for (int j = 0; j < CW; ++j) M[r][j] *= mul;
                }
                if (t < T && me.rg == 0) *(fc*)(a.dk1 + row * DK + me.col) = o;
            }
        }
        __syncthreads();
    }
    if constexpr (FWD) {
        if (a.dsf) {  // <d_final, S_T> over this wave's key columns (the tile was multiplied out after the last token)
            float s = 0.f;
#pragma unroll
            for (int r = 0; r < RT; ++r)
#pragma unroll
                for (int j = 0; j < CW; ++j)
                    s += a.dsf[((size_t)me.bh * DK + me.col + j) * DV + me.rg * RT + r] * M[r][j];
            s = all_groups(row_all(s));
            if (me.lane == 0) a.corr[(size_t)(me.slice * kWaves + me.wave) * a.B * a.H + me.bh] = s;
        }
    }
}

// ------------------------------------------------------------------------------------------------------------
// Finishing: sums of the partial planes; gate gradients through the head softmax (Eq. 4); dbeta; the per-token
// scalar G^Q dG^Q - G^K dG^K whose suffix sums are dlog_decay.
// ------------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kEw) void gdn_bwd_finish_kernel(const GArgs a, int planes_q, int planes_v, float* dql,
                                                             float* dkl, float* dbeta, float* e) {
    __shared__ float sx[kEw];
    const int H = a.H, per = kEw / H, tid = threadIdx.x, lr = tid / H, h = tid - lr * H;
    const size_t rows = a.rows, row = (size_t)blockIdx.x * per + lr;
    bool ok = lr < per && row < rows;
    if (a.cu) {  // packed batch: rows outside [cu[0], cu[B]) belong to no sequence and are left untouched
        const int total = (int)rows, lo = min(max(a.cu[0], 0), total), hi = min(max(a.cu[a.B], lo), total);
        ok = ok && row >= (size_t)lo && row < (size_t)hi;
    }
    const size_t i = ok ? row * H + h : 0;
    float dgq = 0.f, dgk = 0.f, db = 0.f, gq = 0.f, gk = 0.f;
    if (ok) {
        for (int p = 0; p < planes_q; ++p) dgq += a.part_q[(size_t)p * a.plane + i];
        for (int p = 0; p < planes_v; ++p) {
            dgk += a.part_k[(size_t)p * a.plane + i];
            db += a.part_b[(size_t)p * a.plane + i];
        }
        gq = a.gq[i];
        gk = a.gk[i];
        dbeta[i] = db;
        e[i] = gq * dgq - gk * dgk;
    }
    sx[tid] = gq * dgq;
    __syncthreads();
    if (ok) {
        float dot = 0.f;
        for (int j = 0; j < H; ++j) dot += sx[lr * H + j];
        dql[i] = gq * (dgq - dot);
    }
    __syncthreads();
    if (!dkl) return;
    sx[tid] = gk * dgk;
    __syncthreads();
    if (ok) {
        float dot = 0.f;
        for (int j = 0; j < H; ++j) dot += sx[lr * H + j];
        dkl[i] = gk * (dgk - dot);
    }
}

// dlog_decay[b,t,h] = <d_final, S_T>[b,h] + sum_{s >= t} e[b,s,h], in spans of 2 * kEw tokens.  With anchors
// (phi != null) the sum restarts at every span boundary from the exact value there, the sum over `planes` partials
// of <X, S> entering that token, so the spans are independent: grid (B * H, spans).  Without, one workgroup per
// (b, h) takes the spans from the last to the first: grid (B * H, 1).
constexpr int kSpan = 2 * kEw;
static_assert(kSpan == kGdnAnchor, "one span of the scan per anchor interval");
__global__ __launch_bounds__(kEw) void gdn_bwd_decay_scan_kernel(const float* e, const float* corr, int planes, int B,
                                                                 int Ttot, int H, const int* cu, const float* phi,
                                                                 float* dld) {
    __shared__ float sx[kEw];
    const int bh = blockIdx.x, b = bh / H, h = bh % H, tid = threadIdx.x;
    int T = Ttot;
    size_t tok0 = (size_t)b * Ttot;
    if (cu) {
        const int start = min(max(cu[b], 0), Ttot), end = min(max(cu[b + 1], start), Ttot);
        T = end - start;
        tok0 = (size_t)start;
    }
    const float* src = e + tok0 * H + h;
    float* dst = dld + tok0 * H + h;
    float carry = 0.f;  // the value at the end of the span in hand
    if (corr)
        for (int p = 0; p < planes; ++p) carry += corr[(size_t)p * B * H + bh];
    const int nspan = (T + kSpan - 1) / kSpan;
    const int first = phi ? (int)blockIdx.y : 0, last = phi ? (int)blockIdx.y : nspan - 1;
    if (first >= nspan) return;
    for (int m = last; m >= first; --m) {
        const int t0 = m * kSpan + 2 * tid;
        const float v0 = t0 < T ? src[(size_t)t0 * H] : 0.f, v1 = t0 + 1 < T ? src[(size_t)(t0 + 1) * H] : 0.f;
        if (phi && m < nspan - 1) {
            const size_t aid = (tok0 + (size_t)(m + 1) * kSpan) / kGdnAnchor;
            carry = 0.f;
            for (int p = 0; p < planes; ++p) carry += phi[(aid * H + h) * (size_t)planes + p];
        }
        sx[tid] = v0 + v1;
        __syncthreads();
        float run = carry, total = 0.f;
        for (int j = 0; j < kEw; ++j) {
            const float x = sx[j];
            total += x;
            if (j > tid) run += x;
        }
        if (t0 + 1 < T) dst[(size_t)(t0 + 1) * H] = run + v1;
        if (t0 < T) dst[(size_t)t0 * H] = run + v1 + v0;
        carry += total;
        __syncthreads();
    }
}

__global__ __launch_bounds__(kEw) void gdn_bwd_pass_state_kernel(const f4* src, f4* dst, size_t count) {
    const size_t i = (size_t)blockIdx.x * kEw + threadIdx.x;
    if (i < count) dst[i] = src ? src[i] : f4{0.f, 0.f, 0.f, 0.f};
}

size_t round4(size_t n) { return (n + 3) & ~(size_t)3; }

template <typename K>
bool allow_lds(K kernel, int lds) {
    if (hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds) == hipSuccess)
        return true;
    (void)hipGetLastError();
    return false;
}

template <class E, int DK, int DV>
int launch_sweeps(const GArgs& a, hipStream_t stream) {
    constexpr int lds1 = 2 * 4 * (kChunk * DK + kChunk * kSlice + kScal * kChunk);
    constexpr int lds2 = 2 * 4 * (2 * kChunk * DK + 3 * kChunk * kSlice + kScal * kChunk);
    constexpr int lds3 = 2 * 4 * (3 * kChunk * DV + 3 * kChunk * kSlice + kScal * kChunk);
    static_assert(lds1 <= 160 * 1024 && lds2 <= 160 * 1024 && lds3 <= 160 * 1024, "fits the LDS of a compute unit");
    // once per device and instantiation (bit d = done on device d); not a stream operation
    static std::atomic<uint64_t> configured{0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();
        return SLA_ERR_HIP;
    }
    if (!((configured.load(std::memory_order_acquire) >> dev) & 1u)) {
        if (!allow_lds(gdn_bwd_state_kernel<E, DK, DV>, lds1) || !allow_lds(gdn_bwd_cotangent_kernel<E, DK, DV>, lds2) ||
            !allow_lds(gdn_bwd_key_kernel<E, DK, DV, false>, lds3) || !allow_lds(gdn_bwd_key_kernel<E, DK, DV, true>, lds3))
            return SLA_ERR_HIP;
        configured.fetch_or(uint64_t(1) << dev, std::memory_order_release);
    }
    const unsigned bh = (unsigned)(a.B * a.H);
    const dim3 block(kThreads);
    auto grid = [bh](unsigned slices) { return dim3(((bh + 7u) / 8u) * 8u * slices); };  // see where()
    hipLaunchKernelGGL((gdn_bwd_state_kernel<E, DK, DV>), grid(DV / kSlice), block, (size_t)lds1, stream, a);
    hipLaunchKernelGGL((gdn_bwd_cotangent_kernel<E, DK, DV>), grid(DV / kSlice), block, (size_t)lds2, stream, a);
    hipLaunchKernelGGL((gdn_bwd_key_kernel<E, DK, DV, false>), grid(DK / kSlice), block, (size_t)lds3, stream, a);
    hipLaunchKernelGGL((gdn_bwd_key_kernel<E, DK, DV, true>), grid(DK / kSlice), block, (size_t)lds3, stream, a);
    return hipGetLastError() == hipSuccess ? SLA_OK : SLA_ERR_HIP;
}

template <class E, int DK>
int launch_dv(const GArgs& a, int dv, hipStream_t stream) {
    switch (dv) {
        case 64: return launch_sweeps<E, DK, 64>(a, stream);
        case 128: return launch_sweeps<E, DK, 128>(a, stream);
        case 256: return launch_sweeps<E, DK, 256>(a, stream);
        default: return SLA_ERR_UNSUPPORTED;
    }
}

}  // namespace

// Workspace, in floats: gates 2 [B,T,H]; dk/8 partial planes of dG^Q, dv/8 each of dG^K and dbeta; the decay scalar
// [B,T,H]; dk/8 planes of <d_final, S_T> [B,H]; res and w [B,T,H,dv]; the first part of dk [B,T,H,dk].
size_t backward_gdn_workspace_floats(const sla_params& p, bool packed) {
    const size_t rows = packed ? (size_t)p.T : (size_t)p.B * p.T, n = round4(rows * p.H);
    if (p.dtype == SLA_BF16) {  // block form: a plane per 16 columns; the sweeps' own workspace behind them
        const size_t pv = (size_t)p.dv / 16, pk = (size_t)p.dk / 16, na = gdn_anchor_count(rows);
        return n * (3 + 2 * pv + pk) + round4(pk * p.B * p.H) + round4(na * p.H * pk) + na * p.H * p.dk * p.dv +
               gdn_block_workspace_floats(p.B, p.T, p.H, p.dk, p.dv, packed);
    }
    const size_t pv = (size_t)p.dv / (4 * CW), pk = (size_t)p.dk / (4 * CW);  // planes per compute wave and slice
    return n * (3 + 2 * pv + pk) + round4(pk * p.B * p.H) + 2 * round4(rows * p.H * p.dv) + round4(rows * p.H * p.dk);
}

int launch_backward_gdn(const sla_params& p, const void* q, const void* k, const void* v, const float* ql,
                        const float* kl, const float* ld, const float* beta, const float* s0, const void* dout,
                        const float* dsf, void* dq, void* dk, void* dv, float* dql, float* dkl, float* dld,
                        float* dbeta, float* ds0, float* ws, const int* cu, hipStream_t stream) {
    const size_t rows = cu ? (size_t)p.T : (size_t)p.B * p.T, n = round4(rows * p.H);
    const bool block_form = p.dtype == SLA_BF16;  // bf16: block form on the matrix cores; fp32: token by token
    // partial planes: one per compute wave and slice
    const int pv = block_form ? p.dv / 16 : p.dv / (4 * CW), pk = block_form ? p.dk / 16 : p.dk / (4 * CW);
    if (rows == 0) {
        if (ds0 && p.B > 0) {  // no tokens: the cotangent of the final state is that of the initial state
            const size_t count = (size_t)p.B * p.H * p.dk * p.dv / 4;
            hipLaunchKernelGGL(gdn_bwd_pass_state_kernel, dim3((unsigned)((count + kEw - 1) / kEw)), dim3(kEw), 0,
                               stream, (const f4*)dsf, (f4*)ds0, count);
            if (hipGetLastError() != hipSuccess) return SLA_ERR_HIP;
        }
        return SLA_OK;
    }
    GArgs a;
    a.q = q; a.k = k; a.v = v; a.dout = dout;
    a.ld = ld; a.beta = beta; a.s0 = s0; a.dsf = dsf;
    a.dq = dq; a.dk = dk; a.dv = dv; a.ds0 = ds0;
    float* w = ws;
    float* gq = w; w += n;
    float* gk = w; w += n;
    float* e = w; w += n;
    a.gq = gq; a.gk = gk;
    a.part_q = w; w += n * pk;
    a.part_k = w; w += n * pv;
    a.part_b = w; w += n * pv;
    a.corr = w; w += round4((size_t)pk * p.B * p.H);
    float* anchor_phi = nullptr;
    float* anchor_x = nullptr;
    if (block_form) {  // the exact decay gradient every 512 tokens
        const size_t na = gdn_anchor_count(rows);
        anchor_phi = w; w += round4(na * p.H * pk);
        anchor_x = w; w += na * p.H * p.dk * p.dv;
    }
    a.res = w; w += round4(rows * p.H * p.dv);
    a.w = w; w += round4(rows * p.H * p.dv);
    a.dk1 = w;
    a.plane = n;
    a.rows = rows;
    a.cu = cu;
    a.B = p.B; a.T = p.T; a.H = p.H;

    int rc = launch_bwd_gates(ql, kl, gq, gk, rows, p.H, stream);
    if (rc != SLA_OK) return rc;
    if (block_form) {
        GdnBlockArgs g;
        g.q = (const uint16_t*)q; g.k = (const uint16_t*)k; g.v = (const uint16_t*)v; g.dout = (const uint16_t*)dout;
        g.ld = ld; g.beta = beta; g.gq = gq; g.gk = gk; g.s0 = s0; g.dsf = dsf;
        g.dq = (uint16_t*)dq; g.dk = (uint16_t*)dk; g.dv = (uint16_t*)dv; g.ds0 = ds0;
        g.part_q = a.part_q; g.part_k = a.part_k; g.part_b = a.part_b; g.corr = a.corr;
        g.anchor_x = anchor_x; g.anchor_phi = anchor_phi;
        g.plane = n;
        g.block_ws = a.res;  // everything behind the planes
        g.rows = rows; g.cu = cu;
        g.B = p.B; g.T = p.T; g.H = p.H; g.dim_k = p.dk; g.dim_v = p.dv;
        rc = launch_gdn_block_sweeps(g, stream);
    } else {
        rc = p.dk == 64 ? launch_dv<float, 64>(a, p.dv, stream) : launch_dv<float, 128>(a, p.dv, stream);
    }
    if (rc != SLA_OK) return rc;
    const unsigned per = kEw / (unsigned)p.H, eg = (unsigned)((rows + per - 1) / per);
    hipLaunchKernelGGL(gdn_bwd_finish_kernel, dim3(eg), dim3(kEw), 0, stream, a, pk, pv, dql, kl ? dkl : nullptr,
                       dbeta, e);
    const unsigned spans = anchor_phi ? (unsigned)((p.T + kSpan - 1) / kSpan) : 1u;
    hipLaunchKernelGGL(gdn_bwd_decay_scan_kernel, dim3((unsigned)(p.B * p.H), spans), dim3(kEw), 0, stream, (const float*)e,
                       dsf ? (const float*)a.corr : nullptr, pk, p.B, p.T, p.H, cu, (const float*)anchor_phi, dld);
    return hipGetLastError() == hipSuccess ? SLA_OK : SLA_ERR_HIP;
}

}  // namespace sla
