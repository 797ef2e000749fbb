// Backward pass of sla_forward for the RetNet and GLA recurrences (Sec. 5.1) with SLA's head gates (Eq. 4-6), fp32
// tensors: every product in fp32 vector arithmetic, token by token, so that the gradients agree with an fp64
// evaluation to fp32 rounding.  (bf16 tensors take the block form on the matrix cores in sla_backward.hip.)
//
// Forward step, per head:  S_t = diag(alpha_t) S_{t-1} + G^K_t k_t^T v_t,  out_t = G^Q_t q_t S_t,  alpha_t =
// exp(log_decay_t) (GLA: one factor per key dimension and token; RetNet: one constant per head).  With X_t the
// gradient with respect to S_t including token t's own read-out term:
//     X_t = diag(alpha_{t+1}) X_{t+1} + q_t^T (G^Q_t dout_t)
//     dv_t = G^K_t k_t X_t         dG^K_t = v_t . (k_t X_t)
//     dk_t = G^K_t v_t X_t^T       dq_t = G^Q_t dout_t S_t^T       dG^Q_t = q_t . (dout_t S_t^T)
//     dlog_decay_t = rowsum(X_T' * S_T) + sum_{s >= t} (q_s * dq_s - k_s * dk_s)     (GLA; X_T' the caller's cotangent
//     of the final state; a writer j and a reader s contribute the same amount to q_s dq_s and to k_j dk_j and cross
//     token t's decay exactly when j < t <= s)
// Every output contracts a state over one of its two dimensions, so the pass is three sweeps that each carry one
// state tile in registers, sliced over the dimension that is not contracted:
//   dv sweep, backward in time, X[dk rows, 64 value columns]:  dv, partial dG^K, d_initial_state;
//   dq sweep, forward in time, S^T[dv rows, 64 key columns]:   dq, partial dG^Q, rowsum(X_T' * S_T);
//   dk sweep, backward in time, X^T[dv rows, 64 key columns]:  dk, dlog_decay (a running sum in fp64 per key column).
// The gate gradients then go through the head softmax in sla_bwd_logits_kernel (sla_backward.hip).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "sla.h"
#include "sla_token_sweep.h"

namespace sla {

int launch_bwd_gates(const float* ql, const float* kl, float* gq, float* gk, size_t rows, int H, hipStream_t stream);
int launch_bwd_logits(const float* g, const float* part, int planes, size_t plane, float* dl, size_t rows, int H,
                      const int* cu, int B, hipStream_t stream);

namespace {

using namespace tok;

struct FArgs {
    const float* q;        // [B,T,H,dk] (head-major: [B,H,T,dk])
    const float* k;
    const float* v;        // [B,T,H,dv]
    const float* dout;
    const float* ld;       // GLA: log-decay, laid out like q; else null
    const float* ld_head;  // RetNet: [H]; else null
    const float* gq;       // gates [B,T,H]
    const float* gk;
    const float* s0;       // [B,H,dk,dv] or null
    const float* dsf;
    float* dq;
    float* dk;
    float* dv;
    float* dld;            // GLA: laid out like q
    float* ds0;
    float* part_q;         // [dk/8][plane]: partial q . (dout S^T)
    float* part_k;         // [dv/8][plane]: partial v . (k X)
    float* corr;           // GLA: [B,H,dk] rowsum(X_T' * S_T)
    size_t plane;          // floats between partial planes (>= rows * H)
    size_t rows;           // tokens in all
    const int* cu;         // packed batch (see Where), else null
    int B, T, H;
    bool head_major;
};

constexpr int kSc = 4;  // per-token scalars {G^Q, G^K, alpha of the head (RetNet; 1 for GLA), -}

// Where a head's rows start and how far tokens are apart, for a tensor of row width D.
struct Rows {
    size_t base, step;
};
__device__ __forceinline__ Rows rows_of(const FArgs& a, const Where& me, int D) {
    if (a.head_major) return Rows{((size_t)me.bh * a.T) * D, (size_t)D};
    return Rows{(me.tok0 * a.H + me.h) * D, (size_t)a.H * D};
}

// The decay factors of 16 tokens: staged like any fp32 tensor, written as exp(x); a token past the end gets 1.
template <int NC>
struct RegsA : RegsF<NC> {
    typedef RegsF<NC> Base;
    __device__ __forceinline__ f4 factor(int n, bool ok) const {
        const f4 x = this->x[n];
        return ok ? f4{__builtin_amdgcn_exp2f(x[0] * kLog2e), __builtin_amdgcn_exp2f(x[1] * kLog2e),
                       __builtin_amdgcn_exp2f(x[2] * kLog2e), __builtin_amdgcn_exp2f(x[3] * kLog2e)}
                  : f4{1.f, 1.f, 1.f, 1.f};
    }
    __device__ __forceinline__ void put_exp(float* dst, int t0, int T, int lt) const {
#pragma unroll
        for (int n = 0; n < Base::N; ++n) {
            const int it = lt + kLoaders * n, tok = it / (NC / 4), c4 = it % (NC / 4);
            if (it < Base::items) *(f4*)(dst + tok * NC + 4 * c4) = factor(n, t0 + tok < T);
        }
    }
    __device__ __forceinline__ void put_rows_exp(float* dst, int t0, int T, int lt) const {
#pragma unroll
        for (int n = 0; n < Base::N; ++n) {
            const int it = lt + kLoaders * n, tok = it / (NC / 4), c4 = it % (NC / 4);
            if (it < Base::items) *(f4*)(dst + tok * NC + row_slot<NC / 16>(4 * c4)) = factor(n, t0 + tok < T);
        }
    }
};

struct RegsG {  // the gates of 16 tokens (lanes 0..15 of the first loader wave)
    float gq, gk;
    __device__ __forceinline__ void load(const FArgs& a, size_t tok0, int h, int t0, int T, int lt) {
        const size_t i = (tok0 + (size_t)min(t0 + (lt & (kChunk - 1)), T - 1)) * a.H + h;
        gq = a.gq[i]; gk = a.gk[i];
    }
    __device__ __forceinline__ void put(float* dst, float head_alpha, int t0, int T, int lt) const {
        if (lt < kChunk) {
            const bool ok = t0 + lt < T;
            *(f4*)(dst + kSc * lt) = ok ? f4{gq, gk, head_alpha, 0.f} : f4{0.f, 0.f, 1.f, 0.f};
        }
    }
};

__device__ __forceinline__ float head_alpha_of(const FArgs& a, int h) {
    return a.ld_head ? __builtin_amdgcn_exp2f(a.ld_head[h] * kLog2e) : 1.f;
}

// ------------------------------------------------------------------------------------------------------------
// dv sweep: backward in time, X[dk rows, value columns].
// ------------------------------------------------------------------------------------------------------------
template <bool GLA, int DK, int DV>
__global__ __launch_bounds__(kThreads) void sla_bwd32_dv_kernel(const FArgs a) {
    constexpr int RT = DK / 16;
    constexpr int oK = 0, oQ = oK + kChunk * DK, oA = oQ + kChunk * DK, oV = oA + (GLA ? kChunk * DK : 0),
                  oDO = oV + kChunk * kSlice, oSC = oDO + kChunk * kSlice, kBuf = oSC + kSc * kChunk;
    extern __shared__ __align__(16) unsigned char smem[];
    float* lds = (float*)smem;
    const Where me = where(a, DV / kSlice);
    if (me.bh < 0) return;
    const int T = me.T, nch = (T + kChunk - 1) / kChunk;
    const Rows rk = rows_of(a, me, DK), rv = rows_of(a, me, DV);
    if (me.wave >= kWaves) {  // step c of the sweep covers tokens (nch - 1 - c) * 16 ...
        const int lt = me.tid - 64 * kWaves;
        const float ha = head_alpha_of(a, me.h);
        for (int c = 0; c <= nch; ++c) {
            if (c < nch) {
                const int t0 = (nch - 1 - c) * kChunk;
                float* buf = lds + (c & 1) * kBuf;
                RegsF<DK> xk, xq;
                RegsA<DK> xa;
                RegsF<kSlice> xv, xd;
                RegsG xs;
                xk.load(a.k + rk.base, rk.step, t0, T, lt); xq.load(a.q + rk.base, rk.step, t0, T, lt);
                if constexpr (GLA) xa.load(a.ld + rk.base, rk.step, t0, T, lt);
                xv.load(a.v + rv.base + me.slice * kSlice, rv.step, t0, T, lt);
                xd.load(a.dout + rv.base + me.slice * kSlice, rv.step, t0, T, lt);
                xs.load(a, me.tok0, me.h, t0, T, lt);
                xk.put_rows(buf + oK, t0, T, lt); xq.put_rows(buf + oQ, t0, T, lt);
                if constexpr (GLA) xa.put_rows_exp(buf + oA, t0, T, lt);
                xv.put(buf + oV, t0, T, lt); xd.put(buf + oDO, t0, T, lt);
                xs.put(buf + oSC, ha, t0, T, lt);
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
#pragma unroll 4
        for (int i = kChunk - 1; i >= 0; --i) {
            const f4 sc = *(const f4*)(buf + oSC + kSc * i);
            const float gq = sc[0], gk = sc[1], ha = sc[2];
            float kf[RT], qf[RT], af[RT];
            get_rows<RT>(kf, buf + oK + i * DK + me.rg * 4);
            get_rows<RT>(qf, buf + oQ + i * DK + me.rg * 4);
            if constexpr (GLA) get_rows<RT>(af, buf + oA + i * DK + me.rg * 4);
            const int lc = i * kSlice + me.lcol;
            const fc vv = *(const fc*)(buf + oV + lc), dd = *(const fc*)(buf + oDO + lc);
            float du[CW] = {};
#pragma unroll
            for (int r = 0; r < RT; ++r)
#pragma unroll
                for (int j = 0; j < CW; ++j) {
                    X[r][j] += qf[r] * (gq * dd[j]);
                    du[j] += kf[r] * X[r][j];
                    X[r][j] *= GLA ? af[r] : ha;
                }
            float pk = 0.f;
#pragma unroll
            for (int j = 0; j < CW; ++j) {
                du[j] = row_all(du[j]);
                pk += du[j] * vv[j];
            }
            pk = all_groups(pk);
            const int t = (nch - 1 - c) * kChunk + i;
            if (t < T) {
                if (me.lane == 0)
                    a.part_k[(size_t)(me.slice * kWaves + me.wave) * a.plane + (me.tok0 + t) * a.H + me.h] = pk;
                if (me.rg == 0) *(fc*)(a.dv + rv.base + (size_t)t * rv.step + me.col) = fc{gk * du[0], gk * du[1]};
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
// dq sweep (FWD: forward in time, S^T) and dk sweep (backward in time, X^T): rows are the dv value columns, a
// workgroup owns 64 key columns.  Tile element [r][j]: value column rg * RT + r, key column col + j.
//   FWD:   S^T = S^T diag(alpha) + (G^K v)^T k;   dq' = dout S^T;   dq = G^Q dq'
//   else:  X^T += (G^Q dout)^T q;   dk = G^K v X^T;   run += q dq - k dk;   X^T = X^T diag(alpha)
// ------------------------------------------------------------------------------------------------------------
template <bool GLA, int DK, int DV, bool FWD>
__global__ __launch_bounds__(kThreads) void sla_bwd32_key_kernel(const FArgs a) {
    constexpr int RT = DV / 16;
    constexpr bool NEED_DQ = GLA && !FWD;
    constexpr int oDO = 0, oV = oDO + kChunk * DV, oK = oV + kChunk * DV, oQ = oK + kChunk * kSlice,
                  oA = oQ + kChunk * kSlice, oDQ = oA + (GLA ? kChunk * kSlice : 0),
                  oSC = oDQ + (NEED_DQ ? kChunk * kSlice : 0), kBuf = oSC + kSc * kChunk;
    extern __shared__ __align__(16) unsigned char smem[];
    float* lds = (float*)smem;
    const Where me = where(a, DK / kSlice);
    if (me.bh < 0) return;
    const int T = me.T, nch = (T + kChunk - 1) / kChunk;
    const Rows rk = rows_of(a, me, DK), rv = rows_of(a, me, DV);
    if (me.wave >= kWaves) {
        const int lt = me.tid - 64 * kWaves;
        const float ha = head_alpha_of(a, me.h);
        const size_t ks = rk.base + me.slice * kSlice;
        for (int c = 0; c <= nch; ++c) {
            if (c < nch) {
                const int t0 = (FWD ? c : nch - 1 - c) * kChunk;
                float* buf = lds + (c & 1) * kBuf;
                RegsF<DV> xd, xv;
                RegsF<kSlice> xk, xq, xg;
                RegsA<kSlice> xa;
                RegsG xs;
                xd.load(a.dout + rv.base, rv.step, t0, T, lt); xv.load(a.v + rv.base, rv.step, t0, T, lt);
                xk.load(a.k + ks, rk.step, t0, T, lt); xq.load(a.q + ks, rk.step, t0, T, lt);
                if constexpr (GLA) xa.load(a.ld + ks, rk.step, t0, T, lt);
                if constexpr (NEED_DQ) xg.load(a.dq + ks, rk.step, t0, T, lt);
                xs.load(a, me.tok0, me.h, t0, T, lt);
                xd.put_rows(buf + oDO, t0, T, lt); xv.put_rows(buf + oV, t0, T, lt);
                xk.put(buf + oK, t0, T, lt); xq.put(buf + oQ, t0, T, lt);
                if constexpr (GLA) xa.put_exp(buf + oA, t0, T, lt);
                if constexpr (NEED_DQ) xg.put(buf + oDQ, t0, T, lt);
                xs.put(buf + oSC, ha, t0, T, lt);
            }
            __syncthreads();
        }
        return;
    }
    float M[RT][CW];
    const float* init = FWD ? a.s0 : a.dsf;
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int j = 0; j < CW; ++j)
            M[r][j] = init ? init[((size_t)me.bh * DK + me.col + j) * DV + me.rg * RT + r] : 0.f;
    double run[CW] = {0.0, 0.0};  // dk sweep of GLA: rowsum(X_T' * S_T) + the sum of q dq - k dk over the tokens behind
    if constexpr (NEED_DQ) {
#pragma unroll
        for (int j = 0; j < CW; ++j) run[j] = (double)a.corr[(size_t)me.bh * DK + me.col + j];
    }
    __syncthreads();
    for (int c = 0; c < nch; ++c) {
        const float* buf = lds + (c & 1) * kBuf;
#pragma unroll 4
        for (int ii = 0; ii < kChunk; ++ii) {
            const int i = FWD ? ii : kChunk - 1 - ii;
            const f4 sc = *(const f4*)(buf + oSC + kSc * i);
            const float gq = sc[0], gk = sc[1], ha = sc[2];
            float dd[RT], vv[RT];
            get_rows<RT>(dd, buf + oDO + i * DV + me.rg * 4);
            get_rows<RT>(vv, buf + oV + i * DV + me.rg * 4);
            const int lc = i * kSlice + me.lcol;
            const fc kf = *(const fc*)(buf + oK + lc), qf = *(const fc*)(buf + oQ + lc);
            fc al = fc{ha, ha};
            if constexpr (GLA) al = *(const fc*)(buf + oA + lc);
            const int t = (FWD ? c : nch - 1 - c) * kChunk + i;
            const size_t at = rk.base + (size_t)min(t, max(T - 1, 0)) * rk.step + me.col;
            float y[CW] = {};
            if constexpr (FWD) {
#pragma unroll
                for (int r = 0; r < RT; ++r)
#pragma unroll
                    for (int j = 0; j < CW; ++j) {
                        M[r][j] = M[r][j] * al[j] + (gk * vv[r]) * kf[j];
                        y[j] += dd[r] * M[r][j];
                    }
                float pq = 0.f;
#pragma unroll
                for (int j = 0; j < CW; ++j) {
                    y[j] = row_all(y[j]);  // before the read gate: dG^Q = q . dq'
                    pq += qf[j] * y[j];
                }
                pq = all_groups(pq);
                if (t < T) {
                    if (me.lane == 0)
                        a.part_q[(size_t)(me.slice * kWaves + me.wave) * a.plane + (me.tok0 + t) * a.H + me.h] = pq;
                    if (me.rg == 0) *(fc*)(a.dq + at) = fc{gq * y[0], gq * y[1]};
                }
            } else {
#pragma unroll
                for (int r = 0; r < RT; ++r)
#pragma unroll
                    for (int j = 0; j < CW; ++j) {
                        M[r][j] += (gq * dd[r]) * qf[j];
                        y[j] += vv[r] * M[r][j];
                        M[r][j] *= al[j];
                    }
                fc dk;
#pragma unroll
                for (int j = 0; j < CW; ++j) dk[j] = gk * row_all(y[j]);
                if constexpr (NEED_DQ) {
                    const fc dqf = *(const fc*)(buf + oDQ + lc);
#pragma unroll
                    for (int j = 0; j < CW; ++j) run[j] += (double)qf[j] * (double)dqf[j] - (double)kf[j] * (double)dk[j];
                }
                if (t < T && me.rg == 0) {
                    *(fc*)(a.dk + at) = dk;
                    if constexpr (NEED_DQ) *(fc*)(a.dld + at) = fc{(float)run[0], (float)run[1]};
                }
            }
        }
        __syncthreads();
    }
    if constexpr (FWD && GLA) {  // rowsum(X_T' * S_T) for this lane's key columns
        float s[CW] = {};
        if (a.dsf) {
#pragma unroll
            for (int r = 0; r < RT; ++r)
#pragma unroll
                for (int j = 0; j < CW; ++j)
                    s[j] += a.dsf[((size_t)me.bh * DK + me.col + j) * DV + me.rg * RT + r] * M[r][j];
        }
#pragma unroll
        for (int j = 0; j < CW; ++j) s[j] = row_all(s[j]);
        if (me.rg == 0) *(fc*)(a.corr + (size_t)me.bh * DK + me.col) = fc{s[0], s[1]};
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

template <bool GLA, int DK, int DV>
int launch_sweeps(const FArgs& a, bool state_only, hipStream_t stream) {
    constexpr int ldsV = 2 * 4 * ((GLA ? 3 : 2) * kChunk * DK + 2 * kChunk * kSlice + kSc * kChunk);
    constexpr int ldsQ = 2 * 4 * (2 * kChunk * DV + (GLA ? 3 : 2) * kChunk * kSlice + kSc * kChunk);
    constexpr int ldsK = 2 * 4 * (2 * kChunk * DV + (GLA ? 4 : 2) * kChunk * kSlice + kSc * kChunk);
    static_assert(ldsV <= 160 * 1024 && ldsQ <= 160 * 1024 && ldsK <= 160 * 1024, "fits the LDS of a compute unit");
    // once per device and instantiation (bit d = done on device d); not a stream operation
    static std::atomic<uint64_t> configured{0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();
        return SLA_ERR_HIP;
    }
    if (!((configured.load(std::memory_order_acquire) >> dev) & 1u)) {
        if (!allow_lds(sla_bwd32_dv_kernel<GLA, DK, DV>, ldsV) ||
            !allow_lds(sla_bwd32_key_kernel<GLA, DK, DV, true>, ldsQ) ||
            !allow_lds(sla_bwd32_key_kernel<GLA, DK, DV, false>, ldsK))
            return SLA_ERR_HIP;
        configured.fetch_or(uint64_t(1) << dev, std::memory_order_release);
    }
    const unsigned bh = (unsigned)(a.B * a.H);
    const dim3 block(kThreads);
    auto grid = [bh](unsigned slices) { return dim3(((bh + 7u) / 8u) * 8u * slices); };  // see tok::where()
    hipLaunchKernelGGL((sla_bwd32_dv_kernel<GLA, DK, DV>), grid(DV / kSlice), block, (size_t)ldsV, stream, a);
    if (!state_only) {
        hipLaunchKernelGGL((sla_bwd32_key_kernel<GLA, DK, DV, true>), grid(DK / kSlice), block, (size_t)ldsQ, stream, a);
        hipLaunchKernelGGL((sla_bwd32_key_kernel<GLA, DK, DV, false>), grid(DK / kSlice), block, (size_t)ldsK, stream, a);
    }
    return hipGetLastError() == hipSuccess ? SLA_OK : SLA_ERR_HIP;
}

template <bool GLA, int DK>
int launch_dv(const FArgs& a, int dv, bool state_only, hipStream_t stream) {
    switch (dv) {
        case 64: return launch_sweeps<GLA, DK, 64>(a, state_only, stream);
        case 128: return launch_sweeps<GLA, DK, 128>(a, state_only, stream);
        case 256: return launch_sweeps<GLA, DK, 256>(a, state_only, stream);
        default: return SLA_ERR_UNSUPPORTED;
    }
}

template <bool GLA>
int launch_dk(const FArgs& a, int dk, int dv, bool state_only, hipStream_t stream) {
    switch (dk) {
        case 64: return launch_dv<GLA, 64>(a, dv, state_only, stream);
        case 128: return launch_dv<GLA, 128>(a, dv, state_only, stream);
        default: return SLA_ERR_UNSUPPORTED;
    }
}

}  // namespace

// Workspace, in floats: gates 2 [B,T,H]; dk/8 partial planes of dG^Q and dv/8 of dG^K (one per compute wave and
// slice); for GLA rowsum(X_T' * S_T) [B,H,dk].
size_t backward_f32_workspace_floats(const sla_params& p, bool packed) {
    const size_t rows = packed ? (size_t)p.T : (size_t)p.B * p.T, n = round4(rows * p.H);
    return n * (2 + (size_t)p.dk / (4 * CW) + (size_t)p.dv / (4 * CW)) +
           (p.variant == SLA_GLA ? round4((size_t)p.B * p.H * p.dk) : 0);
}

int launch_backward_f32(const sla_params& p, const void* q, const void* k, const void* v, const float* ql,
                        const float* kl, const void* ld, const float* s0, const void* dout, const float* dsf, void* dq,
                        void* dk, void* dv, float* dql, float* dkl, void* dld, float* ds0, float* ws, const int* cu,
                        hipStream_t stream) {
    const size_t rows = cu ? (size_t)p.T : (size_t)p.B * p.T, n = round4(rows * p.H);
    const int pq = p.dk / (4 * CW), pv = p.dv / (4 * CW);
    FArgs a;
    a.q = (const float*)q; a.k = (const float*)k; a.v = (const float*)v; a.dout = (const float*)dout;
    a.ld = p.variant == SLA_GLA ? (const float*)ld : nullptr;
    a.ld_head = p.variant == SLA_RETNET ? (const float*)ld : nullptr;
    a.s0 = s0; a.dsf = dsf;
    a.dq = (float*)dq; a.dk = (float*)dk; a.dv = (float*)dv; a.dld = (float*)dld; a.ds0 = ds0;
    float* w = ws;
    float* gq = w; w += n;
    float* gk = w; w += n;
    a.gq = gq; a.gk = gk;
    a.part_q = w; w += n * pq;
    a.part_k = w; w += n * pv;
    a.corr = w;
    a.plane = n; a.rows = rows; a.cu = cu;
    a.B = p.B; a.T = p.T; a.H = p.H;
    a.head_major = (p.flags & SLA_FLAG_HEAD_MAJOR) != 0;
    const bool state_only = rows == 0;  // no tokens: the final state's cotangent is the initial state's
    int rc = launch_bwd_gates(ql, kl, gq, gk, rows, p.H, stream);
    if (rc != SLA_OK) return rc;
    rc = p.variant == SLA_GLA ? launch_dk<true>(a, p.dk, p.dv, state_only, stream)
                              : launch_dk<false>(a, p.dk, p.dv, state_only, stream);
    if (rc != SLA_OK || state_only) return rc;
    rc = launch_bwd_logits(gq, a.part_q, pq, n, dql, rows, p.H, cu, p.B, stream);
    if (rc == SLA_OK && kl) rc = launch_bwd_logits(gk, a.part_k, pv, n, dkl, rows, p.H, cu, p.B, stream);
    return rc;
}

}  // namespace sla
