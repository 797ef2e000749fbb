// C-ABI entry points of libsla: argument validation and dispatch.  All checks that do not need the
// device run first, so a bad call is rejected before any HIP call (and sla_check_args runs them alone).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include <mutex>

#include "sla.h"

namespace sla {
int launch_forward(const sla_params& p, int dvw, int nseg, int seg_len, const void* q, const void* k, const void* v,
                   const float* ql, const float* kl, const void* ld, const float* beta, const float* s0, void* out,
                   float* sT, float* workspace, const int* cu, hipStream_t stream);
size_t segment_workspace_floats(const sla_params& p, int nseg);
size_t backward_workspace_floats(const sla_params& p, bool packed);
int launch_backward(const sla_params& p, const void* q, const void* k, const void* v, const float* ql, const float* kl,
                    const void* ld, const float* s0, const void* dout, const float* dsf, void* dq, void* dk, void* dv,
                    float* dql, float* dkl, void* dld, float* ds0, float* ws, const int* cu, hipStream_t stream);
size_t backward_segment_extra_floats(const sla_params& p, int nseg);
sla_params packed_segments(const sla_params& p, int nseg);
int launch_backward_segments(const sla_params& p, int nseg, int seg_len, int dvw, const void* q, const void* k,
                             const void* v, const float* ql, const float* kl, const void* ld, const float* s0,
                             const void* dout, const float* dsf, void* dq, void* dk, void* dv, float* dql, float* dkl,
                             void* dld, float* ds0, float* ws, hipStream_t stream);
size_t backward_gdn_workspace_floats(const sla_params& p, bool packed);
// any supported key width: heads of width 32 run zero-padded to 64 (sla_backward_narrow.hip)
size_t backward_any_workspace_floats(const sla_params& p, bool packed);
int launch_backward_any(const sla_params& p, const void* q, const void* k, const void* v, const float* ql,
                        const float* kl, const void* ld, const float* s0, const void* dout, const float* dsf, void* dq,
                        void* dk, void* dv, float* dql, float* dkl, void* dld, float* ds0, float* ws, const int* cu,
                        bool packed, hipStream_t stream);
size_t backward_gdn_any_workspace_floats(const sla_params& p, bool packed);
int launch_backward_gdn_any(const sla_params& p, const void* q, const void* k, const void* v, const float* ql,
                            const float* kl, const float* ld, const float* beta, const float* s0, const void* dout,
                            const float* dsf, void* dq, void* dk, void* dv, float* dql, float* dkl, float* dld,
                            float* dbeta, float* ds0, float* ws, const int* cu, bool packed, hipStream_t stream);
int launch_backward_gdn(const sla_params& p, const void* q, const void* k, const void* v, const float* ql,
                        const float* kl, const float* ld, const float* beta, const float* s0, const void* dout,
                        const float* dsf, void* dq, void* dk, void* dv, float* dql, float* dkl, float* dld,
                        float* dbeta, float* ds0, float* ws, const int* cu, hipStream_t stream);
int launch_gate_logits(const sla_params& p, const void* q, const void* k, const float* wq, const float* wk, float* ql,
                       float* kl, int compute_units, hipStream_t stream);
int launch_short_conv_silu(int dtype, int B, int T, int C, int taps, const void* x, const float* w, void* y,
                           hipStream_t stream);
size_t feature_map_partials(int B, int T);
int launch_feature_map(int dtype, int B, int T, int C, int taps, int head_width, float eps, const void* x, const float* w,
                       void* y, hipStream_t stream);
int launch_feature_map_backward(int dtype, int B, int T, int C, int taps, int head_width, float eps, const void* x,
                                const float* w, const void* dy, void* dx, float* dw, float* workspace,
                                hipStream_t stream);
int launch_gate_logits_backward(const sla_params& p, const void* x, const float* w, const float* dl, void* dx, float* dw,
                                float* workspace, hipStream_t stream);
size_t gate_logits_backward_workspace_floats(const sla_params& p);
unsigned int* device_status_word();
int launch_decode(const sla_params& p, const void* q, const void* k, const void* v, const float* ql, const float* kl,
                  const float* wq, const float* wk,
                  const void* ld, const float* beta, float* state, void* out, hipStream_t stream);
}

// Library-owned scratch memory for sla_forward_static: the segment-parallel schedule's workspace for callers that
// cannot allocate.  In host code this name is only a handle for hipGetSymbolAddress; the device address is looked
// up once per device (static_scratch below) and that pointer is what the kernels receive.
static __device__ __align__(256) unsigned char scratch[SLA_STATIC_SCRATCH_BYTES];

// Sticky status word of the device (bits SLA_DEVICE_*), written by the kernels of the other translation units
// through the pointer that device_status_word() hands to their launchers.
static __device__ unsigned int device_status;

namespace {

constexpr int kVersion = 102;  // 0.1.2
constexpr int kMaxHeads = 64;
constexpr int kMaxDevices = 64;

// Device address of a __device__ symbol of this file on the current device (every device holds its own copy at its
// own address); NULL if the runtime refuses.  The first call on a device resolves the symbol; later calls read the
// table.
struct SymbolTable {
    std::mutex lock;
    void* addr[kMaxDevices] = {nullptr};
    template <typename Resolve>
    void* get(Resolve resolve) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
            (void)hipGetLastError();
            return nullptr;
        }
        std::lock_guard<std::mutex> hold(lock);
        if (!addr[dev]) {
            void* ptr = nullptr;
            if (resolve(&ptr) != hipSuccess || !ptr) {
                (void)hipGetLastError();
                return nullptr;
            }
            addr[dev] = ptr;
        }
        return addr[dev];
    }
};

void* static_scratch() {
    static SymbolTable table;
    return table.get([](void** ptr) { return hipGetSymbolAddress(ptr, HIP_SYMBOL(scratch)); });
}

void* status_word() {
    static SymbolTable table;
    return table.get([](void** ptr) { return hipGetSymbolAddress(ptr, HIP_SYMBOL(device_status)); });
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_params(const sla_params* p) {
    if (!p) return SLA_ERR_NULL;
    if (p->variant != SLA_RETNET && p->variant != SLA_GLA && p->variant != SLA_GDN) return SLA_ERR_UNSUPPORTED;
    if (p->dtype != SLA_F32 && p->dtype != SLA_BF16) return SLA_ERR_UNSUPPORTED;
    if ((p->flags & ~SLA_FLAG_HEAD_MAJOR) != 0) return SLA_ERR_UNSUPPORTED;
    if (p->segments < 0 || p->segments > 4096) return SLA_ERR_SHAPE;
    if (p->segments > 1 && p->variant == SLA_GDN) return SLA_ERR_UNSUPPORTED;
    if (p->B < 0 || p->T < 0 || p->H < 1 || p->H > kMaxHeads) return SLA_ERR_SHAPE;
    if (p->dk < 1 || p->dv < 1) return SLA_ERR_SHAPE;
    if ((p->dk != 32 && p->dk != 64 && p->dk != 128) || (p->dv != 64 && p->dv != 128 && p->dv != 256))
        return SLA_ERR_UNSUPPORTED;
    if (p->dv_split != 0) {
        const int s = p->dv_split;
        if (s != 16 && s != 32 && s != 64 && s != 128) return SLA_ERR_SHAPE;
        if (s > p->dv) return SLA_ERR_SHAPE;
        if (s > 64) return SLA_ERR_UNSUPPORTED;
    }
    // index arithmetic in the kernels uses size_t for element offsets but int for token counts
    if ((int64_t)p->B * p->T > (int64_t)1 << 30) return SLA_ERR_SHAPE;
    {
        // the kernels address one batch row through 32-bit byte offsets (buffer descriptors)
        const int64_t es = p->dtype == SLA_BF16 ? 2 : 4;
        const int64_t wide = p->dk > p->dv ? p->dk : p->dv;
        if (((int64_t)p->T + 256) * p->H * wide * es > (int64_t)INT32_MAX) return SLA_ERR_SHAPE;
    }
    return SLA_OK;
}

int check(const sla_params* p, const void* q, const void* k, const void* v, const float* ql, const float* kl,
          const void* ld, const float* beta, const float* s0, const void* out, const float* sT) {
    const int rc = check_params(p);
    if (rc != SLA_OK) return rc;
    const bool empty = (p->B == 0);
    if (!empty && p->T > 0) {
        if (!q || !k || !v || !ql || !ld || !out) return SLA_ERR_NULL;
        if (p->variant == SLA_GDN && !beta) return SLA_ERR_NULL;
    }
    if (p->variant != SLA_GDN && beta) return SLA_ERR_NULL;
    const void* ptrs[] = {q, k, v, ql, kl, ld, beta, s0, out, sT};
    for (const void* x : ptrs)
        if (x && !aligned16(x)) return SLA_ERR_ALIGN;
    return SLA_OK;
}

int device_compute_units() {
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();
        return -1;
    }
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) {
            (void)hipGetLastError();
            return -1;
        }
        cached[dev] = n;
    }
    return cached[dev];
}

constexpr int kMinSegment = 256;  // tokens; shorter segments are not worth a pre-pass

// Segment-parallel schedule (RetNet, GLA): how many segments to cut T into so that, with 64-column
// slices, every compute unit gets a workgroup.  1 = single fused pass.  seg_len is a multiple of 64.
int choose_segments(const sla_params& p, int cus, int* seg_len) {
    *seg_len = p.T;
    if (p.variant == SLA_GDN || p.segments == 1) return 1;
    const int64_t rows = (int64_t)p.B * p.H * (p.dv / (p.dv >= 64 ? 64 : p.dv));
    int want = p.segments > 1 ? p.segments : (int)((cus + rows - 1) / rows);
    if (want <= 1) return 1;
    int len = (p.T + want - 1) / want;
    len = ((len + 63) / 64) * 64;
    if (len < kMinSegment) len = kMinSegment;
    const int nseg = (p.T + len - 1) / len;
    if (nseg <= 1) return 1;
    *seg_len = len;
    return nseg;
}

int choose_dv_split(const sla_params& p, int cus, int nseg = 1) {
    if (p.dv_split != 0) return p.dv_split;
    // The widest slice that still gives every compute unit a workgroup; narrower slices repeat the
    // per-token decay work of a head in more workgroups, so never go narrower than needed.
    const int64_t seqs = (int64_t)p.B * p.H * nseg;
    const int widths[] = {64, 32, 16};
    for (int w : widths) {
        if (w > p.dv) continue;
        if (seqs * (p.dv / w) >= cus) return w;
    }
    return 16;
}

}  // namespace

namespace sla {
unsigned int* device_status_word() { return (unsigned int*)status_word(); }
}

extern "C" {

int sla_check_args(const sla_params* p, const void* q, const void* k, const void* v, const float* q_head_logits,
                   const float* k_head_logits, const void* log_decay, const float* beta, const float* initial_state,
                   const void* out, const float* final_state) {
    return check(p, q, k, v, q_head_logits, k_head_logits, log_decay, beta, initial_state, out, final_state);
}

int sla_forward_ws(const sla_params* p, const void* q, const void* k, const void* v, const float* q_head_logits,
                   const float* k_head_logits, const void* log_decay, const float* beta, const float* initial_state,
                   void* out, float* final_state, void* workspace, size_t workspace_bytes, void* stream) {
    const int rc = check(p, q, k, v, q_head_logits, k_head_logits, log_decay, beta, initial_state, out, final_state);
    if (rc != SLA_OK) return rc;
    if (workspace && !aligned16(workspace)) return SLA_ERR_ALIGN;
    if (p->B == 0) return SLA_OK;
    if (p->T == 0 && !final_state) return SLA_OK;
    int seg_len = p->T;
    if (p->segments > 1) {  // an explicit request does not depend on the device: reject it before any HIP call
        const int n = choose_segments(*p, 1, &seg_len);
        if (n > 1 && (!workspace || sla::segment_workspace_floats(*p, n) * sizeof(float) > workspace_bytes))
            return SLA_ERR_WORKSPACE;
    }
    const int cus = device_compute_units();
    if (cus <= 0) return SLA_ERR_HIP;
    int nseg = choose_segments(*p, cus, &seg_len);
    if (nseg > 1 && (!workspace || sla::segment_workspace_floats(*p, nseg) * sizeof(float) > workspace_bytes)) {
        nseg = 1;  // the library's own choice without room for it: one fused pass
        seg_len = p->T;
    }
    const int dvw = choose_dv_split(*p, cus, nseg);
    return sla::launch_forward(*p, dvw, nseg, seg_len, q, k, v, q_head_logits, k_head_logits, log_decay, beta,
                               initial_state, out, final_state, (float*)workspace, nullptr, (hipStream_t)stream);
}

int sla_init(void) { return (static_scratch() && status_word()) ? SLA_OK : SLA_ERR_HIP; }

int sla_device_status(uint32_t* status, int reset, void* stream) {
    if (!status) return SLA_ERR_NULL;
    void* word = status_word();
    if (!word) return SLA_ERR_HIP;
    hipStream_t st = (hipStream_t)stream;
    uint32_t value = 0;
    if (hipMemcpyAsync(&value, word, sizeof(value), hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess) {
        (void)hipGetLastError();
        return SLA_ERR_HIP;
    }
    if (reset && value != 0) {
        const uint32_t zero = 0;
        if (hipMemcpyAsync(word, &zero, sizeof(zero), hipMemcpyHostToDevice, st) != hipSuccess ||
            hipStreamSynchronize(st) != hipSuccess) {
            (void)hipGetLastError();
            return SLA_ERR_HIP;
        }
    }
    *status = value;
    return SLA_OK;
}

size_t sla_static_scratch_bytes(void) { return SLA_STATIC_SCRATCH_BYTES; }

int sla_forward_static(const sla_params* p, const void* q, const void* k, const void* v, const float* q_head_logits,
                       const float* k_head_logits, const void* log_decay, const float* beta,
                       const float* initial_state, void* out, float* final_state, void* stream) {
    const int rc = check(p, q, k, v, q_head_logits, k_head_logits, log_decay, beta, initial_state, out, final_state);
    if (rc != SLA_OK) return rc;
    if (p->B == 0) return SLA_OK;
    if (p->T == 0 && !final_state) return SLA_OK;
    int seg_len = p->T;
    if (p->segments > 1) {  // an explicit request does not depend on the device: reject it before any HIP call
        const int n = choose_segments(*p, 1, &seg_len);
        if (sla::segment_workspace_floats(*p, n) * sizeof(float) > SLA_STATIC_SCRATCH_BYTES) return SLA_ERR_SCRATCH;
    }
    const int cus = device_compute_units();
    if (cus <= 0) return SLA_ERR_HIP;
    const int nseg = choose_segments(*p, cus, &seg_len);
    if (sla::segment_workspace_floats(*p, nseg) * sizeof(float) > SLA_STATIC_SCRATCH_BYTES) return SLA_ERR_SCRATCH;
    float* ws = nullptr;
    if (nseg > 1) {
        ws = (float*)static_scratch();
        if (!ws) return SLA_ERR_HIP;
    }
    const int dvw = choose_dv_split(*p, cus, nseg);
    return sla::launch_forward(*p, dvw, nseg, seg_len, q, k, v, q_head_logits, k_head_logits, log_decay, beta,
                               initial_state, out, final_state, ws, nullptr, (hipStream_t)stream);
}

int sla_forward_varlen(const sla_params* p, const void* q, const void* k, const void* v, const float* q_head_logits,
                       const float* k_head_logits, const void* log_decay, const float* beta,
                       const int32_t* cu_seqlens, const float* initial_state, void* out, float* final_state,
                       void* stream) {
    const int rc = check(p, q, k, v, q_head_logits, k_head_logits, log_decay, beta, initial_state, out, final_state);
    if (rc != SLA_OK) return rc;
    if (p->segments > 1 || p->flags != 0) return SLA_ERR_UNSUPPORTED;
    if (p->B > 0 && !cu_seqlens) return SLA_ERR_NULL;
    if (cu_seqlens && (reinterpret_cast<uintptr_t>(cu_seqlens) & 3u)) return SLA_ERR_ALIGN;
    if (p->B == 0) return SLA_OK;
    if (p->T == 0 && !final_state) return SLA_OK;
    const int cus = device_compute_units();
    if (cus <= 0) return SLA_ERR_HIP;
    const int dvw = choose_dv_split(*p, cus, 1);
    return sla::launch_forward(*p, dvw, 1, p->T, q, k, v, q_head_logits, k_head_logits, log_decay, beta, initial_state,
                               out, final_state, nullptr, p->T == 0 ? nullptr : cu_seqlens, (hipStream_t)stream);
}

int sla_forward(const sla_params* p, const void* q, const void* k, const void* v, const float* q_head_logits,
                const float* k_head_logits, const void* log_decay, const float* beta, const float* initial_state,
                void* out, float* final_state, void* stream) {
    return sla_forward_ws(p, q, k, v, q_head_logits, k_head_logits, log_decay, beta, initial_state, out, final_state,
                          nullptr, 0, stream);
}

int sla_decode_step(const sla_params* p, const void* q, const void* k, const void* v, const float* q_head_logits,
                    const float* k_head_logits, const void* log_decay, const float* beta, float* state, void* out,
                    void* stream) {
    const int rc = check(p, q, k, v, q_head_logits, k_head_logits, log_decay, beta, state, out, state);
    if (rc != SLA_OK) return rc;
    if (p->T != 1) return SLA_ERR_SHAPE;
    if (p->B == 0) return SLA_OK;
    if (!state) return SLA_ERR_NULL;
    // one token per sequence: [B,1,H,d] and [B,H,1,d] are the same memory, so the layout flag changes nothing
    return sla::launch_decode(*p, q, k, v, q_head_logits, k_head_logits, nullptr, nullptr, log_decay, beta, state, out,
                              (hipStream_t)stream);
}

int sla_decode_step_fused(const sla_params* p, const void* q, const void* k, const void* v, const float* w_gq,
                          const float* w_gk, const void* log_decay, const float* beta, float* state, void* out,
                          void* stream) {
    // w_gq / w_gk take the place of the logits: same rules (w_gq required, w_gk optional, both 16-byte aligned)
    const int rc = check(p, q, k, v, w_gq, w_gk, log_decay, beta, state, out, state);
    if (rc != SLA_OK) return rc;
    if (p->T != 1) return SLA_ERR_SHAPE;
    if (p->B == 0) return SLA_OK;
    if (!state) return SLA_ERR_NULL;
    return sla::launch_decode(*p, q, k, v, nullptr, nullptr, w_gq, w_gk, log_decay, beta, state, out,
                              (hipStream_t)stream);
}

// The backward pass cuts batch rows into segments only on request (p->segments >= 2), so that its workspace size
// does not depend on the device; the cut itself is the forward's.
static int backward_segments(const sla_params& p, bool packed, int* seg_len) {
    *seg_len = p.T;
    if (packed || p.segments < 2 || p.T == 0) return 1;
    return choose_segments(p, 1, seg_len);
}

static size_t backward_floats(const sla_params& p, bool packed) {
    int len = 0;
    const int nseg = backward_segments(p, packed, &len);
    if (nseg <= 1) return sla::backward_any_workspace_floats(p, packed);
    return sla::backward_workspace_floats(sla::packed_segments(p, nseg), true) +
           sla::backward_segment_extra_floats(p, nseg);
}

static int backward_impl(const sla_params* p, const void* q, const void* k, const void* v, const float* q_head_logits,
                         const float* k_head_logits, const void* log_decay, const float* initial_state,
                         const void* d_out, const float* d_final_state, void* dq, void* dk, void* dv,
                         float* dq_head_logits, float* dk_head_logits, void* dlog_decay, float* d_initial_state,
                         void* workspace, size_t workspace_bytes, const int32_t* cu, bool packed, void* stream) {
    int rc = check_params(p);
    if (rc != SLA_OK) return rc;
    if (p->variant == SLA_GDN || (packed && p->flags != 0)) return SLA_ERR_UNSUPPORTED;
    // fp32 tensors and key heads of width 32: the single pass only
    if ((p->dtype == SLA_F32 || p->dk < 64) && p->segments >= 2) return SLA_ERR_UNSUPPORTED;
    if (p->B > 0 && p->T > 0) {
        if (!q || !k || !v || !q_head_logits || !log_decay || !d_out || !dq || !dk || !dv || !dq_head_logits)
            return SLA_ERR_NULL;
        if (p->variant == SLA_GLA && !dlog_decay) return SLA_ERR_NULL;
    }
    if (p->variant == SLA_RETNET && dlog_decay) return SLA_ERR_NULL;
    if ((k_head_logits != nullptr) != (dk_head_logits != nullptr)) return SLA_ERR_NULL;
    if (packed && p->B > 0 && !cu) return SLA_ERR_NULL;
    const void* ptrs[] = {q, k, v, q_head_logits, k_head_logits, log_decay, initial_state, d_out, d_final_state,
                          dq, dk, dv, dq_head_logits, dk_head_logits, dlog_decay, d_initial_state, workspace};
    for (const void* x : ptrs)
        if (x && !aligned16(x)) return SLA_ERR_ALIGN;
    if (cu && (reinterpret_cast<uintptr_t>(cu) & 3u)) return SLA_ERR_ALIGN;
    if (p->B == 0) return SLA_OK;
    if (p->T == 0 && !d_initial_state) return SLA_OK;
    if (!workspace || backward_floats(*p, packed) * sizeof(float) > workspace_bytes) return SLA_ERR_WORKSPACE;
    int seg_len = 0;
    const int nseg = backward_segments(*p, packed, &seg_len);
    if (nseg > 1) {
        if (p->flags != 0) return SLA_ERR_UNSUPPORTED;  // the segments run as a packed batch: [B,T,H,d] only
        return sla::launch_backward_segments(*p, nseg, seg_len, 64, q, k, v, q_head_logits, k_head_logits, log_decay,
                                             initial_state, d_out, d_final_state, dq, dk, dv, dq_head_logits,
                                             dk_head_logits, dlog_decay, d_initial_state, (float*)workspace,
                                             (hipStream_t)stream);
    }
    return sla::launch_backward_any(*p, q, k, v, q_head_logits, k_head_logits, log_decay, initial_state, d_out,
                                    d_final_state, dq, dk, dv, dq_head_logits, dk_head_logits, dlog_decay,
                                    d_initial_state, (float*)workspace, packed && p->T > 0 ? cu : nullptr, packed,
                                    (hipStream_t)stream);
}

int sla_backward(const sla_params* p, const void* q, const void* k, const void* v, const float* q_head_logits,
                 const float* k_head_logits, const void* log_decay, const float* initial_state, const void* d_out,
                 const float* d_final_state, void* dq, void* dk, void* dv, float* dq_head_logits,
                 float* dk_head_logits, void* dlog_decay, float* d_initial_state, void* workspace,
                 size_t workspace_bytes, void* stream) {
    return backward_impl(p, q, k, v, q_head_logits, k_head_logits, log_decay, initial_state, d_out, d_final_state, dq,
                         dk, dv, dq_head_logits, dk_head_logits, dlog_decay, d_initial_state, workspace,
                         workspace_bytes, nullptr, false, stream);
}

int sla_backward_varlen(const sla_params* p, const void* q, const void* k, const void* v, const float* q_head_logits,
                        const float* k_head_logits, const void* log_decay, const int32_t* cu_seqlens,
                        const float* initial_state, const void* d_out, const float* d_final_state, void* dq, void* dk,
                        void* dv, float* dq_head_logits, float* dk_head_logits, void* dlog_decay,
                        float* d_initial_state, void* workspace, size_t workspace_bytes, void* stream) {
    return backward_impl(p, q, k, v, q_head_logits, k_head_logits, log_decay, initial_state, d_out, d_final_state, dq,
                         dk, dv, dq_head_logits, dk_head_logits, dlog_decay, d_initial_state, workspace,
                         workspace_bytes, cu_seqlens, true, stream);
}

static int backward_gdn_impl(const sla_params* p, const void* q, const void* k, const void* v,
                             const float* q_head_logits, const float* k_head_logits, const float* log_decay,
                             const float* beta, const int32_t* cu, bool packed, const float* initial_state,
                             const void* d_out, const float* d_final_state, void* dq, void* dk, void* dv,
                             float* dq_head_logits, float* dk_head_logits, float* dlog_decay, float* dbeta,
                             float* d_initial_state, void* workspace, size_t workspace_bytes, void* stream) {
    const int rc = check_params(p);
    if (rc != SLA_OK) return rc;
    if (p->variant != SLA_GDN || p->flags != 0) return SLA_ERR_UNSUPPORTED;
    if (p->B > 0 && p->T > 0) {
        if (!q || !k || !v || !q_head_logits || !log_decay || !beta || !d_out || !dq || !dk || !dv ||
            !dq_head_logits || !dlog_decay || !dbeta)
            return SLA_ERR_NULL;
    }
    if ((k_head_logits != nullptr) != (dk_head_logits != nullptr)) return SLA_ERR_NULL;
    if (packed && p->B > 0 && !cu) return SLA_ERR_NULL;
    const void* ptrs[] = {q, k, v, q_head_logits, k_head_logits, log_decay, beta, initial_state, d_out,
                          d_final_state, dq, dk, dv, dq_head_logits, dk_head_logits, dlog_decay, dbeta,
                          d_initial_state, workspace};
    for (const void* x : ptrs)
        if (x && !aligned16(x)) return SLA_ERR_ALIGN;
    if (cu && (reinterpret_cast<uintptr_t>(cu) & 3u)) return SLA_ERR_ALIGN;
    if (p->B == 0) return SLA_OK;
    if (p->T == 0 && !d_initial_state) return SLA_OK;
    if (p->T > 0 && (!workspace || sla::backward_gdn_any_workspace_floats(*p, packed) * sizeof(float) > workspace_bytes))
        return SLA_ERR_WORKSPACE;
    return sla::launch_backward_gdn_any(*p, q, k, v, q_head_logits, k_head_logits, log_decay, beta, initial_state,
                                        d_out, d_final_state, dq, dk, dv, dq_head_logits, dk_head_logits, dlog_decay,
                                        dbeta, d_initial_state, (float*)workspace, packed && p->T > 0 ? cu : nullptr,
                                        packed, (hipStream_t)stream);
}

int sla_backward_gdn(const sla_params* p, const void* q, const void* k, const void* v, const float* q_head_logits,
                     const float* k_head_logits, const float* log_decay, const float* beta,
                     const float* initial_state, const void* d_out, const float* d_final_state, void* dq, void* dk,
                     void* dv, float* dq_head_logits, float* dk_head_logits, float* dlog_decay, float* dbeta,
                     float* d_initial_state, void* workspace, size_t workspace_bytes, void* stream) {
    return backward_gdn_impl(p, q, k, v, q_head_logits, k_head_logits, log_decay, beta, nullptr, false, initial_state,
                             d_out, d_final_state, dq, dk, dv, dq_head_logits, dk_head_logits, dlog_decay, dbeta,
                             d_initial_state, workspace, workspace_bytes, stream);
}

int sla_backward_gdn_varlen(const sla_params* p, const void* q, const void* k, const void* v,
                            const float* q_head_logits, const float* k_head_logits, const float* log_decay,
                            const float* beta, const int32_t* cu_seqlens, const float* initial_state,
                            const void* d_out, const float* d_final_state, void* dq, void* dk, void* dv,
                            float* dq_head_logits, float* dk_head_logits, float* dlog_decay, float* dbeta,
                            float* d_initial_state, void* workspace, size_t workspace_bytes, void* stream) {
    return backward_gdn_impl(p, q, k, v, q_head_logits, k_head_logits, log_decay, beta, cu_seqlens, true,
                             initial_state, d_out, d_final_state, dq, dk, dv, dq_head_logits, dk_head_logits,
                             dlog_decay, dbeta, d_initial_state, workspace, workspace_bytes, stream);
}

size_t sla_backward_gdn_workspace_bytes(const sla_params* p) {
    if (check_params(p) != SLA_OK || p->variant != SLA_GDN) return 0;
    return sla::backward_gdn_any_workspace_floats(*p, false) * sizeof(float);
}

size_t sla_backward_gdn_varlen_workspace_bytes(const sla_params* p) {
    if (check_params(p) != SLA_OK || p->variant != SLA_GDN) return 0;
    return sla::backward_gdn_any_workspace_floats(*p, true) * sizeof(float);
}

int sla_gate_logits(const sla_params* p, const void* q, const void* k, const float* w_gq, const float* w_gk,
                    float* q_head_logits, float* k_head_logits, void* stream) {
    const int rc = check_params(p);
    if (rc != SLA_OK) return rc;
    if (p->flags != 0) return SLA_ERR_UNSUPPORTED;
    const bool work = p->B > 0 && p->T > 0;
    if (work && (!q || !w_gq || !q_head_logits)) return SLA_ERR_NULL;
    if ((k != nullptr) != (w_gk != nullptr) || (k != nullptr) != (k_head_logits != nullptr)) return SLA_ERR_NULL;
    const void* ptrs[] = {q, k, w_gq, w_gk, q_head_logits, k_head_logits};
    for (const void* x : ptrs)
        if (x && !aligned16(x)) return SLA_ERR_ALIGN;
    if (!work) return SLA_OK;
    const int cus = device_compute_units();
    if (cus <= 0) return SLA_ERR_HIP;
    return sla::launch_gate_logits(*p, q, k, w_gq, w_gk, q_head_logits, k_head_logits, cus, (hipStream_t)stream);
}

int sla_short_conv_silu(int dtype, int B, int T, int channels, int taps, const void* x, const float* w, void* y,
                        void* stream) {
    if (dtype != SLA_F32 && dtype != SLA_BF16) return SLA_ERR_UNSUPPORTED;
    if (B < 0 || T < 0 || channels < 8 || channels > 65536 || (channels & 7)) return SLA_ERR_SHAPE;
    if (taps < 1 || taps > 4) return SLA_ERR_UNSUPPORTED;
    if ((int64_t)B * T > (int64_t)1 << 30) return SLA_ERR_SHAPE;
    if (B > 0 && T > 0 && (!x || !w || !y)) return SLA_ERR_NULL;
    if ((x && !aligned16(x)) || (y && !aligned16(y)) || (w && !aligned16(w))) return SLA_ERR_ALIGN;
    if (B == 0 || T == 0) return SLA_OK;
    return sla::launch_short_conv_silu(dtype, B, T, channels, taps, x, w, y, (hipStream_t)stream);
}

static int check_feature_map(int dtype, int B, int T, int channels, int taps, int head_width, float eps) {
    if (dtype != SLA_F32 && dtype != SLA_BF16) return SLA_ERR_UNSUPPORTED;
    if (B < 0 || T < 0 || channels < 8 || channels > 65536 || (channels & 7)) return SLA_ERR_SHAPE;
    if (taps < 1 || taps > 4) return SLA_ERR_UNSUPPORTED;
    if ((int64_t)B * T > (int64_t)1 << 30) return SLA_ERR_SHAPE;
    if (head_width != 0) {
        if (head_width != 32 && head_width != 64 && head_width != 128) return SLA_ERR_UNSUPPORTED;
        // the lanes of a head must share one 16-lane row of a wave: whole rows of 128 channels
        if (channels % 128 != 0) return SLA_ERR_SHAPE;
        if (!(eps >= 0.f)) return SLA_ERR_SHAPE;
    }
    return SLA_OK;
}

int sla_short_conv_silu_l2(int dtype, int B, int T, int channels, int taps, int head_width, float eps, const void* x,
                           const float* w, void* y, void* stream) {
    const int rc = check_feature_map(dtype, B, T, channels, taps, head_width, eps);
    if (rc != SLA_OK) return rc;
    if (B > 0 && T > 0 && (!x || !w || !y)) return SLA_ERR_NULL;
    if ((x && !aligned16(x)) || (y && !aligned16(y)) || (w && !aligned16(w))) return SLA_ERR_ALIGN;
    if (B == 0 || T == 0) return SLA_OK;
    return sla::launch_feature_map(dtype, B, T, channels, taps, head_width, eps, x, w, y, (hipStream_t)stream);
}

size_t sla_short_conv_silu_l2_backward_workspace_bytes(int B, int T, int channels, int taps) {
    if (B <= 0 || T <= 0 || channels < 8 || taps < 1 || taps > 4) return 0;
    return sla::feature_map_partials(B, T) * (size_t)channels * taps * sizeof(float);
}

int sla_short_conv_silu_l2_backward(int dtype, int B, int T, int channels, int taps, int head_width, float eps,
                                    const void* x, const float* w, const void* dy, void* dx, float* dw,
                                    void* workspace, size_t workspace_bytes, void* stream) {
    const int rc = check_feature_map(dtype, B, T, channels, taps, head_width, eps);
    if (rc != SLA_OK) return rc;
    if (!dw && channels > 0) return SLA_ERR_NULL;
    if (B > 0 && T > 0 && (!x || !w || !dy || !dx)) return SLA_ERR_NULL;
    const void* ptrs[] = {x, w, dy, dx, dw, workspace};
    for (const void* q : ptrs)
        if (q && !aligned16(q)) return SLA_ERR_ALIGN;
    if (B == 0 || T == 0) return SLA_OK;  // nothing flows; dw is left untouched
    if (!workspace || sla_short_conv_silu_l2_backward_workspace_bytes(B, T, channels, taps) > workspace_bytes)
        return SLA_ERR_WORKSPACE;
    return sla::launch_feature_map_backward(dtype, B, T, channels, taps, head_width, eps, x, w, dy, dx, dw,
                                            (float*)workspace, (hipStream_t)stream);
}

size_t sla_gate_logits_backward_workspace_bytes(const sla_params* p) {
    if (check_params(p) != SLA_OK || p->B == 0 || p->T == 0) return 0;
    return sla::gate_logits_backward_workspace_floats(*p) * sizeof(float);
}

int sla_gate_logits_backward(const sla_params* p, const void* x, const float* w, const float* d_head_logits, void* dx,
                             float* dw, void* workspace, size_t workspace_bytes, void* stream) {
    const int rc = check_params(p);
    if (rc != SLA_OK) return rc;
    if (p->flags != 0) return SLA_ERR_UNSUPPORTED;
    const bool work = p->B > 0 && p->T > 0;
    if (work && (!x || !w || !d_head_logits || !dx || !dw)) return SLA_ERR_NULL;
    const void* ptrs[] = {x, w, d_head_logits, dx, dw, workspace};
    for (const void* q : ptrs)
        if (q && !aligned16(q)) return SLA_ERR_ALIGN;
    if (!work) return SLA_OK;
    if (!workspace || sla_gate_logits_backward_workspace_bytes(p) > workspace_bytes) return SLA_ERR_WORKSPACE;
    return sla::launch_gate_logits_backward(*p, x, w, d_head_logits, dx, dw, (float*)workspace, (hipStream_t)stream);
}

size_t sla_backward_workspace_bytes(const sla_params* p) {
    if (check_params(p) != SLA_OK || p->variant == SLA_GDN) return 0;
    if ((p->dtype == SLA_F32 || p->dk < 64) && p->segments >= 2) return 0;
    return backward_floats(*p, false) * sizeof(float);
}

size_t sla_backward_varlen_workspace_bytes(const sla_params* p) {
    if (check_params(p) != SLA_OK || p->variant == SLA_GDN) return 0;
    return sla::backward_any_workspace_floats(*p, true) * sizeof(float);
}

size_t sla_workspace_bytes(const sla_params* p, int compute_units) {
    if (compute_units <= 0 || check_params(p) != SLA_OK || p->B == 0 || p->T == 0) return 0;
    int seg_len = 0;
    const int nseg = choose_segments(*p, compute_units, &seg_len);
    return sla::segment_workspace_floats(*p, nseg) * sizeof(float);
}

int sla_backward_segments(const sla_params* p, int compute_units) {
    const int rc = check_params(p);
    if (rc != SLA_OK) return rc;
    if (compute_units <= 0) return SLA_ERR_SHAPE;
    if (p->B == 0 || p->T == 0 || p->variant == SLA_GDN || p->flags != 0 || p->dk < 64 || p->dtype == SLA_F32)
        return 1;  // no backward, or no segment schedule, there
    const int64_t wgs = (int64_t)p->B * p->H * ((p->dk < p->dv ? p->dk : p->dv) / 64);
    const int want = (int)((compute_units + wgs - 1) / wgs);
    if (want <= 1) return 1;
    sla_params q = *p;
    q.segments = want;
    int seg_len = 0;
    return choose_segments(q, 1, &seg_len);
}

int sla_segments(const sla_params* p, int compute_units) {
    const int rc = check_params(p);
    if (rc != SLA_OK) return rc;
    if (compute_units <= 0) return SLA_ERR_SHAPE;
    if (p->B == 0 || p->T == 0) return 1;
    int seg_len = 0;
    return choose_segments(*p, compute_units, &seg_len);
}

int sla_default_dv_split(const sla_params* p, int compute_units) {
    if (!p) return SLA_ERR_NULL;
    if (compute_units <= 0) return SLA_ERR_SHAPE;
    if ((p->dv != 64 && p->dv != 128 && p->dv != 256) || p->B < 0 || p->H < 1) return SLA_ERR_SHAPE;
    sla_params c = *p;
    c.dv_split = 0;
    int seg_len = 0;
    const int nseg = (c.segments > 1 && c.T > 0) ? choose_segments(c, compute_units, &seg_len) : 1;
    return choose_dv_split(c, compute_units, nseg);
}

const char* sla_kernel_name(const sla_params* p) {
    static thread_local char buf[128];
    if (!p) return nullptr;
    if (p->variant < 0 || p->variant > 2 || (p->dtype != SLA_F32 && p->dtype != SLA_BF16)) return nullptr;
    if (p->dv != 64 && p->dv != 128 && p->dv != 256) return nullptr;
    int seg_len = 0;  // dv_split == 0 is resolved as on a 256-CU device, for the schedule p->segments asks for
    const int nseg = (p->segments > 1 && p->T > 0 && p->variant != SLA_GDN) ? choose_segments(*p, 256, &seg_len) : 1;
    const int dvw = choose_dv_split(*p, 256, nseg);
    const int head_regs = p->H <= 16 ? 4 : (p->H <= 32 ? 8 : 16);
    snprintf(buf, sizeof(buf), "sla_fwd_kernel<sla::%s, %d, %d, %d, %d, false>", p->dtype == SLA_BF16 ? "PrecBF16" : "PrecF32",
             p->variant, p->dk, dvw, head_regs);
    return buf;
}

const char* sla_status_string(int status) {
    switch (status) {
        case SLA_OK: return "ok";
        case SLA_ERR_NULL: return "a required pointer is NULL (or beta given for a variant without it)";
        case SLA_ERR_SHAPE: return "a size is negative or out of range";
        case SLA_ERR_UNSUPPORTED: return "variant, dtype, head width or flag not supported";
        case SLA_ERR_ALIGN: return "a pointer is not 16-byte aligned";
        case SLA_ERR_HIP: return "the HIP runtime refused the call";
        case SLA_ERR_WORKSPACE: return "segments requested but the workspace is missing or too small";
        case SLA_ERR_SCRATCH: return "the schedule for this shape needs more than the library's static scratch buffer holds";
        default: return "unknown status";
    }
}

int sla_version(void) { return kVersion; }

}  // extern "C"
