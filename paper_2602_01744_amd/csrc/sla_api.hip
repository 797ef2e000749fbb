// C-ABI entry points of libsla: argument validation and dispatch.  All checks that do not need the
// device run first, so a bad call is rejected before any HIP call (and sla_check_args runs them alone).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "sla.h"

namespace sla {
int launch_forward(const sla_params& p, int dvw, const void* q, const void* k, const void* v, const float* ql,
                   const float* kl, const void* ld, const float* beta, const float* s0, void* out, float* sT,
                   hipStream_t stream);
}

namespace {

constexpr int kVersion = 100;  // 0.1.0
constexpr int kMaxHeads = 64;

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check(const sla_params* p, const void* q, const void* k, const void* v, const float* ql, const float* kl,
          const void* ld, const float* beta, const float* s0, const void* out, const float* sT) {
    if (!p) return SLA_ERR_NULL;
    if (p->variant != SLA_RETNET && p->variant != SLA_GLA && p->variant != SLA_GDN) return SLA_ERR_UNSUPPORTED;
    if (p->dtype != SLA_F32 && p->dtype != SLA_BF16) return SLA_ERR_UNSUPPORTED;
    if (p->flags != 0) return SLA_ERR_UNSUPPORTED;
    if (p->B < 0 || p->T < 0 || p->H < 1 || p->H > kMaxHeads) return SLA_ERR_SHAPE;
    if (p->dk < 1 || p->dv < 1) return SLA_ERR_SHAPE;
    if ((p->dk != 64 && p->dk != 128) || (p->dv != 64 && p->dv != 128)) return SLA_ERR_UNSUPPORTED;
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

int choose_dv_split(const sla_params& p, int cus) {
    if (p.dv_split != 0) return p.dv_split;
    // The widest slice that still gives every compute unit a workgroup; narrower slices repeat the
    // per-token decay work of a head in more workgroups, so never go narrower than needed.
    const int64_t seqs = (int64_t)p.B * p.H;
    const int widths[] = {64, 32, 16};
    for (int w : widths) {
        if (w > p.dv) continue;
        if (seqs * (p.dv / w) >= cus) return w;
    }
    return 16;
}

}  // namespace

extern "C" {

int sla_check_args(const sla_params* p, const void* q, const void* k, const void* v, const float* q_head_logits,
                   const float* k_head_logits, const void* log_decay, const float* beta, const float* initial_state,
                   const void* out, const float* final_state) {
    return check(p, q, k, v, q_head_logits, k_head_logits, log_decay, beta, initial_state, out, final_state);
}

int sla_forward(const sla_params* p, const void* q, const void* k, const void* v, const float* q_head_logits,
                const float* k_head_logits, const void* log_decay, const float* beta, const float* initial_state,
                void* out, float* final_state, void* stream) {
    const int rc = check(p, q, k, v, q_head_logits, k_head_logits, log_decay, beta, initial_state, out, final_state);
    if (rc != SLA_OK) return rc;
    if (p->B == 0) return SLA_OK;
    if (p->T == 0 && !final_state) return SLA_OK;
    const int cus = device_compute_units();
    if (cus <= 0) return SLA_ERR_HIP;
    const int dvw = choose_dv_split(*p, cus);
    return sla::launch_forward(*p, dvw, q, k, v, q_head_logits, k_head_logits, log_decay, beta, initial_state, out,
                               final_state, (hipStream_t)stream);
}

int sla_default_dv_split(const sla_params* p, int compute_units) {
    if (!p) return SLA_ERR_NULL;
    if (compute_units <= 0) return SLA_ERR_SHAPE;
    if ((p->dv != 64 && p->dv != 128) || p->B < 0 || p->H < 1) return SLA_ERR_SHAPE;
    sla_params c = *p;
    c.dv_split = 0;
    return choose_dv_split(c, compute_units);
}

const char* sla_kernel_name(const sla_params* p) {
    static thread_local char buf[128];
    if (!p) return nullptr;
    if (p->variant < 0 || p->variant > 2 || (p->dtype != SLA_F32 && p->dtype != SLA_BF16)) return nullptr;
    if (p->dv != 64 && p->dv != 128) return nullptr;
    const int dvw = choose_dv_split(*p, 256);  // dv_split == 0 is resolved as on a 256-CU device
    const int head_regs = p->H <= 16 ? 4 : (p->H <= 32 ? 8 : 16);
    snprintf(buf, sizeof(buf), "sla_fwd_kernel<sla::%s, %d, %d, %d, %d>", p->dtype == SLA_BF16 ? "PrecBF16" : "PrecF32",
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
        default: return "unknown status";
    }
}

int sla_version(void) { return kVersion; }

}  // extern "C"
