// Driver for the sanitizer build of the library's host-side validation (csrc/sla_api.hip compiled with
// -fsanitize=address,undefined on the host pass; tests/test_sanitizers.py builds and runs it).  The launchers of
// the other translation units are replaced by stubs that must never be reached: every call below is either
// rejected by the checks that run before any device work, or is a no-op by definition (B = 0, T = 0 without a
// state), or stops at the first HIP call because this program runs where there is no GPU.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>

#include "sla.h"

namespace sla {
static int reached(const char* what) {
    std::fprintf(stderr, "stub launcher %s reached: validation let a call through\n", what);
    std::abort();
}
int launch_forward(const sla_params&, int, int, int, const void*, const void*, const void*, const float*, const float*,
                   const void*, const float*, const float*, void*, float*, float*, const int*, hipStream_t) { return reached("forward"); }
size_t segment_workspace_floats(const sla_params& p, int nseg) {
    return nseg <= 1 ? 0 : (size_t)p.B * p.H * ((size_t)nseg * p.dk * p.dv + (size_t)(nseg - 1) * 8 * p.dk);
}
size_t backward_workspace_floats(const sla_params& p, bool) { return (size_t)p.B * p.T * p.H * 20 + 1024; }
int launch_backward(const sla_params&, const void*, const void*, const void*, const float*, const float*, const void*,
                    const float*, const void*, const float*, void*, void*, void*, float*, float*, void*, float*, float*,
                    const int*, hipStream_t) { return reached("backward"); }
size_t backward_segment_extra_floats(const sla_params& p, int nseg) { return (size_t)p.B * nseg * p.H * p.dk * p.dv * 3; }
sla_params packed_segments(const sla_params& p, int nseg) { sla_params q = p; q.B = p.B * nseg; q.T = p.B * p.T; return q; }
int launch_backward_segments(const sla_params&, int, int, int, const void*, const void*, const void*, const float*,
                             const float*, const void*, const float*, const void*, const float*, void*, void*, void*,
                             float*, float*, void*, float*, float*, hipStream_t) { return reached("backward segments"); }
size_t backward_gdn_workspace_floats(const sla_params& p, bool) { return (size_t)p.B * p.T * p.H * 400 + 1024; }
int launch_backward_gdn(const sla_params&, const void*, const void*, const void*, const float*, const float*,
                        const float*, const float*, const float*, const void*, const float*, void*, void*, void*,
                        float*, float*, float*, float*, float*, float*, const int*, hipStream_t) { return reached("backward gdn"); }
size_t backward_any_workspace_floats(const sla_params& p, bool packed) { return backward_workspace_floats(p, packed); }
int launch_backward_any(const sla_params&, const void*, const void*, const void*, const float*, const float*, const void*,
                        const float*, const void*, const float*, void*, void*, void*, float*, float*, void*, float*,
                        float*, const int*, bool, hipStream_t) { return reached("backward"); }
size_t backward_gdn_any_workspace_floats(const sla_params& p, bool packed) { return backward_gdn_workspace_floats(p, packed); }
int launch_backward_gdn_any(const sla_params&, const void*, const void*, const void*, const float*, const float*,
                            const float*, const float*, const float*, const void*, const float*, void*, void*, void*,
                            float*, float*, float*, float*, float*, float*, const int*, bool, hipStream_t) {
    return reached("backward gdn");
}
int launch_gate_logits(const sla_params&, const void*, const void*, const float*, const float*, float*, float*, int,
                       hipStream_t) { return reached("gate logits"); }
int launch_short_conv_silu(int, int, int, int, int, const void*, const float*, void*, hipStream_t) { return reached("conv"); }
size_t feature_map_partials(int B, int T) { return (size_t)B * ((T + 63) / 64); }
int launch_feature_map(int, int, int, int, int, int, float, const void*, const float*, void*, hipStream_t) { return reached("feature map"); }
int launch_feature_map_backward(int, int, int, int, int, int, float, const void*, const float*, const void*, void*,
                                float*, float*, hipStream_t) { return reached("feature map backward"); }
int launch_gate_logits_backward(const sla_params&, const void*, const float*, const float*, void*, float*, float*,
                                hipStream_t) { return reached("gate logits backward"); }
size_t gate_logits_backward_workspace_floats(const sla_params& p) { return (size_t)1024 * p.H * p.dk; }
int launch_decode(const sla_params&, const void*, const void*, const void*, const float*, const float*, const float*,
                  const float*, const void*, const float*, float*, void*, hipStream_t) { return reached("decode"); }
}  // namespace sla

static int failures = 0;
#define EXPECT(call, want)                                                                            \
    do {                                                                                              \
        const long long got_ = (long long)(call);                                                     \
        if (got_ != (long long)(want)) {                                                              \
            std::fprintf(stderr, "%s:%d: %s = %lld, expected %lld\n", __FILE__, __LINE__, #call, got_, \
                         (long long)(want));                                                          \
            ++failures;                                                                               \
        }                                                                                             \
    } while (0)

int main() {
    void* A = (void*)(uintptr_t)(1u << 20);  // a 16-byte aligned fake address; validation never dereferences it
    float* F = (float*)A;
    sla_params ok = {SLA_GLA, SLA_BF16, 2, 128, 4, 128, 128, 0, 0, 0};
    // every combination of a small grid of fields goes through the checks (results vary; none may trip a sanitizer)
    const int variants[] = {-1, 0, 1, 2, 3}, dtypes[] = {-1, 0, 1, 2}, sizes[] = {-5, 0, 1, 2, 63, 64, 4096, 1 << 30};
    const int widths[] = {0, 16, 32, 48, 64, 96, 128, 256, 512}, heads[] = {-1, 0, 1, 16, 64, 65};
    const int splits[] = {-16, 0, 8, 16, 32, 64, 128, 256}, segs[] = {-1, 0, 1, 2, 7, 4096, 4097};
    long long calls = 0;
    for (int v : variants) for (int d : dtypes) for (int B : sizes) for (int T : sizes) for (int H : heads)
        for (int dk : widths) for (int dv : widths) {
            sla_params p = {v, d, B, T, H, dk, dv, 0, 0, 0};
            (void)sla_check_args(&p, A, A, A, F, F, A, v == 2 ? F : nullptr, nullptr, A, F);
            (void)sla_workspace_bytes(&p, 256);
            (void)sla_segments(&p, 256);
            (void)sla_backward_segments(&p, 256);
            (void)sla_backward_workspace_bytes(&p);
            (void)sla_backward_varlen_workspace_bytes(&p);
            (void)sla_backward_gdn_workspace_bytes(&p);
            (void)sla_gate_logits_backward_workspace_bytes(&p);
            (void)sla_default_dv_split(&p, 256);
            (void)sla_kernel_name(&p);
            calls += 10;
        }
    for (int s : splits) for (int g : segs) for (int T : sizes) {
        sla_params p = ok;
        p.dv_split = s; p.segments = g; p.T = T;
        (void)sla_check_args(&p, A, A, A, F, F, A, nullptr, nullptr, A, F);
        (void)sla_workspace_bytes(&p, 1); (void)sla_workspace_bytes(&p, 256); (void)sla_workspace_bytes(&p, 0);
        (void)sla_segments(&p, 304);
        (void)sla_default_dv_split(&p, 304);
        calls += 6;
    }
    // a few fixed expectations, as in the Python ABI tests
    EXPECT(sla_check_args(&ok, A, A, A, F, F, A, nullptr, nullptr, A, F), SLA_OK);
    EXPECT(sla_check_args(nullptr, A, A, A, F, F, A, nullptr, nullptr, A, F), SLA_ERR_NULL);
    EXPECT(sla_check_args(&ok, A, (char*)A + 4, A, F, F, A, nullptr, nullptr, A, F), SLA_ERR_ALIGN);
    sla_params bad = ok; bad.dk = 96;
    EXPECT(sla_forward(&bad, A, A, A, F, F, A, nullptr, nullptr, A, F, nullptr), SLA_ERR_UNSUPPORTED);
    sla_params empty = ok; empty.B = 0;
    EXPECT(sla_forward(&empty, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr), SLA_OK);
    sla_params big = {SLA_GLA, SLA_BF16, 4, 8192, 16, 128, 128, 0, 0, 8};
    EXPECT(sla_forward_static(&big, A, A, A, F, F, A, nullptr, nullptr, A, F, nullptr), SLA_ERR_SCRATCH);
    EXPECT(sla_forward_ws(&big, A, A, A, F, F, A, nullptr, nullptr, A, F, A, 16, nullptr), SLA_ERR_WORKSPACE);
    EXPECT(sla_backward(&ok, A, A, A, F, F, A, nullptr, A, nullptr, A, A, A, F, F, A, nullptr, A, 15, nullptr), SLA_ERR_WORKSPACE);
    EXPECT(sla_short_conv_silu_l2(SLA_BF16, 2, 64, 200, 4, 64, 1e-6f, A, F, A, nullptr), SLA_ERR_SHAPE);
    EXPECT(sla_short_conv_silu_l2_backward(SLA_BF16, 2, 100, 256, 4, 64, 1e-6f, A, F, A, A, F, A, 16, nullptr), SLA_ERR_WORKSPACE);
    EXPECT(sla_gate_logits_backward(&ok, A, F, nullptr, A, F, A, (size_t)1 << 30, nullptr), SLA_ERR_NULL);
    for (int code = -9; code <= 1; ++code)
        if (!sla_status_string(code)) ++failures;
    EXPECT(sla_version() >= 100, 1);
    std::printf("%lld validation calls, %d failures\n", calls + 12, failures);
    return failures != 0;
}
