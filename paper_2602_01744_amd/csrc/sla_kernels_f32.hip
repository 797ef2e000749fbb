// Forward kernels for f32 tensors: every instantiation of sla_fwd_kernels.h for this element type.
#include "sla_fwd_kernels.h"

namespace sla {

int dispatch_forward_f32(const KArgs& a, int variant, int dk, int dvw, hipStream_t stream) {
    return dispatch_variant<PrecF32>(a, variant, dk, dvw, stream);
}

}  // namespace sla
