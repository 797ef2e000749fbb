// Forward kernels for bf16 tensors: every instantiation of sla_fwd_kernels.h for this element type.
#include "sla_fwd_kernels.h"

namespace sla {

int dispatch_forward_bf16(const KArgs& a, int variant, int dk, int dvw, hipStream_t stream) {
    return dispatch_variant<PrecBF16>(a, variant, dk, dvw, stream);
}

}  // namespace sla
