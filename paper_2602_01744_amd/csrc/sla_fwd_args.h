// Argument block of the forward kernels, shared by the kernel templates (sla_fwd_kernels.h) and the host-side
// launcher (sla_kernels.hip).
#pragma once
#include <stddef.h>

namespace sla {

static constexpr int kMaxSlots = 8;  // LDS ring slots = producer waves (at most)

struct KArgs {
    const void* q;
    const void* k;
    const void* v;
    const float* ql;
    const float* kl;
    const void* ld;
    const float* beta;
    const float* s0;
    void* out;
    float* sT;
    int B, T, H, dv;
    int nslice;
    // Segment-parallel schedule: T is cut into nseg segments of Ls tokens (the last may be shorter) and
    // every (batch, segment) pair is scheduled like a batch row.  nseg_grid is the number of segments a
    // launch covers: nseg for the main pass, nseg - 1 for the pre-pass that only computes the end state
    // of each segment from a zero entry state.  ws_state[b][s][h] holds that state and, after the
    // combine kernel, the entry state of segment s + 1; ws_decay[b][s][h][8][dk] the decay of segment s
    // as partial products, one per producer wave (GLA).
    int Ls, nseg, nseg_grid;
    int nparts;  // producer waves of the pre-pass: partial decay products per segment in ws_decay
    float* ws_state;
    float* ws_decay;
    // Used by the backward pass's segment schedule, which wants only what the pre-pass and the combine kernel
    // produce: the entry state of every segment (ws_state) and, in ws_total[b][s][h][dk], the total decay of each
    // segment but the last.  states_only stops the call after the combine kernel.
    float* ws_total;
    bool states_only;
    // Packed variable-length batch: B sequences laid end to end in tensors of T tokens in all; sequence b covers
    // tokens cu[b] .. cu[b + 1] - 1.  Null for the rectangular layout.
    const int* cu;
    // q, k, v, out and the GLA decay laid out [B,H,T,d] instead of [B,T,H,d]: every (batch, head) streams one
    // contiguous region.  Logits, beta, the delta rule's decay and the states keep their layouts.
    bool head_major;
    // Sticky device status word (bits of SLA_DEVICE_*): a bounded wait that expired, a GLA block decay outside the
    // documented range.  Never null.
    unsigned int* status;
};

}  // namespace sla
