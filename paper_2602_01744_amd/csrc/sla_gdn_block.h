// Arguments of the block-form backward sweeps of the gated delta rule (sla_backward_gdn_block.hip), filled by
// launch_backward_gdn (sla_backward_gdn.hip), which also runs the gate, finishing and decay-scan kernels around them.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "sla.h"

namespace sla {

struct GdnBlockArgs {
    const uint16_t* q;      // [rows,H,dk] bf16
    const uint16_t* k;
    const uint16_t* v;      // [rows,H,dv]
    const uint16_t* dout;
    const float* ld;        // [rows,H]
    const float* beta;
    const float* gq;        // gates [rows,H] (already through the head softmax)
    const float* gk;
    const float* s0;        // [B,H,dk,dv] or null
    const float* dsf;       // cotangent of the final state, or null
    uint16_t* dq;
    uint16_t* dk;
    uint16_t* dv;
    float* ds0;             // or null
    float* part_q;          // [dk/16][plane]: partial q . (dout S^T)
    float* part_k;          // [dv/16][plane]: partial w . v
    float* part_b;          // [dv/16][plane]: partial du . res
    float* corr;            // [dk/16][B*H]: partial <d_final, S_T>
    float* anchor_x;        // [rows/512 + 1][H][dk][dv]: the state cotangent entering every 512th token of a sequence
    float* anchor_phi;      // [rows/512 + 1][H][dk/16]: partial <that cotangent, the state there>
    size_t plane;           // floats between partial planes (>= rows * H)
    float* block_ws;        // gdn_block_workspace_floats() floats, 16-byte aligned
    size_t rows;            // tokens in all: B * T, or the packed total T
    const int* cu;          // packed batch: sequence b is tokens cu[b] .. cu[b+1]-1 of the T in all; else null
    int B, T, H, dim_k, dim_v;
};

// The decay gradient is a suffix sum of per-token scalars built from bf16-operand products, whose rounding adds up
// like a random walk over the tokens behind; every kGdnAnchor tokens of a sequence it is re-derived exactly as
// <X, S> at that boundary (sweep 3 leaves X there, sweep 4 forms the product).  Anchors are numbered by absolute
// token position / kGdnAnchor: sequences do not overlap, so neither do their anchors (fewer than rows / 512 + 1).
constexpr int kGdnAnchor = 512;
inline size_t gdn_anchor_count(size_t rows) { return rows / kGdnAnchor + 1; }
// Floats of block_ws for this shape.
size_t gdn_block_workspace_floats(int B, int T, int H, int dk, int dv, bool packed);
// Runs the block-local pre-pass and the four state sweeps on `stream`.
int launch_gdn_block_sweeps(const GdnBlockArgs& a, hipStream_t stream);

}  // namespace sla
