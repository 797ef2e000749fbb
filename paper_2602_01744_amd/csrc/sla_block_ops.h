// Building blocks of the 32-token block kernels of the gated delta rule (sla_backward_gdn_block.hip): bf16 operands
// of v_mfma_f32_16x16x32_bf16 taken from row-major LDS arrays by rows or, through the transposing LDS read of gfx950, by columns; accumulator tiles reused as operands; small reductions.
//
// Conventions.  Lane (r, g) = (lane % 16, lane / 16).  An accumulator tile of a product D = A B holds D[4g + i][r] in
// register i.  The contraction index of operand slot (half, g, e) is 16 half + 4 g + e in both operands, which makes
// an accumulator tile pair (X[0], X[1]) of a 32-row matrix X directly the B operand "X" (column r) and the A operand
// "X^T" (row r) of the next product.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sla.h"

namespace sla {
namespace blk {

typedef __attribute__((ext_vector_type(4))) float f4;
typedef __attribute__((ext_vector_type(4))) uint32_t u4;
typedef __attribute__((ext_vector_type(2))) uint32_t u2;
typedef __attribute__((ext_vector_type(4))) short s4;
typedef __attribute__((ext_vector_type(8))) short s8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf2;
typedef __attribute__((ext_vector_type(8))) __bf16 bf8;
typedef uint16_t bf;
typedef __attribute__((address_space(3))) s4 lds_s4;

constexpr int C = 32;            // tokens per block
// LDS row strides, in elements.  A row read (op_rows: 16 rows x 16 bytes per half-wave) is conflict-free when
// consecutive rows are 16 bytes apart modulo the 256 bytes of the 64 banks, a column read (op_cols: 8 rows x 32 bytes
// per half-wave) when they are 32 bytes apart: arrays get 8 or 16 elements of padding according to how the sweep
// reads them (k, which sweeps 1 and 2 read both ways, is staged twice).
constexpr int kSmR = 40, kSmC = 48;   // 32 elements per row: read by rows / by columns
constexpr int kSlR = 72, kSlC = 80;   // a 64-column slice of token rows
constexpr int rows_stride(int width) { return width + 8; }
constexpr int cols_stride(int width) { return width + 16; }
constexpr float kLog2e = 1.4426950408889634f;

// per-token scalars of a block: kinds x 32 floats
enum { kP = 0, kAP = 1, kBeta = 2, kGq = 3, kGk = 4, kCl = 5, kA = 6, kKinds = 8 };
constexpr int kScal = kKinds * C;            // floats per (block, head)

__device__ __forceinline__ float bf_lo(uint32_t p) { return __uint_as_float(p << 16); }
__device__ __forceinline__ float bf_hi(uint32_t p) { return __uint_as_float(p & 0xffff0000u); }
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {  // the hardware conversion: nearest even, NaN kept
    bf2 t;
    t.x = (__bf16)lo;
    t.y = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, t);
}
__device__ __forceinline__ u2 pack4(f4 x) { return u2{pack2(x[0], x[1]), pack2(x[2], x[3])}; }
__device__ __forceinline__ s8 pack8(f4 x, f4 y) {
    const u4 t = {pack2(x[0], x[1]), pack2(x[2], x[3]), pack2(y[0], y[1]), pack2(y[2], y[3])};
    return __builtin_bit_cast(s8, t);
}
__device__ __forceinline__ f4 unpack4(u2 t) { return f4{bf_lo(t.x), bf_hi(t.x), bf_lo(t.y), bf_hi(t.y)}; }
__device__ __forceinline__ f4 unpack4(s4 v) { return unpack4(__builtin_bit_cast(u2, v)); }
// the operand with slot (half, g, e) multiplied by lo[e] (half 0) or hi[e] (half 1)
__device__ __forceinline__ s8 scale8(s8 v, f4 lo, f4 hi) {
    const u4 t = __builtin_bit_cast(u4, v);
    return pack8(unpack4(u2{t.x, t.y}) * lo, unpack4(u2{t.z, t.w}) * hi);
}
__device__ __forceinline__ s8 join(s4 a, s4 b) { return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7); }
__device__ __forceinline__ void mma(f4& c, s8 a, s8 b) {
    c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf8, a), __builtin_bit_cast(bf8, b), c, 0, 0, 0);
}

// Operand of a 32-slot product from a row-major LDS array: lane (r, g) takes row `row`, slots k0 + 4g .. and
// k0 + 16 + 4g ..
__device__ __forceinline__ s8 op_rows(const bf* base, int stride, int row, int k0, int g) {
    const bf* p = base + row * stride + k0 + 4 * g;
    return join(*(const s4*)p, *(const s4*)(p + 16));
}
// The same from the array's columns: lane (r, g) takes column c0 + r, slot rows j0 + 4g .. and j0 + 16 + 4g ..
// (transposing read: lane l of a group of 16 addresses row l/4, columns 4 (l%4) .. +3, and receives column l of the
// four rows).
__device__ __forceinline__ s4 lds_tr(const bf* p) { return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4*)p); }
__device__ __forceinline__ s8 op_cols(const bf* base, int stride, int j0, int c0, int r, int g) {
    const bf* p = base + (j0 + 4 * g + (r >> 2)) * stride + c0 + 4 * (r & 3);
    return join(lds_tr(p), lds_tr(p + 16 * stride));
}
// Four rows j0 + 4g .. +3 of column c0 + r (an accumulator-shaped piece of a row-major array).
__device__ __forceinline__ f4 tile_cols(const bf* base, int stride, int j0, int c0, int r, int g) {
    return unpack4(lds_tr(base + (j0 + 4 * g + (r >> 2)) * stride + c0 + 4 * (r & 3)));
}
__device__ __forceinline__ f4 sc4(const float* sc, int kind, int t) { return *(const f4*)(sc + kind * C + t); }

// Sum over the four lane groups of the wave; every lane gets the total.
__device__ __forceinline__ float all_groups(float x) {
    const uint32_t xi = __float_as_uint(x);
    const u2 a = __builtin_amdgcn_permlane16_swap(xi, xi, false, false);
    const uint32_t yi = __float_as_uint(__uint_as_float(a[0]) + __uint_as_float(a[1]));
    const u2 b = __builtin_amdgcn_permlane32_swap(yi, yi, false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
    return __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(x), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float row_all(float x) {  // sum over the 16 lanes of a group
    x += dpp_move<0x128>(x);
    x += dpp_move<0x124>(x);
    x += dpp_move<0x122>(x);
    x += dpp_move<0x121>(x);
    return x;
}

// fp32 product on the matrix cores: lane (r, g) gives A[r][g] and B[g][r] of a 16 x 4 by 4 x 16 step
__device__ __forceinline__ void mma_f32(f4& c, float a, float b) { c = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0); }

}  // namespace blk
}  // namespace sla
