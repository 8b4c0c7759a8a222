// Small helpers for the matrix cores of gfx950 shared by the kernels that use v_mfma_f32_16x16x32_f16.
//
// Operand layout of one 16 x 16 x 32 step, lane = 16 g + c (g = 0..3, c = 0..15):
//   A: the lane holds A[i = c][k = 8 g .. 8 g + 7]      B: the lane holds B[k = 8 g .. 8 g + 7][j = c]
//   result: the lane holds D[i = 4 g + rr][j = c], rr = 0..3
#ifndef CF_MFMA_DEVICE_H
#define CF_MFMA_DEVICE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cf {
namespace mfma {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x4 mfma16(const h8 &a, const h8 &b, const f32x4 &c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// w[u] = row u, eight adjacent columns  ->  f[c] = column c, rows 0..7 (8 x 8 transpose of 16-bit values in a lane):
// turns eight 16-byte pieces of row-major rows into eight B operands (contraction over the rows).
__device__ __forceinline__ void transpose8(const h8 *w, h8 (&f)[8])
{
#pragma unroll
    for (int c2 = 0; c2 < 4; ++c2) {
        u32x4 e, o;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const uint32_t lo = __builtin_bit_cast(u32x4, w[2 * d])[c2], hi = __builtin_bit_cast(u32x4, w[2 * d + 1])[c2];
            e[d] = __builtin_amdgcn_perm(hi, lo, 0x05040100u);    // {lo.low half, hi.low half}
            o[d] = __builtin_amdgcn_perm(hi, lo, 0x07060302u);    // {lo.high half, hi.high half}
        }
        f[2 * c2] = __builtin_bit_cast(h8, e);
        f[2 * c2 + 1] = __builtin_bit_cast(h8, o);
    }
}

}  // namespace mfma
}  // namespace cf

#endif
