// bf16 MFMA fragments from LDS tiles (gfx950): shared by the grouped GEMM and the fused
// wide-output-layer kernels.
//
// v_mfma_f32_32x32x16_bf16 takes, per lane, 8 consecutive k values of one row of each operand:
// lane l holds row l % 32, k = 8 (l / 32) .. 8 (l / 32) + 7 of the 16-deep k-step.
//   - a tile stored [row][k] (k contiguous) gives that as one 128-bit LDS read;
//   - a tile stored [k][row] (rows contiguous, as the matrix lies in memory when k is its slow index)
//     gives it through the transposing LDS read ds_read_b64_tr_b16, two per fragment.
// With the operands swapped, mma(b, a, c), accumulator register v of a lane is row l % 32 of the a
// operand and column 8 (v / 4) + 4 (l / 32) + v % 4 of the b operand: four consecutive registers are four
// consecutive columns.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ist {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

__device__ inline f32x16 bf16_mma(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// rows rb .. rb + 31, k-step ks (16 k values) of a [row][k] tile with row pitch ld (elements)
__device__ inline bf16x8 bf16_frag_k(const uint16_t *lds, int rb, int ks, int lane, int ld)
{
    return *reinterpret_cast<const bf16x8 *>(lds + (rb + (lane & 31)) * ld + ks * 16 + (lane >> 5) * 8);
}

// the same fragment from a [k][row] tile with k-row pitch ld (elements)
__device__ inline bf16x8 bf16_frag_m(const uint16_t *lds, int rb, int ks, int lane, int ld)
{
    // 16-lane block: lane q supplies the address of 4 consecutive row-elements
    // [k0 + q/4][m0 + 4*(q%4)] and receives [k0 .. k0+3][m0 + q].
    const int q = lane & 15;
    const int m0 = rb + ((lane >> 4) & 1) * 16;
    const int k0 = ks * 16 + (lane >> 5) * 8;
    const uint16_t *p0 = lds + (k0 + (q >> 2)) * ld + m0 + 4 * (q & 3);
    const uint16_t *p1 = p0 + 4 * ld;
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p0));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p1));
    s16x8 r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
}

}  // namespace ist
