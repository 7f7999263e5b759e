// Small wrappers around the bf16 matrix-core instruction used by the attention kernels.
//
// v_mfma_f32_16x16x32_bf16 computes D[16x16] += A[16x32] . B[32x16].  Lane l supplies the 8 contraction
// entries k = 8*(l/16) .. +7 of A's row l%16 and of B's column l%16, and receives D[4*(l/16)+i][l%16]
// in register i.
#pragma once

#include "stream_kv.hpp"

namespace ra {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ floatx4_t mfma16(uint4 a, uint4 b, floatx4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c,
                                                   0, 0, 0);
}
// Largest of the eight logits a lane holds of one 16-row x 32-token score tile.
__device__ __forceinline__ float max8(floatx4_t a, floatx4_t b) {
    float m = vmax(a[0], a[1]);  // a chain: the compiler pairs its links into three-operand maxima
#pragma unroll
    for (int i = 2; i < 4; ++i) m = vmax(m, a[i]);
#pragma unroll
    for (int i = 0; i < 4; ++i) m = vmax(m, b[i]);
    return m;
}
// Two floats -> packed bf16 pair by truncation (low half = a, high half = b).
__device__ __forceinline__ uint32_t pack_trunc(float a, float b) { return (as_u32(b) & 0xffff0000u) | (as_u32(a) >> 16); }
// Same value with one byte-permute instruction: bytes 2,3 of a, then bytes 2,3 of b.
__device__ __forceinline__ uint32_t pack_hi16(float a, float b) {
    return __builtin_amdgcn_perm(as_u32(b), as_u32(a), 0x07060302u);
}
__device__ __forceinline__ float trunc_bf16(float a) { return as_f32(as_u32(a) & 0xffff0000u); }

}  // namespace ra
