// Device-side helpers shared by the kernels (not part of the ABI): vector types, the MFMA
// wrapper, the 16-bit storage conversions and the padding bias.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fk {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx2 __attribute__((ext_vector_type(2)));

// Score bias of centroid rows beyond K: it must survive having its low mantissa bits
// overwritten by the packed argmax (-inf would turn into a NaN pattern) and still lose against
// every real score.
constexpr float kPadBias = -3.0e38f;

__device__ __forceinline__ float lp_to_float(uint16_t v, bool bf) {
    return bf ? __uint_as_float((uint32_t)v << 16) : (float)__builtin_bit_cast(_Float16, v);
}

// round-to-nearest-even from fp32 (finite input)
__device__ __forceinline__ uint16_t float_to_lp(float f, bool bf) {
    if (bf) {
        uint32_t u = __float_as_uint(f);
        u += 0x7FFFu + ((u >> 16) & 1u);
        return (uint16_t)(u >> 16);
    }
    return __builtin_bit_cast(uint16_t, (_Float16)f);
}

// D = A (32 x 16) * B (16 x 32) + C with fp32 accumulation; lane (r = lane % 32, h = lane / 32)
// supplies A[r][8h .. 8h+7] and B[8h .. 8h+7][r] and receives D[8*(i/4) + 4h + i%4][r], i < 16.
template <bool BF>
__device__ __forceinline__ floatx16 mfma32(uintx4 a, uintx4 b, floatx16 c) {
    if constexpr (BF)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, a),
                                                      __builtin_bit_cast(half8, b), c, 0, 0, 0);
}

// 32-bit LDS address of a pointer into shared memory (for hand-issued LDS instructions)
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return (uint32_t)(uintptr_t)((__attribute__((address_space(3))) const void*)p);
}

}  // namespace fk
