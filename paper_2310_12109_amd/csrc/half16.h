// The two 16-bit element types of the matrix-core kernels (bf16_t, f16_t) behind one set of helpers: a kernel
// templated on the element type E differs only in how a pair of floats is rounded to a packed pair, how the halves
// of a packed pair are widened, and which matrix instruction takes the operands.
#pragma once

#include "common.h"

namespace monarch {
namespace h16 {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t op8;   // one MFMA operand: 8 packed 16-bit values of either type

template <typename E> __device__ __forceinline__ uint32_t pack16(float lo, float hi)
{
    typedef __attribute__((ext_vector_type(2))) E pair_t;
    pair_t p = {(E)lo, (E)hi};
    return __builtin_bit_cast(uint32_t, p);
}
template <typename E> __device__ __forceinline__ float lo32(uint32_t d);
template <typename E> __device__ __forceinline__ float hi32(uint32_t d);
template <> __device__ __forceinline__ float lo32<bf16_t>(uint32_t d) { return __uint_as_float(d << 16); }
template <> __device__ __forceinline__ float hi32<bf16_t>(uint32_t d) { return __uint_as_float(d & 0xffff0000u); }
template <> __device__ __forceinline__ float lo32<f16_t>(uint32_t d)
{
    typedef __attribute__((ext_vector_type(2))) f16_t pair_t;
    return (float)__builtin_bit_cast(pair_t, d)[0];
}
template <> __device__ __forceinline__ float hi32<f16_t>(uint32_t d)
{
    typedef __attribute__((ext_vector_type(2))) f16_t pair_t;
    return (float)__builtin_bit_cast(pair_t, d)[1];
}

// D = A B + C, 16 x 16 x 32, fp32 accumulation
template <typename E> __device__ __forceinline__ f32x4 mfma(op8 a, op8 b, f32x4 c);
template <> __device__ __forceinline__ f32x4 mfma<bf16_t>(op8 a, op8 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
template <> __device__ __forceinline__ f32x4 mfma<f16_t>(op8 a, op8 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

}  // namespace h16
}  // namespace monarch
