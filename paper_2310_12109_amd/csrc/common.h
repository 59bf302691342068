// Shared host/device helpers of the Monarch library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "monarch.h"

namespace monarch {

typedef __bf16 bf16_t;
typedef _Float16 f16_t;

// Thread-local message of the last failing call; returns `code` for tail calls.
int fail(int code, const char *fmt, ...);
void clear_error();

#define MONARCH_HIP_CHECK(expr)                                                        \
    do {                                                                               \
        hipError_t e__ = (expr);                                                       \
        if (e__ != hipSuccess)                                                         \
            return ::monarch::fail(MONARCH_EHIP, "%s failed: %s", #expr, hipGetErrorString(e__)); \
    } while (0)

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }
__device__ __forceinline__ float to_f32(f16_t v) { return (float)v; }

template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }
template <> __device__ __forceinline__ f16_t from_f32<f16_t>(float v) { return (f16_t)v; }

// Accesses to data that a launch touches once (activation rows in, result rows out) carry the non-temporal hint:
// they do not displace tables, weights and kernels that other waves still need from L2, and the results leave no
// dirty lines behind for the end of the kernel.  Data that is read again soon (weights, k, rows handed to the next
// launch of the same call) keeps ordinary accesses.
typedef uint32_t stream_u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t stream_u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 load_stream16(const void *p)
{
    const stream_u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const stream_u32x4 *>(p));
    return make_uint4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ uint2 load_stream8(const void *p)
{
    const stream_u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const stream_u32x2 *>(p));
    return make_uint2(v[0], v[1]);
}
__device__ __forceinline__ uint32_t load_stream4(const void *p) { return __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(p)); }
__device__ __forceinline__ void store_stream16(void *p, uint4 v)
{
    __builtin_nontemporal_store((stream_u32x4){v.x, v.y, v.z, v.w}, reinterpret_cast<stream_u32x4 *>(p));
}
__device__ __forceinline__ void store_stream8(void *p, uint2 v)
{
    __builtin_nontemporal_store((stream_u32x2){v.x, v.y}, reinterpret_cast<stream_u32x2 *>(p));
}
__device__ __forceinline__ void store_stream4(void *p, uint32_t v) { __builtin_nontemporal_store(v, reinterpret_cast<uint32_t *>(p)); }

// exp(+2*pi*i*e/N) for 0 <= e < N.  sincospif reduces its argument exactly, and
// 2e/N is exact in fp32 whenever N is a power of two (N <= 2^24).
__device__ __forceinline__ float2 omega(int e, int N)
{
    float s, c;
    sincospif(2.0f * (float)e / (float)N, &s, &c);
    return make_float2(c, s);
}

__device__ __forceinline__ float2 cmul(float2 a, float2 b)
{
    return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}

__device__ __forceinline__ float gelu_erf(float z) { return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f)); }

__device__ __forceinline__ float activate(float z, int act)
{
    if (act == 1) return z > 0.0f ? z : 0.0f;
    if (act == 2) return gelu_erf(z);
    return z;
}

static inline size_t dtype_size(monarch_dtype dt) { return dt == MONARCH_F32 ? 4 : 2; }

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace monarch
