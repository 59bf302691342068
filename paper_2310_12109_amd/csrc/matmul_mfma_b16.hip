// Order-2 Monarch matrix multiply y = P L P R P x for the square case b = 16 (N = 256), fp32 or bf16
// tensors, fp32 arithmetic (Sec. 3.1).  HBM-bound: 2 KB (fp32) of traffic and 16 KFLOP per vector.
//
// Persistent waves, each on its own tile of 16 vectors; vectors sit on the MFMA column index.
//   stage 1, block a:  T_a[i, v] = sum_c R_a[i, c] x[v][16c + a]     (16x16x4 fp32 MFMA, 4 k-steps)
//   stage 2, block i:  Y_i[k, v] = sum_a L_i[k, a] T_a[i, v]
// Both block-diagonal factors live in registers for the whole kernel (128 VGPRs).  The first P is
// the operand gather (x is loaded as 16-byte pieces x[v][16c + 4q .. +3], one piece feeding the same
// k-step of four blocks); the middle P is the index map of the per-wave LDS tile, written as
// (row i, column a) by stage 1 and read row by row by stage 2; stage 2 overwrites row i in place with
// (row i, column k), and the last P is the index map of the read that feeds the coalesced 16-byte
// stores.  The next tile's x is requested as soon as stage 1 has consumed the current one.
#include "kernels.h"

namespace monarch {

typedef __attribute__((ext_vector_type(4))) float f32x4;

namespace mm16 {

constexpr int B = 16, N = 256, TV = 16;   // block size, vector length, vectors per tile
// Tile element (v, row, col) sits at v * LD + row * RS + col.  RS = 18 and LD = 3 (mod 32) keep every
// access pattern below at two or three lanes per LDS bank.
constexpr int RS = 18, LD = B * RS + 3;
constexpr int WAVES = 4;
constexpr size_t LDS_BYTES = sizeof(float) * WAVES * TV * LD;

__device__ __forceinline__ f32x4 mfma(float a, float b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// Orders the LDS traffic of one wave: the hardware runs a wave's LDS operations in order, the
// compiler must not move them across this point.
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// four consecutive elements as floats (float: 16-byte aligned; bf16: 8-byte aligned)
__device__ __forceinline__ f32x4 ld4(const float *p) { return *reinterpret_cast<const f32x4 *>(p); }
__device__ __forceinline__ f32x4 ld4(const bf16_t *p)
{
    const uint2 w = *reinterpret_cast<const uint2 *>(p);
    return f32x4{__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xffff0000u), __uint_as_float(w.y << 16),
                 __uint_as_float(w.y & 0xffff0000u)};
}
__device__ __forceinline__ void st4(float *p, f32x4 v) { *reinterpret_cast<f32x4 *>(p) = v; }
__device__ __forceinline__ void st4(bf16_t *p, f32x4 v)
{
    const bf16_t h[4] = {from_f32<bf16_t>(v[0]), from_f32<bf16_t>(v[1]), from_f32<bf16_t>(v[2]), from_f32<bf16_t>(v[3])};
    *reinterpret_cast<uint2 *>(p) = *reinterpret_cast<const uint2 *>(h);
}

// the same for vectors that a launch writes once (y: a wave instruction covers whole cache lines): streaming stores.
// (The loads of x take a cache line in four instructions of a lane and need it to stay in the cache meanwhile:
// with streaming loads the kernel ran 1.7 times slower.)
__device__ __forceinline__ void st4s(float *p, f32x4 v) { __builtin_nontemporal_store(v, reinterpret_cast<f32x4 *>(p)); }
__device__ __forceinline__ void st4s(bf16_t *p, f32x4 v) { st4(p, v); }   // 8 bytes per lane: no gain measured

// T: type of x, R, L and y in memory; registers, LDS and the arithmetic are float.
template <typename T>
__global__ __launch_bounds__(256, 2) void monarch_b16_kernel(const T *__restrict__ x, const T *__restrict__ R,
                                                             const T *__restrict__ L, T *__restrict__ y,
                                                             int64_t batch)
{
    extern __shared__ __attribute__((aligned(16))) float tiles[];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63, l16 = lane & 15, kg = lane >> 4;
    float *tile = tiles + wave * (TV * LD);

    // A operands: k-step s of block m holds W_m[row l16][4kg + s]
    float Rw[B][4], Lw[B][4];
#pragma unroll
    for (int m = 0; m < B; ++m) {
        const f32x4 r = ld4(R + (m * B + l16) * B + 4 * kg);
        const f32x4 l = ld4(L + (m * B + l16) * B + 4 * kg);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            Rw[m][s] = r[s];
            Lw[m][s] = l[s];
        }
    }

    const int64_t ntiles = (batch + TV - 1) / TV;
    const int64_t stride = (int64_t)gridDim.x * WAVES;
    int64_t t = (int64_t)blockIdx.x * WAVES + wave;
    if (t >= ntiles) return;

    // x[v][16(4kg + s) + 4q .. +3]: component e of piece (s, q) is the k-step-s operand of block 4q + e.
    // Columns past the batch are clamped to its last vector: computed, never stored.
    f32x4 xq[4][4];
    auto request = [&](int64_t tile_index) {
        int64_t v = tile_index * TV + l16;
        if (v >= batch) v = batch - 1;
        const T *xrow = x + v * N + 64 * kg;
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int q = 0; q < 4; ++q) xq[s][q] = ld4(xrow + 16 * s + 4 * q);
    };
    request(t);

    float *mine = tile + l16 * LD;   // this lane's vector (MFMA column)
    for (; t < ntiles; t += stride) {
        const int64_t v0 = t * TV;
        // stage 1: rows i = 4kg + r of block a, column v  ->  (v, row i, col a)
#pragma unroll
        for (int a = 0; a < B; ++a) {
            f32x4 acc = {0, 0, 0, 0};
#pragma unroll
            for (int s = 0; s < 4; ++s) acc = mfma(Rw[a][s], xq[s][a >> 2][a & 3], acc);
#pragma unroll
            for (int r = 0; r < 4; ++r) mine[(4 * kg + r) * RS + a] = acc[r];
        }
        request(t + stride);   // in flight during stage 2 and the stores
        wave_sync();
        // stage 2: block i contracts a = 4kg + s, read from row i; rows k = 4kg + r of the result go
        // back into row i (columns 4kg .. 4kg + 3 of row i are read and written by this lane only)
#pragma unroll
        for (int i = 0; i < B; ++i) {
            f32x4 acc = {0, 0, 0, 0};
#pragma unroll
            for (int s = 0; s < 4; ++s) acc = mfma(Lw[i][s], mine[i * RS + 4 * kg + s], acc);
#pragma unroll
            for (int r = 0; r < 4; ++r) mine[i * RS + 4 * kg + r] = acc[r];
        }
        wave_sync();
        // y[v][16k + i] = (v, row i, col k).  Lane -> (k = lane / 4, i = 4 (lane % 4) + e): one 16-byte
        // (bf16: 8-byte) store per lane, a whole vector (contiguous) per instruction.
        const float *src = tile + (4 * (lane & 3)) * RS + (lane >> 2);
#pragma unroll
        for (int vv = 0; vv < TV; ++vv) {
            f32x4 val;
#pragma unroll
            for (int e = 0; e < 4; ++e) val[e] = src[vv * LD + e * RS];
            if (v0 + vv < batch) st4s(y + (v0 + vv) * N + 4 * lane, val);
        }
        wave_sync();
    }
}

}  // namespace mm16

bool matmul_mfma_b16_supported(int nbR, int r_out, int r_in, int nbL, int l_out, int l_in, monarch_dtype dt)
{
    return (dt == MONARCH_F32 || dt == MONARCH_BF16) && nbR == 16 && r_out == 16 && r_in == 16 && nbL == 16 && l_out == 16 && l_in == 16;
}

int launch_matmul_mfma_b16(const void *x, const void *R, const void *L, void *y, int64_t batch, monarch_dtype dt,
                           hipStream_t s)
{
    int dev = 0, ncu = 0;
    MONARCH_HIP_CHECK(hipGetDevice(&dev));
    MONARCH_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
    const int64_t ntiles = (batch + mm16::TV - 1) / mm16::TV;
    const int64_t wgs_needed = (ntiles + mm16::WAVES - 1) / mm16::WAVES;
    const int64_t slots = 2 * (int64_t)ncu;   // two workgroups (8 waves) per compute unit
    const unsigned grid = (unsigned)(wgs_needed < slots ? wgs_needed : slots);
    if (dt == MONARCH_F32) {
        MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)mm16::monarch_b16_kernel<float>,
                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)mm16::LDS_BYTES));
        hipLaunchKernelGGL(mm16::monarch_b16_kernel<float>, dim3(grid), dim3(256), mm16::LDS_BYTES, s, (const float *)x,
                           (const float *)R, (const float *)L, (float *)y, batch);
    } else {
        MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)mm16::monarch_b16_kernel<bf16_t>,
                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)mm16::LDS_BYTES));
        hipLaunchKernelGGL(mm16::monarch_b16_kernel<bf16_t>, dim3(grid), dim3(256), mm16::LDS_BYTES, s, (const bf16_t *)x,
                           (const bf16_t *)R, (const bf16_t *)L, (bf16_t *)y, batch);
    }
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

}  // namespace monarch
