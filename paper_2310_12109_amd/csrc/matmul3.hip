// General (learned) order-3 Monarch product and its gradients (Sec. 3.1 and the appendix definition of order-p
// Monarch matrices, p = 3).  N = b^3, three block-diagonal factors B1, B2, B3 of b^2 blocks of b x b, B1 applied
// first:  M = P^R B3 P_(b,b^2,N) B2 P_(b^2,b^3,N) B1 P^R.  With the input index j = j2 b^2 + j1 b + j0 and the
// output index m = m2 b^2 + m1 b + m0 (block (p, q) is block p b + q):
//   t1[(j0,j1), m0] = sum_j2 B1[(j0,j1)][m0, j2] x[j2, j1, j0]
//   t2[(m0,j0), m1] = sum_j1 B2[(m0,j0)][m1, j1] t1[(j0,j1), m0]
//   y[m2, m1, m0]   = sum_j0 B3[(m0,m1)][m2, j0] t2[(m0,j0), m1]
// The permutations are LDS index maps; rows stay on chip between the factors.  fp32 arithmetic on tiles of rows
// in LDS (the order-3 counterpart of the shape-generic order-2 kernels).
#include "kernels.h"

namespace monarch {

namespace mm3 {

constexpr int THREADS = 256;

// Where factor S (1, 2, 3) reads the element that meets column c of row (p, q, .) of its blocks.
template <int S>
__device__ __forceinline__ int in_index(int p, int q, int c, int b)
{
    if (S == 1) return (c * b + q) * b + p;   // x[j2 = c, j1 = q, j0 = p]
    if (S == 2) return (q * b + c) * b + p;   // t1[(j0 = q, j1 = c), m0 = p]
    return (p * b + c) * b + q;               // t2[(m0 = p, j0 = c), m1 = q]
}

// One factor on TV rows: out[v][(p, q, r)] = sum_c W[(p, q)][r, c] in[v][in_index(p, q, c)]; the last factor
// writes y[r, q, p] instead.
template <typename T, int TV, int S>
__device__ __forceinline__ void factor(const float *in, float *out, int N, int b, const T *__restrict__ W)
{
    for (int o = threadIdx.x; o < N; o += THREADS) {
        const int r = o % b, pq = o / b, q = pq % b, p = pq / b;
        float acc[TV];
#pragma unroll
        for (int v = 0; v < TV; ++v) acc[v] = 0.0f;
        const T *w = W + (size_t)o * b;
        for (int c = 0; c < b; ++c) {
            const float wv = to_f32(w[c]);
            const int at = in_index<S>(p, q, c, b);
#pragma unroll
            for (int v = 0; v < TV; ++v) acc[v] = fmaf(wv, in[v * N + at], acc[v]);
        }
        const int to = S == 3 ? (r * b + q) * b + p : o;
#pragma unroll
        for (int v = 0; v < TV; ++v) out[v * N + to] = acc[v];
    }
}

template <typename T, int TV>
__global__ __launch_bounds__(THREADS) void forward_kernel(const T *__restrict__ x, const T *__restrict__ B1,
                                                          const T *__restrict__ B2, const T *__restrict__ B3,
                                                          T *__restrict__ y, int64_t batch, int b)
{
    extern __shared__ float lds[];
    const int N = b * b * b;
    float *a = lds, *t = lds + TV * N;
    const int64_t ntiles = (batch + TV - 1) / TV;
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t v0 = tile * TV;
        for (int idx = threadIdx.x; idx < TV * N; idx += THREADS) {
            const int v = idx / N;
            a[idx] = v0 + v < batch ? to_f32(x[v0 * N + idx]) : 0.0f;
        }
        __syncthreads();
        factor<T, TV, 1>(a, t, N, b, B1);
        __syncthreads();
        factor<T, TV, 2>(t, a, N, b, B2);
        __syncthreads();
        factor<T, TV, 3>(a, t, N, b, B3);
        __syncthreads();
        for (int idx = threadIdx.x; idx < TV * N; idx += THREADS)
            if (v0 + idx / N < batch) y[v0 * N + idx] = from_f32<T>(t[idx]);
        __syncthreads();
    }
}

// Gradients on tiles of TV rows (four buffers of TV rows of N floats in LDS: x, t1, t2 and the running gradient).
// Adjoint of each step, last step first; every entry of dB1, dB2, dB3 is summed over the rows of a tile in a
// register and receives one atomic add per tile.
template <typename T, int TV>
__global__ __launch_bounds__(THREADS) void backward_kernel(const T *__restrict__ x, const T *__restrict__ B1,
                                                           const T *__restrict__ B2, const T *__restrict__ B3,
                                                           const T *__restrict__ dy, T *__restrict__ dx,
                                                           float *__restrict__ dB1, float *__restrict__ dB2,
                                                           float *__restrict__ dB3, int64_t batch, int b)
{
    extern __shared__ float lds[];
    const int N = b * b * b;
    float *xs = lds, *t1 = xs + TV * N, *t2 = t1 + TV * N, *g = t2 + TV * N;
    const int64_t ntiles = (batch + TV - 1) / TV;
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t v0 = tile * TV;
        for (int idx = threadIdx.x; idx < TV * N; idx += THREADS) {
            const int v = idx / N, j = idx - v * N;
            const bool live = v0 + v < batch;   // rows past the end are zero: they add nothing to the sums
            xs[idx] = live ? to_f32(x[v0 * N + idx]) : 0.0f;
            // g3[(m0, m1), m2] = dy[m2, m1, m0]
            const int m0 = j % b, m1 = (j / b) % b, m2 = j / (b * b);
            g[v * N + (m0 * b + m1) * b + m2] = live ? to_f32(dy[v0 * N + idx]) : 0.0f;
        }
        __syncthreads();
        factor<T, TV, 1>(xs, t1, N, b, B1);
        __syncthreads();
        factor<T, TV, 2>(t1, t2, N, b, B2);
        __syncthreads();
        // dB3[(p, q)][r, c] += g3[(p, q), r] t2[(p, c), q]
        if (dB3)
            for (int e = threadIdx.x; e < N * b; e += THREADS) {
                const int c = e % b, o = e / b, pq = o / b, q = pq % b, p = pq / b;
                const int at = in_index<3>(p, q, c, b);
                float acc = 0.0f;
#pragma unroll
                for (int v = 0; v < TV; ++v) acc = fmaf(g[v * N + o], t2[v * N + at], acc);
                atomicAdd(dB3 + e, acc);
            }
        __syncthreads();
        // g2[(p, c), q] = sum_r B3[(p, q)][r, c] g3[(p, q), r]   -> over t2
        for (int o2 = threadIdx.x; o2 < N; o2 += THREADS) {
            const int q = o2 % b, pc = o2 / b, c = pc % b, p = pc / b;
            float acc[TV];
#pragma unroll
            for (int v = 0; v < TV; ++v) acc[v] = 0.0f;
            for (int r = 0; r < b; ++r) {
                const float w = to_f32(B3[(((size_t)p * b + q) * b + r) * b + c]);
#pragma unroll
                for (int v = 0; v < TV; ++v) acc[v] = fmaf(w, g[v * N + (p * b + q) * b + r], acc[v]);
            }
#pragma unroll
            for (int v = 0; v < TV; ++v) t2[v * N + o2] = acc[v];
        }
        __syncthreads();
        // dB2[(p, q)][r, c] += g2[(p, q), r] t1[(q, c), p]
        if (dB2)
            for (int e = threadIdx.x; e < N * b; e += THREADS) {
                const int c = e % b, o = e / b, pq = o / b, q = pq % b, p = pq / b;
                const int at = in_index<2>(p, q, c, b);
                float acc = 0.0f;
#pragma unroll
                for (int v = 0; v < TV; ++v) acc = fmaf(t2[v * N + o], t1[v * N + at], acc);
                atomicAdd(dB2 + e, acc);
            }
        __syncthreads();
        // g1[(q, c), p] = sum_r B2[(p, q)][r, c] g2[(p, q), r]   -> over g
        for (int o1 = threadIdx.x; o1 < N; o1 += THREADS) {
            const int p = o1 % b, qc = o1 / b, c = qc % b, q = qc / b;
            float acc[TV];
#pragma unroll
            for (int v = 0; v < TV; ++v) acc[v] = 0.0f;
            for (int r = 0; r < b; ++r) {
                const float w = to_f32(B2[(((size_t)p * b + q) * b + r) * b + c]);
#pragma unroll
                for (int v = 0; v < TV; ++v) acc[v] = fmaf(w, t2[v * N + (p * b + q) * b + r], acc[v]);
            }
#pragma unroll
            for (int v = 0; v < TV; ++v) g[v * N + o1] = acc[v];
        }
        __syncthreads();
        // dB1[(p, q)][r, c] += g1[(p, q), r] x[c, q, p]
        if (dB1)
            for (int e = threadIdx.x; e < N * b; e += THREADS) {
                const int c = e % b, o = e / b, pq = o / b, q = pq % b, p = pq / b;
                const int at = in_index<1>(p, q, c, b);
                float acc = 0.0f;
#pragma unroll
                for (int v = 0; v < TV; ++v) acc = fmaf(g[v * N + o], xs[v * N + at], acc);
                atomicAdd(dB1 + e, acc);
            }
        // dx[c, q, p] = sum_r B1[(p, q)][r, c] g1[(p, q), r]
        if (dx)
            for (int j = threadIdx.x; j < N; j += THREADS) {
                const int p = j % b, q = (j / b) % b, c = j / (b * b);
                float acc[TV];
#pragma unroll
                for (int v = 0; v < TV; ++v) acc[v] = 0.0f;
                for (int r = 0; r < b; ++r) {
                    const float w = to_f32(B1[(((size_t)p * b + q) * b + r) * b + c]);
#pragma unroll
                    for (int v = 0; v < TV; ++v) acc[v] = fmaf(w, g[v * N + (p * b + q) * b + r], acc[v]);
                }
#pragma unroll
                for (int v = 0; v < TV; ++v)
                    if (v0 + v < batch) dx[(v0 + v) * N + j] = from_f32<T>(acc[v]);
            }
        __syncthreads();
    }
}

__global__ void fill3_kernel(float *a, float *b, float *c, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        if (a) a[i] = 0.0f;
        if (b) b[i] = 0.0f;
        if (c) c[i] = 0.0f;
    }
}

static int compute_units(int *ncu)
{
    int dev = 0;
    MONARCH_HIP_CHECK(hipGetDevice(&dev));
    MONARCH_HIP_CHECK(hipDeviceGetAttribute(ncu, hipDeviceAttributeMultiprocessorCount, dev));
    return MONARCH_OK;
}

template <typename T>
static int launch_forward(const void *x, const void *B1, const void *B2, const void *B3, void *y, int64_t batch, int b,
                          hipStream_t s)
{
    const int N = b * b * b;
    // (more rows per tile: every weight read from L2 serves more rows)
    int tv = 8;
    while (tv > 1 && (size_t)2 * tv * N * sizeof(float) > 128 * 1024) tv >>= 1;
    const size_t lds = (size_t)2 * tv * N * sizeof(float);
    int ncu = 0;
    if (int rc = compute_units(&ncu)) return rc;
    const int64_t ntiles = (batch + tv - 1) / tv;
    int64_t grid = (int64_t)ncu * (lds <= 32 * 1024 ? 4 : lds <= 80 * 1024 ? 2 : 1);
    if (grid > ntiles) grid = ntiles;
#define MONARCH_LAUNCH_MM3(TVV)                                                                                  \
    do {                                                                                                         \
        auto kern = forward_kernel<T, TVV>;                                                                      \
        if (lds > 64 * 1024)                                                                                     \
            MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, \
                                                  (int)lds));                                                    \
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(THREADS), lds, s, (const T *)x, (const T *)B1,       \
                           (const T *)B2, (const T *)B3, (T *)y, batch, b);                                      \
    } while (0)
    switch (tv) {
    case 8: MONARCH_LAUNCH_MM3(8); break;
    case 4: MONARCH_LAUNCH_MM3(4); break;
    case 2: MONARCH_LAUNCH_MM3(2); break;
    default: MONARCH_LAUNCH_MM3(1); break;
    }
#undef MONARCH_LAUNCH_MM3
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

template <typename T>
static int launch_backward(const void *x, const void *B1, const void *B2, const void *B3, const void *dy, void *dx,
                           float *dB1, float *dB2, float *dB3, int64_t batch, int b, hipStream_t s)
{
    const int N = b * b * b;
    if (dB1 || dB2 || dB3) hipLaunchKernelGGL(fill3_kernel, dim3(64), dim3(256), 0, s, dB1, dB2, dB3, (size_t)N * b);
    if (batch > 0) {
        int ncu = 0;
        if (int rc = compute_units(&ncu)) return rc;
        int tv = 8;
        while (tv > 1 && (size_t)4 * tv * N * sizeof(float) > 128 * 1024) tv >>= 1;
        const size_t lds = (size_t)4 * tv * N * sizeof(float);
        const int64_t ntiles = (batch + tv - 1) / tv;
        int64_t grid = (int64_t)ncu * (lds <= 40 * 1024 ? 4 : lds <= 80 * 1024 ? 2 : 1);
        if (grid > ntiles) grid = ntiles;
#define MONARCH_LAUNCH_MM3B(TVV)                                                                                  \
    do {                                                                                                          \
        auto kern = backward_kernel<T, TVV>;                                                                      \
        if (lds > 64 * 1024)                                                                                      \
            MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, \
                                                  (int)lds));                                                     \
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(THREADS), lds, s, (const T *)x, (const T *)B1,        \
                           (const T *)B2, (const T *)B3, (const T *)dy, (T *)dx, dB1, dB2, dB3, batch, b);        \
    } while (0)
        switch (tv) {
        case 8: MONARCH_LAUNCH_MM3B(8); break;
        case 4: MONARCH_LAUNCH_MM3B(4); break;
        case 2: MONARCH_LAUNCH_MM3B(2); break;
        default: MONARCH_LAUNCH_MM3B(1); break;
        }
#undef MONARCH_LAUNCH_MM3B
    }
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

}  // namespace mm3

// ---- b = 16 (N = 4096), forward, on the matrix cores ---------------------------------------------------
// A workgroup of 8 waves holds a tile of 8 rows in LDS (a tile of 16 would not fit) and works in place: in every
// stage a block reads the 16 elements of a row that it contracts and writes its 16 results to the same places
// (element (d2, d1, d0) of a row sits at d2 S2 + d1 S1 + d0, the digits being (j2, j1, j0) before the first factor,
// (m0, j1, j0), (m0, m1, j0) and (m0, m1, m2) after the first, second and third), so the permutations cost nothing
// and only the store reverses the digits.  Rows sit on the MFMA column index (columns 8..15 repeat rows 0..7); the
// weights, 3 x 256 KB, do not fit on chip: every block's 16 x 16 matrix is read from L2 as the A operand of four
// 16x16x4 fp32 MFMAs by the wave that owns the block (32 blocks per wave and stage).  The strides S1 = 18,
// S2 = 290 and the row pitch (1 mod 64) keep the operand reads of the first two stages free of bank conflicts.
namespace mm3b16 {

typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int B = 16, N = 4096, TV = 8, THREADS = 1024, WAVES = 16;
constexpr int S1 = 18, S2 = 290, ROWP = 4673;
constexpr size_t LDS_BYTES = sizeof(float) * TV * ROWP;

__device__ __forceinline__ f32x4 mfma(float a, float b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}
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

// One factor in place.  Block (p, q) contracts the digit that has stride SK in the tile; its other two digits sit
// at `at(p, q)`.  Lane (n = lane % 16, kg = lane / 16): row n % 8 of the tile, contraction indices 4 kg + s.
template <typename T, int SK, typename At>
__device__ __forceinline__ void stage(float *tile, const T *__restrict__ W, int wave, int lane, At at)
{
    const int l16 = lane & 15, kg = lane >> 4;
    float *mine = tile + (l16 & 7) * ROWP;
    // the weights of the next eight blocks are requested while the current eight are multiplied: the latency of L2
    // is paid once per stage, not once per block
    constexpr int NB = 256 / WAVES, G = 8;
    f32x4 w[2][G];
    // (the pointer passes through an empty asm that also names the latest result, so that the compiler keeps each
    // group's requests where they are written instead of hoisting all 32 to the top, which would need 128 registers)
    float anchor = 0.0f;
    auto request = [&](int g, f32x4 (&dst)[G]) {
        const T *src = W;
        asm volatile("" : "+s"(src) : "v"(anchor));
#pragma unroll
        for (int u = 0; u < G; ++u) dst[u] = ld4(src + ((size_t)(wave * NB + g * G + u) * B + l16) * B + 4 * kg);   // W[blk][row l16][4 kg .. + 3]
    };
    request(0, w[0]);
#pragma unroll
    for (int g = 0; g < NB / G; ++g) {
        if (g + 1 < NB / G) request(g + 1, w[(g + 1) & 1]);
#pragma unroll
        for (int u = 0; u < G; u += 2) {   // two blocks at a time: their accumulators take turns
            const int blk = wave * NB + g * G + u;
            float *e0 = mine + at(blk >> 4, blk & 15), *e1 = mine + at((blk + 1) >> 4, (blk + 1) & 15);
            float b0v[4], b1v[4];
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                b0v[s] = e0[(4 * kg + s) * SK];
                b1v[s] = e1[(4 * kg + s) * SK];
            }
            f32x4 acc0 = {0, 0, 0, 0}, acc1 = {0, 0, 0, 0};
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                acc0 = mfma(w[g & 1][u][s], b0v[s], acc0);
                acc1 = mfma(w[g & 1][u + 1][s], b1v[s], acc1);
            }
            // rows 4 kg + r of each block's result, column = row n of the tile: back where the inputs were
            if (l16 < TV) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    e0[(4 * kg + r) * SK] = acc0[r];
                    e1[(4 * kg + r) * SK] = acc1[r];
                }
            }
            anchor = acc1[0];
        }
    }
}

template <typename T>
__global__ __launch_bounds__(THREADS) void forward_kernel(const T *__restrict__ x, const T *__restrict__ B1,
                                                          const T *__restrict__ B2, const T *__restrict__ B3,
                                                          T *__restrict__ y, int64_t batch)
{
    extern __shared__ __attribute__((aligned(16))) float tile[];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int64_t ntiles = (batch + TV - 1) / TV;
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int64_t v0 = t * TV;
        // rows in: 16 pieces of 4 elements per thread (a piece never crosses a digit d1)
#pragma unroll 4
        for (int it = 0; it < TV * N / 4 / THREADS; ++it) {
            const int piece = it * THREADS + threadIdx.x, v = piece / (N / 4), j = 4 * (piece % (N / 4));
            int64_t r = v0 + v;
            if (r >= batch) r = batch - 1;   // (rows past the end: computed, never stored)
            const f32x4 val = ld4(x + r * N + j);
            float *d = tile + v * ROWP + (j >> 8) * S2 + ((j >> 4) & 15) * S1 + (j & 15);
            d[0] = val[0]; d[1] = val[1]; d[2] = val[2]; d[3] = val[3];
        }
        __syncthreads();
        // factor 1: block (j0, j1) contracts j2 (stride S2); m0 takes j2's place
        stage<T, S2>(tile, B1, wave, lane, [](int p, int q) { return q * S1 + p; });
        __syncthreads();
        // factor 2: block (m0, j0) contracts j1 (stride S1); m1 takes j1's place
        stage<T, S1>(tile, B2, wave, lane, [](int p, int q) { return p * S2 + q; });
        __syncthreads();
        // factor 3: block (m0, m1) contracts j0 (stride 1); m2 takes j0's place
        stage<T, 1>(tile, B3, wave, lane, [](int p, int q) { return p * S2 + q * S1; });
        __syncthreads();
        // rows out: y[m2, m1, m0] sits at (m0, m1, m2); a thread stores m0 = 4 g .. 4 g + 3 of one (m2, m1)
#pragma unroll 4
        for (int it = 0; it < TV * N / 4 / THREADS; ++it) {
            const int piece = it * THREADS + threadIdx.x, v = piece / (N / 4), j = 4 * (piece % (N / 4));
            const int m2 = j >> 8, m1 = (j >> 4) & 15, m0 = j & 15;
            const float *sp = tile + v * ROWP + m0 * S2 + m1 * S1 + m2;
            if (v0 + v < batch) st4(y + (v0 + v) * N + j, f32x4{sp[0], sp[S2], sp[2 * S2], sp[3 * S2]});
        }
        __syncthreads();
    }
}

template <typename T>
static int launch(const void *x, const void *B1, const void *B2, const void *B3, void *y, int64_t batch, hipStream_t s)
{
    int ncu = 0;
    if (int rc = mm3::compute_units(&ncu)) return rc;
    const int64_t ntiles = (batch + TV - 1) / TV;
    int64_t grid = ncu;   // one workgroup (150 KB of LDS) per compute unit
    if (grid > ntiles) grid = ntiles;
    auto kern = forward_kernel<T>;
    MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_BYTES));
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(THREADS), LDS_BYTES, s, (const T *)x, (const T *)B1, (const T *)B2,
                       (const T *)B3, (T *)y, batch);
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}


// ---- b = 16 (N = 4096), gradients, on the matrix cores ------------------------------------------------
// Two tiles of 4 rows in LDS: `fw` takes x and the forward factors in place, `gr` takes dy (digits reversed, the
// layout the forward leaves its result in) and the transposed factors in place, last factor first.  Where the
// gradient of a factor's blocks is formed, its two ingredients sit at the same places of the two tiles:
//   dB3[(m0,m1)][m2, j0] += g3[m0,m1,m2] t2[m0,m1,j0]      g2 = B3^T g3   (digit of stride 1)
//   dB2[(m0,j0)][m1, j1] += g2[m0,m1,j0] t1[m0,j1,j0]      g1 = B2^T g2   (digit of stride S1)
//   dB1[(j0,j1)][m0, j2] += g1[m0,j1,j0] x[j2,j1,j0]       dx = B1^T g1   (digit of stride S2)
// and the sum over the four rows of a tile is ONE 16x16x4 MFMA per block (A = the gradient's 16 values of the four
// rows, B = the forward values).  A wave keeps the 16 x 16 sums of its 16 blocks in registers over all tiles of the
// workgroup and adds them to global memory once at the end (atomics: workgroups share the result).  Registers hold
// the sums of one factor only, so each factor's gradient is a launch of its own, which recomputes the forward and
// transposed stages it needs (7 stage passes in all instead of 5).
constexpr int TVB = 4, NBW = 256 / WAVES;
constexpr size_t LDS_BYTES_B = sizeof(float) * 2 * TVB * ROWP;

// One factor in place on a tile of TVB rows (columns 4..15 of the MFMA repeat the rows).  TRANS: the transposed
// block, A[c][r] = W[r][c].
template <typename T, int SK, bool TRANS, typename At>
__device__ __forceinline__ void stage4(float *tile, const T *__restrict__ W, int wave, int lane, At at)
{
    const int l16 = lane & 15, kg = lane >> 4;
    float *mine = tile + (l16 & (TVB - 1)) * ROWP;
    constexpr int G = 4;
    f32x4 w[2][G];
    float anchor = 0.0f;
    auto request = [&](int g, f32x4 (&dst)[G]) {
        const T *src = W;
        asm volatile("" : "+s"(src) : "v"(anchor));
#pragma unroll
        for (int u = 0; u < G; ++u) {
            const size_t blk = (size_t)(wave * NBW + g * G + u);
            if constexpr (TRANS) {
#pragma unroll
                for (int s2 = 0; s2 < 4; ++s2) dst[u][s2] = to_f32(src[(blk * B + 4 * kg + s2) * B + l16]);   // W[blk][4 kg + s][l16]
            } else {
                dst[u] = ld4(src + (blk * B + l16) * B + 4 * kg);                                              // W[blk][l16][4 kg ..]
            }
        }
    };
    request(0, w[0]);
#pragma unroll
    for (int g = 0; g < NBW / G; ++g) {
        if (g + 1 < NBW / G) request(g + 1, w[(g + 1) & 1]);
#pragma unroll
        for (int u = 0; u < G; u += 2) {
            const int blk = wave * NBW + g * G + u;
            float *e0 = mine + at(blk >> 4, blk & 15), *e1 = mine + at((blk + 1) >> 4, (blk + 1) & 15);
            float b0v[4], b1v[4];
#pragma unroll
            for (int s2 = 0; s2 < 4; ++s2) {
                b0v[s2] = e0[(4 * kg + s2) * SK];
                b1v[s2] = e1[(4 * kg + s2) * SK];
            }
            f32x4 acc0 = {0, 0, 0, 0}, acc1 = {0, 0, 0, 0};
#pragma unroll
            for (int s2 = 0; s2 < 4; ++s2) {
                acc0 = mfma(w[g & 1][u][s2], b0v[s2], acc0);
                acc1 = mfma(w[g & 1][u + 1][s2], b1v[s2], acc1);
            }
            if (l16 < TVB) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    e0[(4 * kg + r) * SK] = acc0[r];
                    e1[(4 * kg + r) * SK] = acc1[r];
                }
            }
            anchor = acc1[0];
        }
    }
}

// sums[u][i] += sum over the tile's rows v of gr_v[r = 4 kg + i] fw_v[c = l16] for block u of this wave
template <int SK, typename At>
__device__ __forceinline__ void outer4(const float *gr, const float *fw, f32x4 (&sums)[NBW], int wave, int lane, At at)
{
    const int l16 = lane & 15, kg = lane >> 4;
#pragma unroll
    for (int u = 0; u < NBW; ++u) {
        const int blk = wave * NBW + u;
        const int off = kg * ROWP + at(blk >> 4, blk & 15) + l16 * SK;   // lane group kg = row kg of the tile
        sums[u] = mfma(gr[off], fw[off], sums[u]);
    }
}

// WHICH = 3, 2: the gradient of that factor's blocks; WHICH = 1: dB1 (if given) and dx (if given).
template <typename T, int WHICH>
__global__ __launch_bounds__(THREADS) void backward_kernel(const T *__restrict__ x, const T *__restrict__ B1,
                                                           const T *__restrict__ B2, const T *__restrict__ B3,
                                                           const T *__restrict__ dy, T *__restrict__ dx,
                                                           float *__restrict__ dB, int64_t batch)
{
    extern __shared__ __attribute__((aligned(16))) float tiles[];
    float *fw = tiles, *gr = tiles + TVB * ROWP;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const auto at1 = [](int p, int q) { return q * S1 + p; };         // block (j0, j1), digit of stride S2
    const auto at2 = [](int p, int q) { return p * S2 + q; };         // block (m0, j0), digit of stride S1
    const auto at3 = [](int p, int q) { return p * S2 + q * S1; };    // block (m0, m1), digit of stride 1
    f32x4 sums[NBW];
#pragma unroll
    for (int u = 0; u < NBW; ++u) sums[u] = f32x4{0, 0, 0, 0};
    const bool need_fw = dB != nullptr;
    const int64_t ntiles = (batch + TVB - 1) / TVB;
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int64_t v0 = t * TVB;
        // rows in (zeros past the end of the batch: they add nothing to the sums)
#pragma unroll 4
        for (int it = 0; it < TVB * N / 4 / THREADS; ++it) {
            const int piece = it * THREADS + threadIdx.x, v = piece / (N / 4), j = 4 * (piece % (N / 4));
            const bool live = v0 + v < batch;
            const int64_t r = live ? v0 + v : 0;
            const int d2 = j >> 8, d1 = (j >> 4) & 15, d0 = j & 15;
            if (need_fw) {
                f32x4 val = ld4(x + r * N + j);
                if (!live) val = f32x4{0, 0, 0, 0};
                float *d = fw + v * ROWP + d2 * S2 + d1 * S1 + d0;
                d[0] = val[0]; d[1] = val[1]; d[2] = val[2]; d[3] = val[3];
            }
            f32x4 g = ld4(dy + r * N + j);   // dy[m2 = d2, m1 = d1, m0 = d0 .. d0 + 3] sits at (m0, m1, m2)
            if (!live) g = f32x4{0, 0, 0, 0};
            float *e = gr + v * ROWP + d0 * S2 + d1 * S1 + d2;
            e[0] = g[0]; e[S2] = g[1]; e[2 * S2] = g[2]; e[3 * S2] = g[3];
        }
        __syncthreads();
        if constexpr (WHICH == 3) {
            stage4<T, S2, false>(fw, B1, wave, lane, at1);
            __syncthreads();
            stage4<T, S1, false>(fw, B2, wave, lane, at2);
            __syncthreads();
            outer4<1>(gr, fw, sums, wave, lane, at3);
        } else if constexpr (WHICH == 2) {
            stage4<T, S2, false>(fw, B1, wave, lane, at1);
            stage4<T, 1, true>(gr, B3, wave, lane, at3);
            __syncthreads();
            outer4<S1>(gr, fw, sums, wave, lane, at2);
        } else {
            stage4<T, 1, true>(gr, B3, wave, lane, at3);
            __syncthreads();
            stage4<T, S1, true>(gr, B2, wave, lane, at2);
            __syncthreads();
            if (dB) outer4<S2>(gr, fw, sums, wave, lane, at1);
            if (dx) {   // (the blocks of the last transposed factor are the blocks whose sums this wave just formed)
                stage4<T, S2, true>(gr, B1, wave, lane, at1);
                __syncthreads();
#pragma unroll 4
                for (int it = 0; it < TVB * N / 4 / THREADS; ++it) {
                    const int piece = it * THREADS + threadIdx.x, v = piece / (N / 4), j = 4 * (piece % (N / 4));
                    const float *sp = gr + v * ROWP + (j >> 8) * S2 + ((j >> 4) & 15) * S1 + (j & 15);
                    if (v0 + v < batch) st4(dx + (v0 + v) * N + j, f32x4{sp[0], sp[1], sp[2], sp[3]});
                }
            }
        }
        __syncthreads();
    }
    if (dB) {
        const int l16 = lane & 15, kg = lane >> 4;
#pragma unroll
        for (int u = 0; u < NBW; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i) atomicAdd(dB + ((size_t)(wave * NBW + u) * B + 4 * kg + i) * B + l16, sums[u][i]);
    }
}

template <typename T>
static int launch_backward(const void *x, const void *B1, const void *B2, const void *B3, const void *dy, void *dx,
                           float *dB1, float *dB2, float *dB3, int64_t batch, hipStream_t s)
{
    if (dB1 || dB2 || dB3)
        hipLaunchKernelGGL(mm3::fill3_kernel, dim3(64), dim3(256), 0, s, dB1, dB2, dB3, (size_t)N * B);
    if (batch > 0) {
        int ncu = 0;
        if (int rc = mm3::compute_units(&ncu)) return rc;
        const int64_t ntiles = (batch + TVB - 1) / TVB;
        int64_t grid = ncu;   // one workgroup (two tiles, 150 KB of LDS) per compute unit
        if (grid > ntiles) grid = ntiles;
#define MONARCH_LAUNCH_MM3B16(WHICHV, DXV, DBV)                                                                    \
    do {                                                                                                           \
        auto kern = backward_kernel<T, WHICHV>;                                                                    \
        MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,      \
                                              (int)LDS_BYTES_B));                                                  \
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(THREADS), LDS_BYTES_B, s, (const T *)x, (const T *)B1, \
                           (const T *)B2, (const T *)B3, (const T *)dy, (T *)(DXV), (float *)(DBV), batch);        \
    } while (0)
        if (dB3) MONARCH_LAUNCH_MM3B16(3, nullptr, dB3);
        if (dB2) MONARCH_LAUNCH_MM3B16(2, nullptr, dB2);
        if (dB1 || dx) MONARCH_LAUNCH_MM3B16(1, dx, dB1);
#undef MONARCH_LAUNCH_MM3B16
    }
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

}  // namespace mm3b16

bool matmul3_fits(int b) { return b >= 1 && b <= 16; }   // four rows of b^3 floats in 64 KB of LDS

int launch_matmul3(const void *x, const void *B1, const void *B2, const void *B3, void *y, int64_t batch, int b,
                   monarch_dtype dt, hipStream_t s)
{
    if (batch == 0) return MONARCH_OK;
    if (b == 16) {
        if (dt == MONARCH_F32) return mm3b16::launch<float>(x, B1, B2, B3, y, batch, s);
        return mm3b16::launch<bf16_t>(x, B1, B2, B3, y, batch, s);
    }
    if (dt == MONARCH_F32) return mm3::launch_forward<float>(x, B1, B2, B3, y, batch, b, s);
    return mm3::launch_forward<bf16_t>(x, B1, B2, B3, y, batch, b, s);
}

int launch_matmul3_backward(const void *x, const void *B1, const void *B2, const void *B3, const void *dy, void *dx,
                            float *dB1, float *dB2, float *dB3, int64_t batch, int b, monarch_dtype dt, hipStream_t s)
{
    if (b == 16) {
        if (dt == MONARCH_F32) return mm3b16::launch_backward<float>(x, B1, B2, B3, dy, dx, dB1, dB2, dB3, batch, s);
        return mm3b16::launch_backward<bf16_t>(x, B1, B2, B3, dy, dx, dB1, dB2, dB3, batch, s);
    }
    if (dt == MONARCH_F32) return mm3::launch_backward<float>(x, B1, B2, B3, dy, dx, dB1, dB2, dB3, batch, b, s);
    return mm3::launch_backward<bf16_t>(x, B1, B2, B3, dy, dx, dB1, dB2, dB3, batch, b, s);
}

}  // namespace monarch
