// General (learned) order-p Monarch product and its gradients (Sec. 3.1: higher-order Monarch matrices; appendix
// definition of the p-variate Monarch matrix and the lemma that numbers the blocks of its factors).  N = b^p,
// p block-diagonal factors B_1 .. B_p of b^(p-1) blocks of b x b, B_1 applied first:
//   M = P^R B_p P B_(p-1) P ... P B_1 P^R,      P^R the reversal of the p base-b digits of an index.
// With the input index j = sum_a j_a b^a and the output index m = sum_a m_a b^a, factor s consumes the input digit
// j_(p-s) and produces the output digit m_(s-1); its block is numbered by the digits produced so far followed by the
// input digits not yet consumed, most significant first, and so is the vector between the factors:
//   t_s[(m_0 .. m_(s-2), j_0 .. j_(p-s-1)), m_(s-1)]
//       = sum_c B_s[(m_0 .. m_(s-2), j_0 .. j_(p-s-1))][m_(s-1), c] t_(s-1)[(m_0 .. m_(s-3), j_0 .. j_(p-s-1), c), m_(s-2)]
// with t_0 = the input in reversed digit order and y = t_p in reversed digit order.  p = 2 is the order-2 product
// P L P R P with R = B_1, L = B_2; p = 3 the order-3 product of csrc/matmul3.hip.
// The permutations are LDS index maps; rows stay on chip between the factors.  fp32 arithmetic on tiles of rows in
// LDS, any b and p with b^p <= 4096 (the shape-generic kernels of the family: no matrix-core path of their own;
// p = 3 with blocks of 16 goes to the matrix-core kernels of csrc/matmul3.hip).
// Forward: in place.  A tile of 8 rows keeps ONE layout from load to store: digit position p - s of the index holds
// j_(p-s) until factor s replaces it by m_(s-1), so a block reads its b values at stride b^(p-s) and writes its b
// results to the same places, the load is a plain copy and only the store reverses the digits.
// Gradients: p + 1 buffers (t_0 .. t_(p-1) and the running gradient) in the layouts of the formula above.
#include "kernels.h"

namespace monarch {

namespace mmp {

constexpr int THREADS = 256;
constexpr int MAXP = 12;

struct Geo {
    int p, b, N;
    int lo[MAXP + 1];   // lo[s] = b^(p-s): the number of values of the unconsumed input digits in a block number of factor s
};

// the index with its p base-b digits reversed
__device__ __forceinline__ int reversed(int j, int b, int p)
{
    int r = 0;
    for (int a = 0; a < p; ++a) {
        r = r * b + j % b;
        j /= b;
    }
    return r;
}

// Where factor s reads the element that meets column 0 of block K (position in t_(s-1)), and the step to the next
// column: the block number (hi, mid, lo) = (m_0 .. m_(s-3), m_(s-2), j_0 .. j_(p-s-1)) reads (hi, lo, c, mid).
__device__ __forceinline__ int in_base(const Geo &g, int s, int K, int &step)
{
    if (s == 1) {
        step = 1;
        return K * g.b;
    }
    const int lo = g.lo[s], hi = K / (lo * g.b), rem = K - hi * lo * g.b, mid = rem / lo, l = rem - mid * lo;
    step = g.b;
    return (hi * lo + l) * g.b * g.b + mid;
}

// t_s = factor s of t_(s-1) on TV rows
template <typename T, int TV>
__device__ __forceinline__ void factor(const Geo &g, int s, const float *in, float *out, const T *__restrict__ W)
{
    const int N = g.N, b = g.b;
    for (int o = threadIdx.x; o < N; o += THREADS) {
        int step;
        const int base = in_base(g, s, o / b, step);
        float acc[TV];
#pragma unroll
        for (int v = 0; v < TV; ++v) acc[v] = 0.0f;
        const T *w = W + (size_t)o * b;
        for (int c = 0; c < b; ++c) {
            const float wv = to_f32(w[c]);
#pragma unroll
            for (int v = 0; v < TV; ++v) acc[v] = fmaf(wv, in[v * N + base + c * step], acc[v]);
        }
#pragma unroll
        for (int v = 0; v < TV; ++v) out[v * N + o] = acc[v];
    }
}

// Forward, in place, tiles of FT rows; BM = b rounded up to 2, 4, 8 or 16 (register arrays of a fixed size; the
// columns beyond b carry zero weights).
constexpr int FT = 8;

template <typename T, int BM>
__global__ __launch_bounds__(THREADS) void forward_kernel(const T *__restrict__ x, const T *__restrict__ B, T *__restrict__ y,
                                                          int64_t batch, Geo g)
{
    extern __shared__ float lds[];
    const int N = g.N, b = g.b, p = g.p, nblk = N / b;
    const int64_t ntiles = (batch + FT - 1) / FT;
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t v0 = tile * FT;
        for (int idx = threadIdx.x; idx < FT * N; idx += THREADS) lds[idx] = v0 + idx / N < batch ? to_f32(x[v0 * N + idx]) : 0.0f;
        __syncthreads();
        for (int s = 1; s <= p; ++s) {
            const int lo = g.lo[s];                                  // the stride of the digit this factor works on
            const T *Ws = B + (size_t)(s - 1) * N * b;
            for (int item = threadIdx.x; item < nblk; item += THREADS) {
                // item = (m_0 .. m_(s-2)) b^(p-s) + (j_(p-s-1) .. j_0); the block number has the j digits in reverse
                const int hi = item / lo, J = item - hi * lo;
                float *at = lds + hi * lo * b + J;
                const T *W = Ws + (size_t)(hi * lo + reversed(J, b, p - s)) * b * b;
                float in[BM][FT];
#pragma unroll
                for (int c = 0; c < BM; ++c)
#pragma unroll
                    for (int v = 0; v < FT; ++v) in[c][v] = c < b ? at[v * N + c * lo] : 0.0f;
                for (int r = 0; r < b; ++r) {
                    float acc[FT];
#pragma unroll
                    for (int v = 0; v < FT; ++v) acc[v] = 0.0f;
#pragma unroll
                    for (int c = 0; c < BM; ++c) {
                        const float w = c < b ? to_f32(W[r * b + c]) : 0.0f;
#pragma unroll
                        for (int v = 0; v < FT; ++v) acc[v] = fmaf(w, in[c][v], acc[v]);
                    }
#pragma unroll
                    for (int v = 0; v < FT; ++v) at[v * N + r * lo] = acc[v];
                }
            }
            __syncthreads();
        }
        // digit position p - 1 - a now holds m_a: y[m] sits at the reversed index
        for (int idx = threadIdx.x; idx < FT * N; idx += THREADS) {
            const int v = idx / N, m = idx - v * N;
            if (v0 + v < batch) y[v0 * N + idx] = from_f32<T>(lds[v * N + reversed(m, b, p)]);
        }
        __syncthreads();
    }
}

// Gradients on tiles of TV rows: p + 1 buffers of TV rows of N floats in LDS (t_0 .. t_(p-1) and the running
// gradient).  The adjoint of each factor, last factor first; the gradient with respect to t_(s-1) overwrites t_(s-1)
// once dB_s has been formed from it.  Every entry of dB is summed over the rows of a tile in a register and receives
// one atomic add per tile.
template <typename T, int TV>
__global__ __launch_bounds__(THREADS) void backward_kernel(const T *__restrict__ x, const T *__restrict__ B, const T *__restrict__ dy,
                                                           T *__restrict__ dx, float *__restrict__ dB, int64_t batch, Geo g)
{
    extern __shared__ float lds[];
    const int N = g.N, b = g.b, p = g.p;
    const int64_t ntiles = (batch + TV - 1) / TV;
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t v0 = tile * TV;
        float *grad = lds + (size_t)p * TV * N;          // buffer p: the gradient with respect to t_p
        for (int idx = threadIdx.x; idx < TV * N; idx += THREADS) {
            const int v = idx / N, j = idx - v * N;
            const bool live = v0 + v < batch;            // rows past the end are zero: they add nothing to the sums
            const int at = v * N + reversed(j, b, p);
            lds[at] = live ? to_f32(x[v0 * N + idx]) : 0.0f;
            grad[at] = live ? to_f32(dy[v0 * N + idx]) : 0.0f;
        }
        __syncthreads();
        for (int s = 1; s < p; ++s) {
            factor<T, TV>(g, s, lds + (size_t)(s - 1) * TV * N, lds + (size_t)s * TV * N, B + (size_t)(s - 1) * N * b);
            __syncthreads();
        }
        for (int s = p; s >= 1; --s) {
            float *prev = lds + (size_t)(s - 1) * TV * N;            // t_(s-1)
            const T *W = B + (size_t)(s - 1) * N * b;
            // dB_s[K][r, c] += grad[K, r] t_(s-1)[position of (K, c)]
            if (dB)
                for (int e = threadIdx.x; e < N * b; e += THREADS) {
                    const int o = e / b, c = e - o * b;
                    int step;
                    const int at = in_base(g, s, o / b, step) + c * step;
                    float acc = 0.0f;
#pragma unroll
                    for (int v = 0; v < TV; ++v) acc = fmaf(grad[v * N + o], prev[v * N + at], acc);
                    atomicAdd(dB + (size_t)(s - 1) * N * b + e, acc);
                }
            if (s == 1 && !dx) break;
            __syncthreads();
            // gradient with respect to t_(s-1): [position of (K, c)] = sum_r B_s[K][r, c] grad[K, r]
            for (int e = threadIdx.x; e < N; e += THREADS) {
                const int K = e / b, c = e - K * b;
                int step;
                const int at = in_base(g, s, K, step) + c * step;
                float acc[TV];
#pragma unroll
                for (int v = 0; v < TV; ++v) acc[v] = 0.0f;
                for (int r = 0; r < b; ++r) {
                    const float w = to_f32(W[((size_t)K * b + r) * b + c]);
#pragma unroll
                    for (int v = 0; v < TV; ++v) acc[v] = fmaf(w, grad[v * N + K * b + r], acc[v]);
                }
#pragma unroll
                for (int v = 0; v < TV; ++v) prev[v * N + at] = acc[v];
            }
            __syncthreads();
            grad = prev;
        }
        if (dx)
            for (int idx = threadIdx.x; idx < TV * N; idx += THREADS) {
                const int v = idx / N, j = idx - v * N;
                if (v0 + v < batch) dx[v0 * N + idx] = from_f32<T>(grad[v * N + reversed(j, b, p)]);
            }
        __syncthreads();
    }
}

__global__ void fill_kernel(float *a, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) a[i] = 0.0f;
}

static Geo geometry(int b, int p)
{
    Geo g = {};
    g.p = p;
    g.b = b;
    g.N = 1;
    for (int a = 0; a < p; ++a) g.N *= b;
    for (int s = 1; s <= p; ++s) {
        g.lo[s] = 1;
        for (int a = 0; a < p - s; ++a) g.lo[s] *= b;
    }
    return g;
}

constexpr size_t LDS_LIMIT = 144 * 1024;

// rows per tile: as many of 8, 4, 2, 1 as nbuf buffers of rows of N floats allow (more rows per tile: every weight
// read from L2 serves more rows)
static int rows_per_tile(int nbuf, int N)
{
    int tv = 8;
    while (tv > 1 && (size_t)nbuf * tv * N * sizeof(float) > 96 * 1024) tv >>= 1;
    return tv;
}

static int compute_units(int *ncu)
{
    int dev = 0;
    MONARCH_HIP_CHECK(hipGetDevice(&dev));
    MONARCH_HIP_CHECK(hipDeviceGetAttribute(ncu, hipDeviceAttributeMultiprocessorCount, dev));
    return MONARCH_OK;
}

static int64_t grid_for(int ncu, size_t lds, int64_t ntiles)
{
    const int64_t grid = (int64_t)ncu * (lds <= 36 * 1024 ? 4 : lds <= 76 * 1024 ? 2 : 1);
    return grid > ntiles ? ntiles : grid;
}

template <typename T, int BM>
static int launch_forward_bm(const void *x, const void *B, void *y, int64_t batch, const Geo &g, hipStream_t s)
{
    const size_t lds = (size_t)FT * g.N * sizeof(float);
    int ncu = 0;
    if (int rc = compute_units(&ncu)) return rc;
    auto kern = forward_kernel<T, BM>;
    if (lds > 64 * 1024)
        MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(kern, dim3((unsigned)grid_for(ncu, lds, (batch + FT - 1) / FT)), dim3(THREADS), lds, s, (const T *)x, (const T *)B,
                       (T *)y, batch, g);
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

template <typename T>
static int launch_forward(const void *x, const void *B, void *y, int64_t batch, const Geo &g, hipStream_t s)
{
    if (g.b <= 2) return launch_forward_bm<T, 2>(x, B, y, batch, g, s);
    if (g.b <= 4) return launch_forward_bm<T, 4>(x, B, y, batch, g, s);
    if (g.b <= 8) return launch_forward_bm<T, 8>(x, B, y, batch, g, s);
    return launch_forward_bm<T, 16>(x, B, y, batch, g, s);
}

template <typename T>
static int launch_backward(const void *x, const void *B, const void *dy, void *dx, float *dB, int64_t batch, const Geo &g, hipStream_t s)
{
    const int nbuf = g.p + 1;
    const int tv = rows_per_tile(nbuf, g.N);
    const size_t lds = (size_t)nbuf * tv * g.N * sizeof(float);
    int ncu = 0;
    if (int rc = compute_units(&ncu)) return rc;
    const int64_t grid = grid_for(ncu, lds, (batch + tv - 1) / tv);
#define MONARCH_LAUNCH_MMP(TVV)                                                                                              \
    do {                                                                                                                     \
        auto kern = backward_kernel<T, TVV>;                                                                                 \
        if (lds > 64 * 1024)                                                                                                 \
            MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)); \
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(THREADS), lds, s, (const T *)x, (const T *)B, (const T *)dy,     \
                           (T *)dx, dB, batch, g);                                                                           \
    } while (0)
    switch (tv) {
    case 8: MONARCH_LAUNCH_MMP(8); break;
    case 4: MONARCH_LAUNCH_MMP(4); break;
    case 2: MONARCH_LAUNCH_MMP(2); break;
    default: MONARCH_LAUNCH_MMP(1); break;
    }
#undef MONARCH_LAUNCH_MMP
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

}  // namespace mmp

// b^p if the shape is one the kernels take (2 <= p <= 12, 2 <= b <= 16, b^p <= 4096, and for the gradients p + 1
// rows of b^p floats within the LDS of a compute unit), else 0
int matmulp_length(int b, int p, bool backward)
{
    if (p < 2 || p > mmp::MAXP || b < 2 || b > 16) return 0;
    int64_t N = 1;
    for (int a = 0; a < p; ++a) {
        N *= b;
        if (N > 4096) return 0;
    }
    if (backward && (size_t)(p + 1) * N * sizeof(float) > mmp::LDS_LIMIT) return 0;
    return (int)N;
}

int launch_matmulp(const void *x, const void *B, void *y, int64_t batch, int b, int p, monarch_dtype dt, hipStream_t s)
{
    const mmp::Geo g = mmp::geometry(b, p);
    const size_t fs = (size_t)g.N * b * dtype_size(dt);           // one factor
    if (p == 3 && b == 16)
        return launch_matmul3(x, B, (const char *)B + fs, (const char *)B + 2 * fs, y, batch, b, dt, s);
    if (dt == MONARCH_F32) return mmp::launch_forward<float>(x, B, y, batch, g, s);
    return mmp::launch_forward<bf16_t>(x, B, y, batch, g, s);
}

int launch_matmulp_backward(const void *x, const void *B, const void *dy, void *dx, float *dB, int64_t batch, int b, int p,
                            monarch_dtype dt, hipStream_t s)
{
    const mmp::Geo g = mmp::geometry(b, p);
    if (p == 3 && b == 16) {
        const size_t fs = (size_t)g.N * b * dtype_size(dt), gs = (size_t)g.N * b;
        return launch_matmul3_backward(x, B, (const char *)B + fs, (const char *)B + 2 * fs, dy, dx, dB, dB ? dB + gs : nullptr,
                                       dB ? dB + 2 * gs : nullptr, batch, b, dt, s);
    }
    if (dB) {
        hipLaunchKernelGGL(mmp::fill_kernel, dim3(64), dim3(256), 0, s, dB, (size_t)p * g.N * b);
        MONARCH_HIP_CHECK(hipGetLastError());
    }
    if (batch == 0) return MONARCH_OK;
    if (dt == MONARCH_F32) return mmp::launch_backward<float>(x, B, dy, dx, dB, batch, g, s);
    return mmp::launch_backward<bf16_t>(x, B, dy, dx, dB, batch, g, s);
}

}  // namespace monarch
