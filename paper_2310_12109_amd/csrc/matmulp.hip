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
// In place: a tile of rows keeps ONE layout from load to store: digit position p - s of the index holds j_(p-s)
// until factor s replaces it by m_(s-1), so a block reads its b values at stride b^(p-s) and writes its b results to
// the same places, the load is a plain copy and only the store reverses the digits.  The gradients keep a second tile
// for the running gradient in the same layout and recompute the forward values each factor needs.
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

// In-place layout of a tile of rows: digit position p - s of the LDS index holds j_(p-s) until factor s replaces it by
// m_(s-1).  Block item = (m_0 .. m_(s-2)) b^(p-s) + (j_(p-s-1) .. j_0) of factor s: its b values sit at `at + c lo`,
// lo = b^(p-s), and its block number has the j digits in reverse.
// Position i of a row sits at LDS word i + i / 32 (row pitch N + N / 32): the digit-reversed gather of the store and
// the unit-stride factors, whose lanes are a power of b apart, would otherwise meet in one bank.
__device__ __forceinline__ int pad(int i) { return i + (i >> 5); }
__host__ __device__ __forceinline__ int pitch(int N) { return N + (N >> 5); }

// four consecutive weights (16- or 8-byte aligned: b a multiple of 4)
__device__ __forceinline__ void load_w4(const float *p, float (&w)[4])
{
    const float4 v = *reinterpret_cast<const float4 *>(p);
    w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
}
__device__ __forceinline__ void load_w4(const bf16_t *p, float (&w)[4])
{
    const uint2 v = *reinterpret_cast<const uint2 *>(p);
    w[0] = __uint_as_float(v.x << 16); w[1] = __uint_as_float(v.x & 0xffff0000u);
    w[2] = __uint_as_float(v.y << 16); w[3] = __uint_as_float(v.y & 0xffff0000u);
}

struct Item {
    int at, K;
};
__device__ __forceinline__ Item block_item(const Geo &g, int s, int item)
{
    const int lo = g.lo[s], hi = item / lo, J = item - hi * lo;
    return {hi * lo * g.b + J, hi * lo + reversed(J, g.b, g.p - s)};
}

// Factor s on a tile of ROWS rows, in place; a work item is a block and NV of the rows.  BM = b rounded up to 2, 4, 8 or
// 16 (register arrays of a fixed size; the columns beyond b carry zero weights).
template <typename T, int BM, int NV, int ROWS = NV>
__device__ __forceinline__ void stage_inplace(const Geo &g, int s, float *buf, const T *__restrict__ B)
{
    const int N = g.N, NP = pitch(N), b = g.b, lo = g.lo[s], nblk = N / b;
    const T *Ws = B + (size_t)(s - 1) * N * b;
    for (int work = threadIdx.x; work < nblk * (ROWS / NV); work += blockDim.x) {
        const int item = work % nblk, chunk = work / nblk;
        const Item it = block_item(g, s, item);
        float *at = buf + chunk * NV * NP;
        const T *W = Ws + (size_t)it.K * b * b;
        float in[BM][NV];
#pragma unroll
        for (int c = 0; c < BM; ++c)
#pragma unroll
            for (int v = 0; v < NV; ++v) in[c][v] = c < b ? at[v * NP + pad(it.at + c * lo)] : 0.0f;
        for (int r = 0; r < b; ++r) {
            float acc[NV];
#pragma unroll
            for (int v = 0; v < NV; ++v) acc[v] = 0.0f;
            // a lane reads its own block (its own cache line per load instruction): four weights per load where b allows
            if (BM >= 4 && (b & 3) == 0) {
#pragma unroll
                for (int c4 = 0; c4 < BM / 4; ++c4) {
                    float w[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                    if (4 * c4 < b) load_w4(W + r * b + 4 * c4, w);
#pragma unroll
                    for (int e = 0; e < 4; ++e)
#pragma unroll
                        for (int v = 0; v < NV; ++v) acc[v] = fmaf(w[e], in[4 * c4 + e][v], acc[v]);
                }
            } else {
#pragma unroll
                for (int c = 0; c < BM; ++c) {
                    const float w = c < b ? to_f32(W[r * b + c]) : 0.0f;
#pragma unroll
                    for (int v = 0; v < NV; ++v) acc[v] = fmaf(w, in[c][v], acc[v]);
                }
            }
#pragma unroll
            for (int v = 0; v < NV; ++v) at[v * NP + pad(it.at + r * lo)] = acc[v];
        }
    }
}

// Forward: tiles of FT rows, one buffer.
constexpr int FT = 8;

template <typename T, int BM>
__global__ __launch_bounds__(1024) void forward_kernel(const T *__restrict__ x, const T *__restrict__ B, T *__restrict__ y,
                                                          int64_t batch, Geo g)
{
    extern __shared__ float lds[];
    const int N = g.N, NP = pitch(N), b = g.b, p = g.p;
    const int64_t ntiles = (batch + FT - 1) / FT;
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t v0 = tile * FT;
        for (int idx = threadIdx.x; idx < FT * N; idx += blockDim.x) {
            const int v = idx / N, j = idx - v * N;
            lds[v * NP + pad(j)] = v0 + v < batch ? to_f32(x[v0 * N + idx]) : 0.0f;
        }
        __syncthreads();
        for (int s = 1; s <= p; ++s) {
            stage_inplace<T, BM, FT / 2, FT>(g, s, lds, B);
            __syncthreads();
        }
        // digit position p - 1 - a now holds m_a: y[m] sits at the reversed index
        for (int idx = threadIdx.x; idx < FT * N; idx += blockDim.x) {
            const int v = idx / N, m = idx - v * N;
            if (v0 + v < batch) y[v0 * N + idx] = from_f32<T>(lds[v * NP + pad(reversed(m, b, p))]);
        }
        __syncthreads();
    }
}

// Gradients: tiles of BT rows in two buffers of the in-place layout, S (forward values) and G (the running gradient).
// G starts as dy in the layout the forward leaves y in (digits reversed).  For s = p .. 1: S <- x and factors 1 .. s - 1
// in place (t_(s-1): recomputed, p (p - 1) / 2 factor applications per tile instead of p + 1 buffers, so four rows
// fit at N = 4096 instead of one); a block's b forward values and its b gradients then sit at the same places of
// S and G: dB_s[K][r, c] += sum over the rows of G[r] S[c] (one atomic add per entry and tile), and the gradient with
// respect to t_(s-1) replaces G in place, G[c] <- sum_r B_s[K][r, c] G[r].  After s = 1 G is dx in natural order.
constexpr int BT = 4;

template <typename T, int BM>
__global__ __launch_bounds__(THREADS) void backward_kernel(const T *__restrict__ x, const T *__restrict__ B, const T *__restrict__ dy,
                                                           T *__restrict__ dx, float *__restrict__ dB, int64_t batch, Geo g)
{
    extern __shared__ float lds[];
    const int N = g.N, NP = pitch(N), b = g.b, p = g.p, nblk = N / b;
    float *S = lds, *G = lds + BT * NP;
    const int64_t ntiles = (batch + BT - 1) / BT;
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t v0 = tile * BT;
        for (int idx = threadIdx.x; idx < BT * N; idx += THREADS) {
            const int v = idx / N, m = idx - v * N;   // rows past the end are zero: they add nothing to the sums
            G[v * NP + pad(reversed(m, b, p))] = v0 + v < batch ? to_f32(dy[v0 * N + idx]) : 0.0f;
        }
        for (int s = p; s >= 1; --s) {
            if (dB) {
                for (int idx = threadIdx.x; idx < BT * N; idx += THREADS) {
                    const int v = idx / N, j = idx - v * N;
                    S[v * NP + pad(j)] = v0 + v < batch ? to_f32(x[v0 * N + idx]) : 0.0f;
                }
                __syncthreads();
                for (int q = 1; q < s; ++q) {
                    stage_inplace<T, BM, BT>(g, q, S, B);
                    __syncthreads();
                }
            } else {
                __syncthreads();
            }
            const bool back = s > 1 || dx != nullptr;   // the gradient with respect to t_(s-1) is needed
            const int lo = g.lo[s];
            const T *Ws = B + (size_t)(s - 1) * N * b;
            float *dBs = dB ? dB + (size_t)(s - 1) * N * b : nullptr;
            // dB_s[K][r, c]: one thread per entry, neighbouring lanes neighbouring entries (the atomic adds of a wave
            // instruction fall into two cache lines; with one thread per block they fell into 64 and the kernel was slower
            // than with one row per tile)
            if (dB) {
                for (int e = threadIdx.x; e < N * b; e += THREADS) {
                    const int c = e % b, o = e / b, r = o % b, K = o / b;
                    const int hi = K / lo, at = hi * lo * b + reversed(K - hi * lo, b, p - s);
                    float acc = 0.0f;
#pragma unroll
                    for (int v = 0; v < BT; ++v) acc = fmaf(G[v * NP + pad(at + r * lo)], S[v * NP + pad(at + c * lo)], acc);
                    atomicAdd(dBs + e, acc);
                }
                if (back) __syncthreads();   // every gradient read before the blocks overwrite G
            }
            if (back)
                for (int item = threadIdx.x; item < nblk; item += THREADS) {
                    const Item it = block_item(g, s, item);
                    float *gat = G;
                    const T *W = Ws + (size_t)it.K * b * b;
                    float out[BM][BT];
#pragma unroll
                    for (int c = 0; c < BM; ++c)
#pragma unroll
                        for (int v = 0; v < BT; ++v) out[c][v] = 0.0f;
                    for (int r = 0; r < b; ++r) {
                        float gr[BT];
#pragma unroll
                        for (int v = 0; v < BT; ++v) gr[v] = gat[v * NP + pad(it.at + r * lo)];
                        if (BM >= 4 && (b & 3) == 0) {
#pragma unroll
                            for (int c4 = 0; c4 < BM / 4; ++c4) {
                                float w[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                                if (4 * c4 < b) load_w4(W + r * b + 4 * c4, w);
#pragma unroll
                                for (int e = 0; e < 4; ++e)
#pragma unroll
                                    for (int v = 0; v < BT; ++v) out[4 * c4 + e][v] = fmaf(w[e], gr[v], out[4 * c4 + e][v]);
                            }
                        } else {
#pragma unroll
                            for (int c = 0; c < BM; ++c) {
                                const float w = c < b ? to_f32(W[r * b + c]) : 0.0f;
#pragma unroll
                                for (int v = 0; v < BT; ++v) out[c][v] = fmaf(w, gr[v], out[c][v]);
                            }
                        }
                    }
#pragma unroll
                    for (int c = 0; c < BM; ++c)
                        if (c < b) {
#pragma unroll
                            for (int v = 0; v < BT; ++v) gat[v * NP + pad(it.at + c * lo)] = out[c][v];
                        }
                }
            __syncthreads();
        }
        if (dx)
            for (int idx = threadIdx.x; idx < BT * N; idx += THREADS)
                if (v0 + idx / N < batch) dx[v0 * N + idx] = from_f32<T>(G[(idx / N) * NP + pad(idx % N)]);
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
    const size_t lds = (size_t)FT * pitch(g.N) * sizeof(float);
    int ncu = 0;
    if (int rc = compute_units(&ncu)) return rc;
    auto kern = forward_kernel<T, BM>;
    if (lds > 64 * 1024)
        MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    // one thread per (block, half of the rows) of a factor, 256 to 1024 of them
    int threads = (2 * (g.N / g.b) + 255) / 256 * 256;
    threads = threads > 1024 ? 1024 : threads;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid_for(ncu, lds, (batch + FT - 1) / FT)), dim3(threads), lds, s, (const T *)x, (const T *)B,
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

template <typename T, int BM>
static int launch_backward_bm(const void *x, const void *B, const void *dy, void *dx, float *dB, int64_t batch, const Geo &g, hipStream_t s)
{
    const size_t lds = (size_t)2 * BT * pitch(g.N) * sizeof(float);
    int ncu = 0;
    if (int rc = compute_units(&ncu)) return rc;
    auto kern = backward_kernel<T, BM>;
    if (lds > 64 * 1024)
        MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(kern, dim3((unsigned)grid_for(ncu, lds, (batch + BT - 1) / BT)), dim3(THREADS), lds, s, (const T *)x, (const T *)B,
                       (const T *)dy, (T *)dx, dB, batch, g);
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

template <typename T>
static int launch_backward(const void *x, const void *B, const void *dy, void *dx, float *dB, int64_t batch, const Geo &g, hipStream_t s)
{
    if (g.b <= 2) return launch_backward_bm<T, 2>(x, B, dy, dx, dB, batch, g, s);
    if (g.b <= 4) return launch_backward_bm<T, 4>(x, B, dy, dx, dB, batch, g, s);
    if (g.b <= 8) return launch_backward_bm<T, 8>(x, B, dy, dx, dB, batch, g, s);
    return launch_backward_bm<T, 16>(x, B, dy, dx, dB, batch, g, s);
}

}  // namespace mmp

// b^p if the shape is one the kernels take (2 <= p <= 12, 2 <= b <= 16, b^p <= 4096), else 0
int matmulp_length(int b, int p, bool backward)
{
    if (p < 2 || p > mmp::MAXP || b < 2 || b > 16) return 0;
    int64_t N = 1;
    for (int a = 0; a < p; ++a) {
        N *= b;
        if (N > 4096) return 0;
    }
    (void)backward;   // forward (8 rows in one buffer) and gradients (4 rows in two) need the same 128 KB at most
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
