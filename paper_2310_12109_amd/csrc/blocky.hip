// Polynomial-parameterised ("blocky") Monarch matrices and the convolution built on them (appendix: the blocky
// Monarch algorithm, the masking lemma, the blocky Monarch convolution and its causality theorem).
//
// Parameters: coefficient matrices Lt, Rt (N x b, real, b = sqrt(N)).  They stand for complex block-diagonal
// factors
//   R_{j1}[i0, j0] = sum_{a<b} Rt[j1 b + a, j0] w_b^(i0 a),      L_{i0}[i1, j1] = sum_{a<N} Lt[a, j1] w_N^((i1 b + i0) a)
// (w_m = exp(+2 pi i / m)), M = P L P R P, and the convolution is  f = M^-1 ( (M k) o (M u) )  with
// M^-1 = P R^-1 P L^-1 P (blockwise inverses).  With the masks of the lemma applied to the coefficients the map
// u -> f[0:n] is causal for n <= b floor(b/2).
//
// Two phases.  prepare (once per parameter update, O(N^1.5 .. N^2.5) work, float64 arithmetic): the factors, their
// blockwise inverses and the kernel in the transform domain, written as complex float32 into a state buffer of the
// caller.  conv (per batch): rows stay on chip from load to store, gates fused, complex float32 arithmetic.
#include "kernels.h"
#include "lds_dma.h"

namespace monarch {

namespace blocky {

struct cdouble {
    double re, im;
};
__device__ __forceinline__ cdouble cmul(cdouble a, cdouble b) { return {a.re * b.re - a.im * b.im, a.re * b.im + a.im * b.re}; }
__device__ __forceinline__ cdouble csub(cdouble a, cdouble b) { return {a.re - b.re, a.im - b.im}; }
__device__ __forceinline__ cdouble cinv(cdouble a)
{
    const double d = a.re * a.re + a.im * a.im;   // 0 for a singular block: the inverse is then not finite
    return {a.re / d, -a.im / d};
}

// layout of the state buffer (byte offsets, each part 256-byte aligned)
struct Layout {
    size_t tw, R1, L1, R2, L2, Kf, Kq, total;
};
__host__ __device__ inline size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }
__host__ __device__ inline Layout layout(int H, int bs)
{
    const size_t N = (size_t)bs * bs, f = up256(N * bs * sizeof(float2));
    Layout l;
    l.tw = 0;
    l.R1 = up256(N * sizeof(cdouble));
    l.L1 = l.R1 + f;
    l.R2 = l.L1 + f;
    l.L2 = l.R2 + f;
    l.Kf = l.L2 + f;
    l.Kq = l.Kf + up256((size_t)H * N * sizeof(float2));
    // bs = 16 only: a second copy of Kf in the order in which the matrix-core kernel's lanes read it
    l.total = l.Kq + (bs == 16 ? up256((size_t)((H + 3) / 4) * 4 * N * sizeof(float2)) : 0);
    return l;
}

// w_N^e for e in [0, N), float64
__global__ void twiddle_kernel(cdouble *tw, int N)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e < N) {
        double s, c;
        sincospi(2.0 * (double)e / (double)N, &s, &c);
        tw[e] = {c, s};
    }
}

// masked coefficient reads (masking lemma); `a` is the degree, the second index the column
__device__ __forceinline__ double coeff_L(const float *Lt, int bs, int a, int j1, bool mask)
{
    if (mask && (a >= bs || a < j1)) return 0.0;
    return (double)Lt[(size_t)a * bs + j1];
}
__device__ __forceinline__ double coeff_R(const float *Rt, int bs, int j1, int a, int j0, bool mask)
{
    if (mask && (a < j0 || (a >= bs / 2 && j0 < bs / 2))) return 0.0;
    return (double)Rt[((size_t)j1 * bs + a) * bs + j0];
}

// One workgroup per block: blocks [0, bs) are those of R, [bs, 2 bs) those of L.  The block is evaluated in
// float64 into LDS, written out as complex float32, inverted in place (Gauss-Jordan, partial pivoting) and the
// inverse written into the factor of M^-1 that it is: R^-1 -> L2, L^-1 -> R2.
__global__ __launch_bounds__(256) void factor_kernel(const float *__restrict__ Lt, const float *__restrict__ Rt,
                                                     const cdouble *__restrict__ tw, float2 *__restrict__ R1,
                                                     float2 *__restrict__ L1, float2 *__restrict__ R2,
                                                     float2 *__restrict__ L2, int bs, int mask)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char raw[];
    cdouble *A = reinterpret_cast<cdouble *>(raw);                      // [bs][bs]
    int *swapped = reinterpret_cast<int *>(raw + (size_t)bs * bs * sizeof(cdouble));   // [bs] + 1
    const int N = bs * bs, tid = threadIdx.x;
    const bool is_L = blockIdx.x >= (unsigned)bs;
    const int blk = is_L ? blockIdx.x - bs : blockIdx.x;
    const int terms = is_L ? (mask ? bs : N) : bs;
    for (int e = tid; e < N; e += blockDim.x) {
        const int row = e / bs, col = e - row * bs;
        cdouble acc = {0.0, 0.0};
        // R: block j1 = blk, row i0, column j0: point w_b^i0 = w_N^(i0 b).  L: block i0 = blk, row i1, column j1:
        // point w_N^(i1 b + i0)
        const int point = is_L ? row * bs + blk : row * bs;
        int ex = 0;   // (point * a) mod N
        for (int a = 0; a < terms; ++a) {
            const double c = is_L ? coeff_L(Lt, bs, a, col, mask) : coeff_R(Rt, bs, blk, a, col, mask);
            const cdouble w = tw[ex];
            acc.re += c * w.re;
            acc.im += c * w.im;
            ex += point;
            if (ex >= N) ex -= N;
        }
        A[e] = acc;
        (is_L ? L1 : R1)[(size_t)blk * N + e] = make_float2((float)acc.re, (float)acc.im);
    }
    __syncthreads();
    for (int p = 0; p < bs; ++p) {
        if (tid == 0) {
            int best = p;
            double bm = A[p * bs + p].re * A[p * bs + p].re + A[p * bs + p].im * A[p * bs + p].im;
            for (int r = p + 1; r < bs; ++r) {
                const cdouble v = A[r * bs + p];
                const double m = v.re * v.re + v.im * v.im;
                if (m > bm) { bm = m; best = r; }
            }
            swapped[p] = best;
        }
        __syncthreads();
        const int piv = swapped[p];
        if (piv != p)
            for (int c = tid; c < bs; c += blockDim.x) {
                const cdouble t = A[p * bs + c];
                A[p * bs + c] = A[piv * bs + c];
                A[piv * bs + c] = t;
            }
        __syncthreads();
        const cdouble pinv = cinv(A[p * bs + p]);
        __syncthreads();
        for (int c = tid; c < bs; c += blockDim.x) A[p * bs + c] = c == p ? pinv : cmul(A[p * bs + c], pinv);
        __syncthreads();
        // eliminate column p from every other row; thread e owns entry (row, col), column p is handled last
        for (int e = tid; e < N; e += blockDim.x) {
            const int row = e / bs, col = e - row * bs;
            if (row == p || col == p) continue;
            A[e] = csub(A[e], cmul(A[row * bs + p], A[p * bs + col]));
        }
        __syncthreads();
        for (int row = tid; row < bs; row += blockDim.x)
            if (row != p) {
                const cdouble f = A[row * bs + p];
                const cdouble r = cmul(f, A[p * bs + p]);
                A[row * bs + p] = {-r.re, -r.im};
            }
        __syncthreads();
    }
    // undo the row exchanges: they are column exchanges of the inverse, in reverse order
    for (int p = bs - 1; p >= 0; --p) {
        const int piv = swapped[p];
        if (piv != p)
            for (int r = tid; r < bs; r += blockDim.x) {
                const cdouble t = A[r * bs + p];
                A[r * bs + p] = A[r * bs + piv];
                A[r * bs + piv] = t;
            }
        __syncthreads();
    }
    for (int e = tid; e < N; e += blockDim.x)
        (is_L ? R2 : L2)[(size_t)blk * N + e] = make_float2((float)A[e].re, (float)A[e].im);
}

constexpr int THREADS = 256;

// One complex block-diagonal factor W [bs][bs][bs] on TV rows held in LDS: block k reads in[v][k ks_in + c cs_in],
// c < cmax, and writes out[v][r bs + k] for the rows r < rmax.  REAL_IN: the input has no imaginary part.
template <int TV, bool REAL_IN>
__device__ __forceinline__ void cfactor(const float2 *in, float2 *out, int N, int bs, const float2 *__restrict__ W,
                                        int cs_in, int ks_in, int cmax, int rmax)
{
    for (int o = threadIdx.x; o < N; o += THREADS) {   // o = k bs + r
        const int k = o / bs, r = o - k * bs;
        if (r >= rmax) continue;
        float2 acc[TV];
#pragma unroll
        for (int v = 0; v < TV; ++v) acc[v] = make_float2(0.0f, 0.0f);
        const float2 *w = W + (size_t)o * bs;
        for (int c = 0; c < cmax; ++c) {
            const float2 wv = w[c];
#pragma unroll
            for (int v = 0; v < TV; ++v) {
                const float2 x = in[v * N + k * ks_in + c * cs_in];
                acc[v].x = fmaf(wv.x, x.x, acc[v].x);
                acc[v].y = fmaf(wv.y, x.x, acc[v].y);
                if (!REAL_IN) {
                    acc[v].x = fmaf(-wv.y, x.y, acc[v].x);
                    acc[v].y = fmaf(wv.x, x.y, acc[v].y);
                }
            }
        }
#pragma unroll
        for (int v = 0; v < TV; ++v) out[v * N + r * bs + k] = acc[v];
    }
}

// Kf[h, :] = M (k[h, :], 0): one workgroup per channel
__global__ __launch_bounds__(THREADS) void kf_kernel(const float *__restrict__ k, const float2 *__restrict__ R1,
                                                     const float2 *__restrict__ L1, float2 *__restrict__ Kf,
                                                     float4 *__restrict__ Kq, int klen, int bs)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char raw[];
    const int N = bs * bs, h = blockIdx.x;
    float2 *a = reinterpret_cast<float2 *>(raw), *t = a + N;
    for (int j = threadIdx.x; j < N; j += THREADS) a[j] = make_float2(j < klen ? k[(size_t)h * klen + j] : 0.0f, 0.0f);
    __syncthreads();
    cfactor<1, true>(a, t, N, bs, R1, bs, 1, (klen + bs - 1) / bs, bs);
    __syncthreads();
    cfactor<1, false>(t, a, N, bs, L1, 1, bs, bs, bs);
    __syncthreads();
    for (int j = threadIdx.x; j < N; j += THREADS) Kf[(size_t)h * N + j] = a[j];
    // bs = 16: the same values as pairs of complex numbers, in the order of blocky16::conv_b16_kernel's loads:
    // piece ((w 4 + kg) 8 + 2 r + half) of channel h holds elements 16 (4 kg + r) + 4 w + 2 half and the next one;
    // four consecutive channels are interleaved piece by piece, so that four neighbouring lanes read 64 bytes
    if (Kq)
        for (int idx = threadIdx.x; idx < N / 2; idx += THREADS) {
            const int p = idx & 7, kg = (idx >> 3) & 3, w = idx >> 5;
            const int j = 16 * (4 * kg + (p >> 1)) + 4 * w + 2 * (p & 1);
            Kq[((size_t)(h >> 2) * (N / 2) + idx) * 4 + (h & 3)] = make_float4(a[j].x, a[j].y, a[j + 1].x, a[j + 1].y);
        }
}

// y[row, 0:n] = g_out o Re( M2 ( Kf[h] o ( M1 (g_in o u, 0) ) ) )[0:n], row = b H + h
template <typename T, int TV>
__global__ __launch_bounds__(THREADS) void conv_kernel(const T *__restrict__ u, const T *__restrict__ g_in,
                                                       const T *__restrict__ g_out, const float2 *__restrict__ R1,
                                                       const float2 *__restrict__ L1, const float2 *__restrict__ R2,
                                                       const float2 *__restrict__ L2, const float2 *__restrict__ Kf,
                                                       T *__restrict__ y, int64_t rows, int H, int n, int bs)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char raw[];
    const int N = bs * bs;
    float2 *a = reinterpret_cast<float2 *>(raw), *t = a + (size_t)TV * N;
    const int live = (n + bs - 1) / bs;   // leading indices c (of the input) and k (of the output) that matter
    const int64_t ntiles = (rows + TV - 1) / TV;
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t r0 = tile * TV;
        for (int idx = threadIdx.x; idx < TV * N; idx += THREADS) {
            const int v = idx / N, j = idx - v * N;
            float x = 0.0f;
            if (r0 + v < rows && j < n) {
                x = to_f32(u[(r0 + v) * n + j]);
                if (g_in) x *= to_f32(g_in[(r0 + v) * n + j]);
            }
            a[idx] = make_float2(x, 0.0f);
        }
        __syncthreads();
        cfactor<TV, true>(a, t, N, bs, R1, bs, 1, live, bs);
        __syncthreads();
        cfactor<TV, false>(t, a, N, bs, L1, 1, bs, bs, bs);
        __syncthreads();
        for (int idx = threadIdx.x; idx < TV * N; idx += THREADS) {
            const int v = idx / N, j = idx - v * N;
            int64_t r = r0 + v;
            if (r >= rows) r = rows - 1;
            const float2 kf = Kf[(r % H) * (int64_t)N + j], x = a[idx];
            a[idx] = make_float2(x.x * kf.x - x.y * kf.y, x.x * kf.y + x.y * kf.x);
        }
        __syncthreads();
        cfactor<TV, false>(a, t, N, bs, R2, bs, 1, bs, bs);
        __syncthreads();
        cfactor<TV, false>(t, a, N, bs, L2, 1, bs, bs, live);
        __syncthreads();
        for (int idx = threadIdx.x; idx < TV * N; idx += THREADS) {
            const int v = idx / N, j = idx - v * N;
            if (r0 + v < rows && j < n) {
                float o = a[idx].x;
                if (g_out) o *= to_f32(g_out[(r0 + v) * n + j]);
                y[(r0 + v) * n + j] = from_f32<T>(o);
            }
        }
        __syncthreads();
    }
}

template <typename T>
static int launch_conv_typed(const void *u, const void *g_in, const void *g_out, const unsigned char *state, void *y,
                             int64_t rows, int H, int n, int bs, hipStream_t s)
{
    const int N = bs * bs;
    const Layout l = layout(H, bs);
    int tv = 8;
    while (tv > 1 && (size_t)2 * tv * N * sizeof(float2) > 64 * 1024) tv >>= 1;
    const size_t lds = (size_t)2 * tv * N * sizeof(float2);
    int dev = 0, ncu = 0;
    MONARCH_HIP_CHECK(hipGetDevice(&dev));
    MONARCH_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
    const int64_t ntiles = (rows + tv - 1) / tv;
    int64_t grid = (int64_t)ncu * (lds <= 32 * 1024 ? 4 : 2);
    if (grid > ntiles) grid = ntiles;
#define MONARCH_LAUNCH_BLOCKY(TVV)                                                                                \
    hipLaunchKernelGGL((conv_kernel<T, TVV>), dim3((unsigned)grid), dim3(THREADS), lds, s, (const T *)u,          \
                       (const T *)g_in, (const T *)g_out, (const float2 *)(state + l.R1),                         \
                       (const float2 *)(state + l.L1), (const float2 *)(state + l.R2),                            \
                       (const float2 *)(state + l.L2), (const float2 *)(state + l.Kf), (T *)y, rows, H, n, bs)
    switch (tv) {
    case 8: MONARCH_LAUNCH_BLOCKY(8); break;
    case 4: MONARCH_LAUNCH_BLOCKY(4); break;
    case 2: MONARCH_LAUNCH_BLOCKY(2); break;
    default: MONARCH_LAUNCH_BLOCKY(1); break;
    }
#undef MONARCH_LAUNCH_BLOCKY
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

}  // namespace blocky


// ---- bs = 16 (N = 256), float32 rows, on the matrix cores ---------------------------------------------
// The four complex block-diagonal products as 16x16x4 float32 MFMAs on real and imaginary parts, rows on the MFMA
// column index.  A workgroup of 4 waves takes a tile of 16 rows; wave w owns blocks 4 w .. 4 w + 3 of every factor
// (real and imaginary A operands: 128 registers for the kernel's lifetime).  The 16 rows of a tile are one
// contiguous piece of memory and arrive by direct-to-LDS loads in chunks of 1 KB (LDS pitch 260 floats per chunk).
//   S1  T_a[i, v]  = sum_c R1_a[i, c] (g_in u)[v][16 c + a]      real input; only the K steps with 16 c < n
//   S2  z[v][16 k + i] = Kf[h_v][16 k + i] sum_a L1_i[k, a] T_a[i, v]
//   S3, S4 the same with R2, L2; of S4 only the real part, of its rows only those with 16 k < n are stored
// Inside a matrix the rows cross between the waves through two LDS tiles (real, imaginary) whose index map is the
// middle permutation; between the matrices z sits as plain rows where u and g_in were.
namespace blocky16 {

typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int B = 16, TV = 16;
constexpr int CH = 260;                    // LDS pitch of a 1 KB chunk (256 floats) of a tile, and of a row of z
constexpr int RS = 18, LD = B * RS + 3;    // tiles between the factors: element (v, p, q) at v LD + p RS + q
constexpr int ROWBUF = 16 * CH;            // 16 chunks, or 16 rows of z
constexpr size_t LDS_BYTES = sizeof(float) * (2 * ROWBUF + 2 * TV * LD);

__device__ __forceinline__ f32x4 mfma(float a, float b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ int chunked(int flat) { return (flat >> 8) * CH + (flat & 255); }

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    const bf16_t a = from_f32<bf16_t>(lo), b = from_f32<bf16_t>(hi);
    return (uint32_t) * reinterpret_cast<const uint16_t *>(&a) | ((uint32_t) * reinterpret_cast<const uint16_t *>(&b) << 16);
}

// KS1: K steps of S1 that can hold live input (2 for n <= 128, else 4); n is a multiple of 16.
// T: type of u, the gates and y in memory.  float tiles arrive by direct-to-LDS loads; bf16 tiles pass through
// registers (8 elements per lane and instruction) and are widened on the way into LDS: everything on chip is float.
template <typename T, int KS1>
__global__ __launch_bounds__(256, 2) void conv_b16_kernel(const T *__restrict__ u, const T *__restrict__ g_in,
                                                          const T *__restrict__ g_out, const float2 *__restrict__ R1,
                                                          const float2 *__restrict__ L1, const float2 *__restrict__ R2,
                                                          const float2 *__restrict__ L2, const f32x4 *__restrict__ Kq,
                                                          T *__restrict__ y, int64_t rows, int H, int n)
{
    constexpr bool F32 = sizeof(T) == 4;
    extern __shared__ __attribute__((aligned(16))) float smem[];
    float *xa = smem;              // u; then Re z; then g_out
    float *xb = xa + ROWBUF;       // g_in; then Im z; then the rows of y
    float *tr = xb + ROWBUF;       // Re, Im of the tile between the two factors of a matrix: (v, i, a)
    float *ti = tr + TV * LD;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63, l16 = lane & 15, kg = lane >> 4;
    const int b0 = 4 * wave;

    // A operands.  S1: K step s, lane group kg holds column c = 4 s + kg (so that whole K steps are dead when n is
    // short); the other three factors: column 4 kg + s.
    float R1r[4][KS1], R1i[4][KS1], L1r[4][4], L1i[4][4], R2r[4][4], R2i[4][4], L2r[4][4], L2i[4][4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int row = ((b0 + q) * B + l16) * B;
            if (s < KS1) {
                const float2 w = R1[row + 4 * s + kg];
                R1r[q][s] = w.x;
                R1i[q][s] = w.y;
            }
            const float2 a = L1[row + 4 * kg + s], b = R2[row + 4 * kg + s], c = L2[row + 4 * kg + s];
            L1r[q][s] = a.x; L1i[q][s] = a.y;
            R2r[q][s] = b.x; R2i[q][s] = b.y;
            L2r[q][s] = c.x; L2i[q][s] = c.y;
        }

    const int64_t ntiles = (rows + TV - 1) / TV;
    const int nchunks = n / 16;                 // 16 n floats per tile, 256 per chunk
    const int64_t last_piece = rows * n - (F32 ? 4 : 8);
    const uint32_t xa_addr = lds_address(xa), xb_addr = lds_address(xb);
    // the 16 n contiguous elements of a tile of one array into an LDS row buffer (chunked layout); elements past
    // the end of the batch repeat the last piece and are never stored
    auto fetch_tile = [&](const T *src, int64_t base, float *dst, uint32_t dst_addr) {
        if constexpr (F32) {
            for (int q = wave; q < nchunks; q += 4) {
                int64_t at = base + 256 * q + 4 * lane;
                if (at > last_piece) at = last_piece;
                dma_16_at(src + at, dst_addr + (uint32_t)q * CH * 4);
            }
        } else {
            // instruction q moves elements 512 q + 8 lane .. + 7 of the tile (two chunks of 256)
            for (int q = wave; 512 * q < 16 * n; q += 4) {
                const int f = 512 * q + 8 * lane;
                if (f < 16 * n) {
                    int64_t at = base + f;
                    if (at > last_piece) at = last_piece;
                    const uint4 w = *reinterpret_cast<const uint4 *>(src + at);
                    float *d = dst + chunked(f);
                    *reinterpret_cast<f32x4 *>(d) = f32x4{__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xffff0000u),
                                                          __uint_as_float(w.y << 16), __uint_as_float(w.y & 0xffff0000u)};
                    *reinterpret_cast<f32x4 *>(d + 4) = f32x4{__uint_as_float(w.z << 16), __uint_as_float(w.z & 0xffff0000u),
                                                              __uint_as_float(w.w << 16), __uint_as_float(w.w & 0xffff0000u)};
                }
            }
        }
    };
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t r0 = tile * TV, base = r0 * n;
        // the kernel entries of S2, (re, im) of elements 16 (4 kg + r) + b0 .. + 3 of the row's channel, requested
        // first: they are in registers long before S2 needs them
        f32x4 k01[4], k23[4];
        {
            int64_t row = r0 + l16;
            if (row >= rows) row = rows - 1;
            const int h = (int)(row % H);
            const f32x4 *kq = Kq + ((size_t)(h >> 2) * 128 + (wave * 4 + kg) * 8) * 4 + (h & 3);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                k01[r] = kq[(2 * r) * 4];
                k23[r] = kq[(2 * r + 1) * 4];
            }
        }
        fetch_tile(u, base, xa, xa_addr);
        if (g_in) fetch_tile(g_in, base, xb, xb_addr);
        wait_loads_at_most<0>();
        __syncthreads();

        // ---- S1: real input, complex R1
        {
            f32x4 xq[KS1];
#pragma unroll
            for (int s = 0; s < KS1; ++s) {
                const int j = 16 * (4 * s + kg) + b0;
                const int at = chunked(l16 * n + j);
                f32x4 v = *reinterpret_cast<const f32x4 *>(xa + at);
                if (g_in) v *= *reinterpret_cast<const f32x4 *>(xb + at);
                xq[s] = j < n ? v : f32x4{0, 0, 0, 0};
            }
            // (eight accumulators in turn: an MFMA never waits for the one issued just before it)
            f32x4 ar[4], ai[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) ar[q] = ai[q] = f32x4{0, 0, 0, 0};
#pragma unroll
            for (int s = 0; s < KS1; ++s)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    ar[q] = mfma(R1r[q][s], xq[s][q], ar[q]);
                    ai[q] = mfma(R1i[q][s], xq[s][q], ai[q]);
                }
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    tr[l16 * LD + (4 * kg + r) * RS + b0 + q] = ar[q][r];
                    ti[l16 * LD + (4 * kg + r) * RS + b0 + q] = ai[q][r];
                }
        }
        __syncthreads();

        // ---- S2: complex L1, then the kernel of the row's channel
        {
            f32x4 zr[4], zi[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) zr[q] = zi[q] = f32x4{0, 0, 0, 0};
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                float tre[4], tim[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    tre[q] = tr[l16 * LD + (b0 + q) * RS + 4 * kg + s];
                    tim[q] = ti[l16 * LD + (b0 + q) * RS + 4 * kg + s];
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    zr[q] = mfma(L1r[q][s], tre[q], zr[q]);
                    zi[q] = mfma(L1r[q][s], tim[q], zi[q]);
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    zr[q] = mfma(L1i[q][s], -tim[q], zr[q]);
                    zi[q] = mfma(L1i[q][s], tre[q], zi[q]);
                }
            }
            // rows k = 4 kg + r of blocks i = b0 .. b0 + 3: elements 16 k + i
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const f32x4 kre = {k01[r][0], k01[r][2], k23[r][0], k23[r][2]}, kim = {k01[r][1], k01[r][3], k23[r][1], k23[r][3]};
                const f32x4 a = {zr[0][r], zr[1][r], zr[2][r], zr[3][r]}, b = {zi[0][r], zi[1][r], zi[2][r], zi[3][r]};
                *reinterpret_cast<f32x4 *>(xa + l16 * CH + 16 * (4 * kg + r) + b0) = a * kre - b * kim;
                *reinterpret_cast<f32x4 *>(xb + l16 * CH + 16 * (4 * kg + r) + b0) = a * kim + b * kre;
            }
        }
        __syncthreads();

        // ---- S3: complex R2 on the rows of z
        {
            f32x4 xr[4], xi[4];
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                xr[s] = *reinterpret_cast<const f32x4 *>(xa + l16 * CH + 16 * (4 * kg + s) + b0);
                xi[s] = *reinterpret_cast<const f32x4 *>(xb + l16 * CH + 16 * (4 * kg + s) + b0);
            }
            f32x4 ar[4], ai[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) ar[q] = ai[q] = f32x4{0, 0, 0, 0};
#pragma unroll
            for (int s = 0; s < 4; ++s) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    ar[q] = mfma(R2r[q][s], xr[s][q], ar[q]);
                    ai[q] = mfma(R2r[q][s], xi[s][q], ai[q]);
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    ar[q] = mfma(R2i[q][s], -xi[s][q], ar[q]);
                    ai[q] = mfma(R2i[q][s], xr[s][q], ai[q]);
                }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    tr[l16 * LD + (4 * kg + r) * RS + b0 + q] = ar[q][r];
                    ti[l16 * LD + (4 * kg + r) * RS + b0 + q] = ai[q][r];
                }
        }
        __syncthreads();   // z is consumed: the output gates land where Re z was while the last factor runs
        if (g_out) fetch_tile(g_out, base, xa, xa_addr);

        // ---- S4: real part of complex L2
        f32x4 o[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) o[q] = f32x4{0, 0, 0, 0};
#pragma unroll
        for (int s = 0; s < 4; ++s) {
#pragma unroll
            for (int q = 0; q < 4; ++q) o[q] = mfma(L2r[q][s], tr[l16 * LD + (b0 + q) * RS + 4 * kg + s], o[q]);
#pragma unroll
            for (int q = 0; q < 4; ++q) o[q] = mfma(L2i[q][s], -ti[l16 * LD + (b0 + q) * RS + 4 * kg + s], o[q]);
        }
        if (g_out) {
            wait_loads_at_most<0>();
            __syncthreads();
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int j = 16 * (4 * kg + r) + b0;
            if (j < n) {
                const int at = chunked(l16 * n + j);
                f32x4 v = {o[0][r], o[1][r], o[2][r], o[3][r]};
                if (g_out) v *= *reinterpret_cast<const f32x4 *>(xa + at);
                *reinterpret_cast<f32x4 *>(xb + at) = v;   // (Im z was consumed before the barrier after S3)
            }
        }
        __syncthreads();
        if constexpr (F32) {
            for (int q = wave; q < nchunks; q += 4) {
                const int64_t at = base + 256 * q + 4 * lane;
                if (at <= last_piece)   // (y is written once per launch: streaming stores)
                    __builtin_nontemporal_store(*reinterpret_cast<const f32x4 *>(xb + q * CH + 4 * lane), reinterpret_cast<f32x4 *>(y + at));
            }
        } else {
            for (int q = wave; 512 * q < 16 * n; q += 4) {
                const int f = 512 * q + 8 * lane;
                if (f < 16 * n && base + f <= last_piece) {
                    const f32x4 lo = *reinterpret_cast<const f32x4 *>(xb + chunked(f));
                    const f32x4 hi = *reinterpret_cast<const f32x4 *>(xb + chunked(f) + 4);
                    store_stream16(y + base + f, uint4{pack_bf16(lo[0], lo[1]), pack_bf16(lo[2], lo[3]), pack_bf16(hi[0], hi[1]), pack_bf16(hi[2], hi[3])});
                }
            }
        }
        __syncthreads();   // before the next tile's rows land
    }
}

static bool supported(int bs, int n, monarch_dtype) { return bs == 16 && n >= 16 && n % 16 == 0; }

static int launch(const void *u, const void *g_in, const void *g_out, const unsigned char *state, void *y, int64_t rows,
                  int H, int n, monarch_dtype dt, hipStream_t s)
{
    const blocky::Layout l = blocky::layout(H, 16);
    int dev = 0, ncu = 0;
    MONARCH_HIP_CHECK(hipGetDevice(&dev));
    MONARCH_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
    const int64_t ntiles = (rows + TV - 1) / TV;
    int64_t grid = 2 * (int64_t)ncu;
    if (grid > ntiles) grid = ntiles;
#define MONARCH_LAUNCH_BLOCKY16(T, KS)                                                                             \
    do {                                                                                                           \
        auto kern = conv_b16_kernel<T, KS>;                                                                        \
        MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,      \
                                              (int)LDS_BYTES));                                                    \
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), LDS_BYTES, s, (const T *)u, (const T *)g_in,     \
                           (const T *)g_out, (const float2 *)(state + l.R1), (const float2 *)(state + l.L1),       \
                           (const float2 *)(state + l.R2), (const float2 *)(state + l.L2),                         \
                           (const f32x4 *)(state + l.Kq), (T *)y, rows, H, n);                                     \
    } while (0)
    if (dt == MONARCH_F32) {
        if (n <= 128) MONARCH_LAUNCH_BLOCKY16(float, 2);
        else MONARCH_LAUNCH_BLOCKY16(float, 4);
    } else {
        if (n <= 128) MONARCH_LAUNCH_BLOCKY16(bf16_t, 2);
        else MONARCH_LAUNCH_BLOCKY16(bf16_t, 4);
    }
#undef MONARCH_LAUNCH_BLOCKY16
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

}  // namespace blocky16

bool blocky_fits(int bs) { return bs >= 2 && bs <= 64; }   // a row twice in LDS as complex float32: 64 KB at bs = 64

size_t blocky_state_bytes(int H, int bs) { return blocky::layout(H, bs).total; }

void blocky_state_offsets(int H, int bs, size_t out[5])
{
    const blocky::Layout l = blocky::layout(H, bs);
    out[0] = l.R1;
    out[1] = l.L1;
    out[2] = l.R2;
    out[3] = l.L2;
    out[4] = l.Kf;
}

int launch_blocky_prepare(const float *Lt, const float *Rt, const float *k, int H, int klen, int bs, int mask,
                          void *state, hipStream_t s)
{
    using namespace blocky;
    const int N = bs * bs;
    const Layout l = layout(H, bs);
    unsigned char *st = static_cast<unsigned char *>(state);
    cdouble *tw = reinterpret_cast<cdouble *>(st + l.tw);
    float2 *R1 = reinterpret_cast<float2 *>(st + l.R1), *L1 = reinterpret_cast<float2 *>(st + l.L1);
    float2 *R2 = reinterpret_cast<float2 *>(st + l.R2), *L2 = reinterpret_cast<float2 *>(st + l.L2);
    hipLaunchKernelGGL(twiddle_kernel, dim3((N + 255) / 256), dim3(256), 0, s, tw, N);
    const size_t lds_f = (size_t)N * sizeof(cdouble) + (bs + 1) * sizeof(int);
    if (lds_f > 64 * 1024)
        MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)factor_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_f));
    hipLaunchKernelGGL(factor_kernel, dim3(2 * bs), dim3(256), lds_f, s, Lt, Rt, (const cdouble *)tw, R1, L1, R2, L2, bs, mask);
    if (H > 0)
        hipLaunchKernelGGL(kf_kernel, dim3(H), dim3(THREADS), (size_t)2 * N * sizeof(float2), s, k, (const float2 *)R1,
                           (const float2 *)L1, reinterpret_cast<float2 *>(st + l.Kf),
                           bs == 16 ? reinterpret_cast<float4 *>(st + l.Kq) : (float4 *)nullptr, klen, bs);
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

int launch_blocky_conv(const void *u, const void *g_in, const void *g_out, const void *state, void *y, int64_t rows,
                       int H, int n, int bs, monarch_dtype dt, hipStream_t s)
{
    if (rows == 0 || n == 0) return MONARCH_OK;
    const unsigned char *st = static_cast<const unsigned char *>(state);
    if (blocky16::supported(bs, n, dt)) return blocky16::launch(u, g_in, g_out, st, y, rows, H, n, dt, s);
    if (blocky_inplace_takes(bs, n, dt)) {   // blocks of 32, 64: in place on LDS tiles on the matrix cores
        const blocky::Layout l = blocky::layout(H, bs);
        return launch_blocky_inplace(u, g_in, g_out, (const float2 *)(st + l.R1), (const float2 *)(st + l.L1), (const float2 *)(st + l.R2),
                                     (const float2 *)(st + l.L2), (const float2 *)(st + l.Kf), y, rows, H, n, bs, dt, s);
    }
    if (dt == MONARCH_F32) return blocky::launch_conv_typed<float>(u, g_in, g_out, st, y, rows, H, n, bs, s);
    return blocky::launch_conv_typed<bf16_t>(u, g_in, g_out, st, y, rows, H, n, bs, s);
}

}  // namespace monarch
