// The gated-convolution layer of the paper's models (appendix algorithm "M2 Hyena layer with heads" at head
// dimension 1; with causal = 0 the bidirectional gated convolution of the M2-BERT sequence mixer, Sec. 5):
//   [X1; X2; V] = W_in u_t + b_in                      three dense projections of every position
//   X1~, X2~, V~ = short causal depthwise convolutions along the sequence
//   O = X1~ o conv(k_long, X2~ o V~)                   monarch_causal_conv with X2~ as input gate and X1~ as output gate
//   y_t = W_out O[:, t] + b_out
// The dense projections are plain GEMMs and go to rocBLAS (loaded on first use: the rest of the library does not
// depend on it), written so that their results land in the (B, d, n) layout of the convolution and back in
// (B, n, d) without a transpose pass; the short convolutions (with the projection bias) are one memory-bound kernel;
// the long convolution is the library's own entry point.
// With a head dimension d_h > 1 (the same algorithm with its heads): the features are grouped in d / d_h heads, the long
// kernel has one row per head, and per head and position
//   XV[i][j] = conv(k_long[head], X2~[i] o V~[j]),  O[j] = sum_i X1~[i] o XV[i][j]          i, j < d_h
// i.e. d_h^2 long convolutions per head.  Here: the d_h^2 products of a head are batch rows of one channel of the long
// convolution (a head's kernel spectrum is formed once per workgroup as for any batch), and one kernel forms the gated
// sum over i in fp32.  For 16-bit tensors and nfft = 2048 = 64 x 32 the fused convolution kernel reads X2~[i] and V~[j]
// through the head's index map and forms the products on its loads; otherwise one kernel writes them as a
// (B d_h^2, d / d_h, n) tensor for the library's convolution.
#include <dlfcn.h>
#include <mutex>

#include <rocblas/rocblas.h>

#include "kernels.h"
#include "monarch.h"

namespace monarch {

namespace hyena {

struct Blas {
    void *so = nullptr;
    decltype(&rocblas_create_handle) create = nullptr;
    decltype(&rocblas_set_stream) set_stream = nullptr;
    decltype(&rocblas_gemm_strided_batched_ex) gemm = nullptr;
    rocblas_handle handle[16] = {};
};
static Blas g_blas;
static std::mutex g_blas_mutex;

// the handle of the current device (created once per device), or null with the error text set
static rocblas_handle blas_handle()
{
    std::lock_guard<std::mutex> lock(g_blas_mutex);
    if (!g_blas.so) {
        void *so = dlopen("librocblas.so", RTLD_NOW | RTLD_LOCAL);
        if (!so) so = dlopen("/opt/rocm/lib/librocblas.so", RTLD_NOW | RTLD_LOCAL);
        if (!so) {
            fail(MONARCH_EHIP, "the dense projections need rocBLAS, which could not be loaded: %s", dlerror());
            return nullptr;
        }
        g_blas.create = (decltype(g_blas.create))dlsym(so, "rocblas_create_handle");
        g_blas.set_stream = (decltype(g_blas.set_stream))dlsym(so, "rocblas_set_stream");
        g_blas.gemm = (decltype(g_blas.gemm))dlsym(so, "rocblas_gemm_strided_batched_ex");
        if (!g_blas.create || !g_blas.set_stream || !g_blas.gemm) {
            fail(MONARCH_EHIP, "rocBLAS lacks an entry point the dense projections need");
            return nullptr;
        }
        g_blas.so = so;
    }
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) {
        fail(MONARCH_EHIP, "no current device for the dense projections");
        return nullptr;
    }
    if (!g_blas.handle[dev] && g_blas.create(&g_blas.handle[dev]) != rocblas_status_success) {
        g_blas.handle[dev] = nullptr;
        fail(MONARCH_EHIP, "rocblas_create_handle failed");
        return nullptr;
    }
    return g_blas.handle[dev];
}

// C (row-major, per batch entry) = op over row-major operands, as one strided-batched GEMM in rocBLAS's
// column-major terms.  All of type dt, fp32 accumulation.
static int gemm(rocblas_handle h, rocblas_operation ta, rocblas_operation tb, int m, int n, int k, const void *a, int lda,
                int64_t sa, const void *b, int ldb, int64_t sb, float beta, void *c, int ldc, int64_t sc, int batch,
                monarch_dtype dt)
{
    const float alpha = 1.0f;
    const rocblas_datatype t = dt == MONARCH_F32 ? rocblas_datatype_f32_r : rocblas_datatype_bf16_r;
    const rocblas_status st = g_blas.gemm(h, ta, tb, m, n, k, &alpha, a, t, lda, sa, b, t, ldb, sb, &beta, c, t, ldc, sc, c, t, ldc,
                                          sc, batch, rocblas_datatype_f32_r, rocblas_gemm_algo_standard, 0, 0);
    if (st != rocblas_status_success) return fail(MONARCH_EHIP, "rocBLAS GEMM failed with status %d", (int)st);
    return MONARCH_OK;
}

// eight consecutive elements with 16-byte accesses (p 16-byte aligned)
__device__ __forceinline__ void load8(const float *p, float (&v)[8])
{
    const float4 a = reinterpret_cast<const float4 *>(p)[0], b = reinterpret_cast<const float4 *>(p)[1];
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16_t *p, float (&v)[8])
{
    const uint4 w = *reinterpret_cast<const uint4 *>(p);
    const uint32_t d[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        v[2 * e] = __uint_as_float(d[e] << 16);
        v[2 * e + 1] = __uint_as_float(d[e] & 0xffff0000u);
    }
}
__device__ __forceinline__ void store8(float *p, const float (&v)[8])
{
    reinterpret_cast<float4 *>(p)[0] = make_float4(v[0], v[1], v[2], v[3]);
    reinterpret_cast<float4 *>(p)[1] = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ __forceinline__ void store8(bf16_t *p, const float (&v)[8])
{
    bf16_t h[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) h[e] = from_f32<bf16_t>(v[e]);
    *reinterpret_cast<uint4 *>(p) = *reinterpret_cast<const uint4 *>(h);
}

// out[r][t] = sum_tau ks[row kernel][tau] (in[r'][t - tau] + bias[row kernel]), rows r = (i, b, c) of the (3, B, d, n)
// tensor with kernel / bias row i d + c; the input is the projections' (B, 3, d, n) tensor, r' = (b, i, c): the three
// projections of a batch entry are one GEMM.  8 consecutive t per thread (16-byte accesses), the taps before them
// from the preceding piece.
template <typename T>
__global__ __launch_bounds__(256) void short_conv_kernel(const T *__restrict__ in, T *__restrict__ out, const T *__restrict__ ks,
                                                         const T *__restrict__ bias, int64_t rows, int Bd, int d, int n, int taps)
{
    const int pieces = n / 8;
    const int64_t total = rows * pieces;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = idx / pieces;
        const int p = (int)(idx - r * pieces);
        const int i3 = (int)(r / Bd), rem = (int)(r - (int64_t)i3 * Bd), b = rem / d, c = rem - b * d;
        const int kr = i3 * d + c;                          // r = (i B + b) d + c  ->  i d + c
        const int64_t rs = ((int64_t)b * 3 + i3) * d + c;   // the same row of the (B, 3, d, n) input
        float w[8], x[16], o[8];
#pragma unroll
        for (int tau = 0; tau < 8; ++tau) w[tau] = tau < taps ? to_f32(ks[(int64_t)kr * taps + tau]) : 0.0f;
        const float bv = bias ? to_f32(bias[kr]) : 0.0f;
        const T *src = in + rs * n + 8 * p;
        float cur[8], prev[8];
        load8(src, cur);
        load8(p > 0 ? src - 8 : src, prev);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            x[8 + e] = cur[e] + bv;
            x[e] = p > 0 ? prev[e] + bv : 0.0f;   // positions before the start of the row contribute nothing
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float acc = 0.0f;
#pragma unroll
            for (int tau = 0; tau < 8; ++tau) acc = fmaf(w[tau], x[8 + e - tau], acc);
            o[e] = acc;
        }
        store8(out + r * n + 8 * p, o);
    }
}

// y[b][t][c] = bias[c] (the output projection then accumulates onto it); d a multiple of 8: 16-byte stores
template <typename T>
__global__ __launch_bounds__(256) void bias_rows_kernel(T *__restrict__ y, const T *__restrict__ bias, int64_t total, int d)
{
    if (d % 8 == 0) {
        for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; 8 * idx < total; idx += (int64_t)gridDim.x * blockDim.x) {
            float v[8];
            load8(bias + (8 * idx) % d, v);
            store8(y + 8 * idx, v);
        }
        return;
    }
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * blockDim.x)
        y[idx] = bias[idx % d];
}

// xv[((b dh + i) dh + j) heads + head][t] = x2[b][head dh + i][t] x v[b][head dh + j][t]: the outer products of a head
// as batch rows of the long convolution.  A thread holds 8 consecutive t of one x2 row and writes its products with
// the dh rows of v.
template <typename T>
__global__ __launch_bounds__(256) void heads_outer_kernel(const T *__restrict__ x2, const T *__restrict__ v, T *__restrict__ xv,
                                                          int64_t total, int heads, int dh, int d, int n)
{
    const int pieces = n / 8;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = idx / pieces;                     // b d + head dh + i: a row of x2
        const int p = (int)(idx - r * pieces);
        const int c = (int)(r % d), head = c / dh, i = c - head * dh;
        const int64_t b = r / d;
        float a[8];
        load8(x2 + r * n + 8 * p, a);
        const T *vrow = v + ((b * d + head * dh) * n + 8 * p);
        T *dst = xv + ((((b * dh + i) * dh) * heads + head) * n + 8 * p);
        for (int j = 0; j < dh; ++j) {
            float w[8], o[8];
            load8(vrow + (int64_t)j * n, w);
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = a[e] * w[e];
            store8(dst + (int64_t)j * heads * n, o);
        }
    }
}

// o[b][head dh + j][t] = sum_i x1[b][head dh + i][t] x yv[((b dh + i) dh + j) heads + head][t], the sum in fp32
template <typename T>
__global__ __launch_bounds__(256) void heads_sum_kernel(const T *__restrict__ x1, const T *__restrict__ yv, T *__restrict__ o,
                                                        int64_t total, int heads, int dh, int d, int n)
{
    const int pieces = n / 8;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = idx / pieces;                     // b d + head dh + j
        const int p = (int)(idx - r * pieces);
        const int c = (int)(r % d), head = c / dh, j = c - head * dh;
        const int64_t b = r / d;
        float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int i = 0; i < dh; ++i) {
            float g[8], y[8];
            load8(x1 + ((b * d + head * dh + i) * n + 8 * p), g);
            load8(yv + ((((b * dh + i) * dh + j) * heads + head) * n + 8 * p), y);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = fmaf(g[e], y[e], acc[e]);
        }
        store8(o + r * n + 8 * p, acc);
    }
}

template <typename T>
static int run(const void *u, const void *W_in, const void *b_in, const void *k_short, const void *k_long, const void *W_out,
               const void *b_out, void *y, int B, int n, int d, int taps, int klen, int nfft, const int *factors, int nf, int causal,
               int dh, monarch_dtype dt, void *ws, size_t ws_bytes, hipStream_t s)
{
    rocblas_handle h = blas_handle();
    if (!h) return MONARCH_EHIP;
    if (g_blas.set_stream(h, s) != rocblas_status_success) return fail(MONARCH_EHIP, "rocblas_set_stream failed");
    const size_t es = sizeof(T);
    const int64_t plane = (int64_t)B * d * n;              // one (B, d, n) tensor
    char *base = (char *)ws;
    T *proj = (T *)base, *shrt = (T *)(base + align_up(3 * plane * es, 256)), *o = (T *)(base + 2 * align_up(3 * plane * es, 256));
    char *after_o = base + 2 * align_up(3 * plane * es, 256) + align_up(plane * es, 256);
    const size_t outer_bytes = dh > 1 ? align_up((size_t)dh * plane * es, 256) : 0;   // B dh^2 (d / dh) n elements
    T *xv = (T *)after_o, *yv = (T *)(after_o + outer_bytes);
    char *conv_ws = after_o + 2 * outer_bytes;
    const size_t conv_ws_bytes = ws_bytes - (size_t)(conv_ws - base);

    // 1. projections: proj[b] (3 d x n) = W_in (3 d x d) times u[b]^T.  fp32: one batched GEMM; bf16: one per projection
    //    (measured in one session at B = 8, n = 1024, d = 768: fp32 401 against 422 us per layer, bf16 109 against 103 us)
    const int parts = dt == MONARCH_F32 ? 1 : 3;
    for (int i = 0; i < parts; ++i) {
        int rc = gemm(h, rocblas_operation_transpose, rocblas_operation_none, n, 3 * d / parts, d, u, d, (int64_t)n * d,
                      (const T *)W_in + (int64_t)i * d * d, d, 0, 0.0f, proj + (int64_t)i * d * n, n, (int64_t)3 * d * n, B, dt);
        if (rc) return rc;
    }
    // 2. short depthwise convolutions (with the projection bias)
    {
        const int64_t rows = (int64_t)3 * B * d, total = rows * (n / 8);
        const int64_t blocks = (total + 255) / 256;
        hipLaunchKernelGGL(short_conv_kernel<T>, dim3((unsigned)(blocks > 65536 ? 65536 : blocks)), dim3(256), 0, s, proj, shrt,
                           (const T *)k_short, (const T *)b_in, rows, B * d, d, n, taps);
        MONARCH_HIP_CHECK(hipGetLastError());
    }
    // 3. O = X1~ o conv(k_long, X2~ o V~); with heads: outer products, d_h^2 convolutions per head, gated sum
    if (dh > 1) {
        const int heads = d / dh;
        if (conv_mfma_2048_supported(n, klen, factors, nf, dt)) {
            // the fused 64 x 32 kernel reads V~[j] and X2~[i] through the head's index map: no tensor of outer products
            int rc = launch_conv_mfma_2048_heads(shrt + 2 * plane, k_long, shrt + plane, yv, B, heads, dh, n, klen, dt, s);
            if (rc) return rc;
        } else {
            const int64_t total = (int64_t)B * d * (n / 8), blocks = (total + 255) / 256;
            hipLaunchKernelGGL(heads_outer_kernel<T>, dim3((unsigned)(blocks > (1 << 20) ? (1 << 20) : blocks)), dim3(256), 0, s,
                               shrt + plane, shrt + 2 * plane, xv, total, heads, dh, d, n);
            MONARCH_HIP_CHECK(hipGetLastError());
            int rc = monarch_causal_conv(xv, k_long, nullptr, nullptr, yv, B * dh * dh, heads, n, klen, nfft, factors, nf, causal, dt,
                                         conv_ws, conv_ws_bytes, (monarch_stream_t)s);
            if (rc) return rc;
        }
        const int64_t total_o = (int64_t)B * d * (n / 8), blocks_o = (total_o + 255) / 256;
        hipLaunchKernelGGL(heads_sum_kernel<T>, dim3((unsigned)(blocks_o > (1 << 20) ? (1 << 20) : blocks_o)), dim3(256), 0, s, shrt, yv, o,
                           total_o, heads, dh, d, n);
        MONARCH_HIP_CHECK(hipGetLastError());
    } else {
        int rc = monarch_causal_conv(shrt + 2 * plane, k_long, shrt + plane, shrt, o, B, d, n, klen, nfft, factors, nf, causal, dt, conv_ws,
                                     conv_ws_bytes, (monarch_stream_t)s);
        if (rc) return rc;
    }
    // 4. y[b] (n x d) = O[b]^T W_out^T (+ b_out, put there first)
    float beta = 0.0f;
    if (b_out) {
        const int64_t total = (int64_t)B * n * d, blocks = (total / 8 + 255) / 256;
        hipLaunchKernelGGL(bias_rows_kernel<T>, dim3((unsigned)(blocks > 65536 ? 65536 : blocks)), dim3(256), 0, s, (T *)y, (const T *)b_out,
                           total, d);
        MONARCH_HIP_CHECK(hipGetLastError());
        beta = 1.0f;
    }
    return gemm(h, rocblas_operation_transpose, rocblas_operation_transpose, d, n, d, W_out, d, 0, o, n, (int64_t)d * n, beta, y, d,
                (int64_t)n * d, B, dt);
}

}  // namespace hyena

size_t hyena_layer_workspace_bytes(int B, int n, int d, int klen, int nfft, const int *factors, int nf, int head_dim, monarch_dtype dt)
{
    const size_t es = dtype_size(dt), plane = (size_t)B * d * n * es;
    const size_t outer = head_dim > 1 ? 2 * align_up((size_t)head_dim * plane, 256) : 0;
    const int conv_B = B * head_dim * head_dim, conv_H = d / head_dim;
    return 2 * align_up(3 * plane, 256) + align_up(plane, 256) + outer +
           monarch_causal_conv_workspace_bytes(conv_B, conv_H, n, klen, nfft, factors, nf, dt);
}

int launch_hyena_layer(const void *u, const void *W_in, const void *b_in, const void *k_short, const void *k_long, const void *W_out,
                       const void *b_out, void *y, int B, int n, int d, int taps, int klen, int nfft, const int *factors, int nf,
                       int causal, int head_dim, monarch_dtype dt, void *ws, size_t ws_bytes, hipStream_t s)
{
    if (dt == MONARCH_F32)
        return hyena::run<float>(u, W_in, b_in, k_short, k_long, W_out, b_out, y, B, n, d, taps, klen, nfft, factors, nf, causal, head_dim, dt,
                                 ws, ws_bytes, s);
    return hyena::run<bf16_t>(u, W_in, b_in, k_short, k_long, W_out, b_out, y, B, n, d, taps, klen, nfft, factors, nf, causal, head_dim, dt, ws,
                              ws_bytes, s);
}

}  // namespace monarch
