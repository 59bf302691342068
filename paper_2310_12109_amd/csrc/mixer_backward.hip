// Gradients of the sequence mixer y = g_out o M2 (K[h] o M1 (g_in o u)) (Sec. 3.2 Eq. 2, gated form; the chain
// rule through its five steps).  Composed from the order-2 product and its gradient kernels (csrc/matmul_mfma_b16,
// csrc/matmul_backward, csrc/generic) with three elementwise kernels between them; the intermediate rows travel
// through a workspace of the caller (five arrays of the size of u):
//   a = g_in o u            s = M1 a            t = K o s            w = M2 t                 (forward again)
//   dg_out = dy o w         dw = dy o g_out     (dt, dR2, dL2) = grad of M2 at (t, dw)
//   dK[h] = sum_b dt o s    ds = dt o K         (da, dR1, dL1) = grad of M1 at (a, ds)
//   du = da o g_in          dg_in = da o u
#include "kernels.h"

namespace monarch {

namespace mixb {

constexpr int THREADS = 256;

typedef __attribute__((ext_vector_type(4))) float f32x4;

// four consecutive elements as floats and back (every array here starts 16-byte aligned and N = bs^2 elements per
// row; the vector kernels run when N is a multiple of 4)
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

// out[i] = p[i] * q[i] (q null: copy of p); out2[i] = p[i] * q2[i] if out2.  V: elements per thread and step (4 or 1)
template <typename T, int V>
__global__ void product_kernel(const T *__restrict__ p, const T *__restrict__ q, const T *__restrict__ q2,
                               T *__restrict__ out, T *__restrict__ out2, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x * V;
    for (size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * V; i < n; i += stride) {
        if constexpr (V == 4) {
            const f32x4 v = ld4(p + i);
            if (out) st4(out + i, q ? v * ld4(q + i) : v);
            if (out2) st4(out2 + i, v * ld4(q2 + i));
        } else {
            const float v = to_f32(p[i]);
            if (out) out[i] = from_f32<T>(q ? v * to_f32(q[i]) : v);
            if (out2) out2[i] = from_f32<T>(v * to_f32(q2[i]));
        }
    }
}

// t[r, j] = K[r % H, j] * s[r, j]
template <typename T, int V>
__global__ void kernel_product_kernel(const T *__restrict__ s, const T *__restrict__ K, T *__restrict__ t, size_t n,
                                      size_t HN)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x * V;
    for (size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * V; i < n; i += stride) {
        if constexpr (V == 4) st4(t + i, ld4(s + i) * ld4(K + i % HN));
        else t[i] = from_f32<T>(to_f32(s[i]) * to_f32(K[i % HN]));
    }
}

// One thread per kernel entry (h, j): dK[h, j] = sum_b dt[b, h, j] s[b, h, j] (no atomics: the sum over the
// batch runs inside the thread, neighbouring threads read neighbouring addresses); ds = dt o K in place.
template <typename T, int V>
__global__ void kernel_gradient_kernel(T *__restrict__ dt_ds, const T *__restrict__ s, const T *__restrict__ K,
                                       float *__restrict__ dK, int64_t B, size_t HN)
{
    const size_t e = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * V;
    if (e >= HN) return;
    if constexpr (V == 4) {
        const f32x4 k = ld4(K + e);
        f32x4 acc = {0, 0, 0, 0};
        for (int64_t b = 0; b < B; ++b) {
            const size_t at = (size_t)b * HN + e;
            const f32x4 d = ld4(dt_ds + at);
            acc += d * ld4(s + at);
            st4(dt_ds + at, d * k);
        }
        if (dK) *reinterpret_cast<f32x4 *>(dK + e) = acc;
    } else {
        const float k = to_f32(K[e]);
        float acc = 0.0f;
        for (int64_t b = 0; b < B; ++b) {
            const size_t at = (size_t)b * HN + e;
            const float d = to_f32(dt_ds[at]);
            acc = fmaf(d, to_f32(s[at]), acc);
            dt_ds[at] = from_f32<T>(d * k);
        }
        if (dK) dK[e] = acc;
    }
}

__global__ void clear_kernel(float *p, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0.0f;
}

static unsigned blocks_for(size_t n)
{
    const size_t b = (n + THREADS - 1) / THREADS;
    return (unsigned)(b < 16384 ? (b ? b : 1) : 16384);
}

static int product(const void *x, const void *R, const void *L, void *y, int64_t rows, int bs, monarch_dtype dt,
                   hipStream_t s)
{
    if (matmul_mfma_b16_supported(bs, bs, bs, bs, bs, bs, dt)) return launch_matmul_mfma_b16(x, R, L, y, rows, dt, s);
    if (monarch_inplace_supported(bs, dt)) return launch_matmul_inplace(x, R, L, y, rows, bs, dt, s);   // blocks of 32, 64
    return launch_matmul_generic(x, R, L, nullptr, y, rows, bs, bs, bs, bs, bs, bs, 2, 0, dt, dt, dt, s);
}

template <typename T>
static int run(const void *u, const void *K, const void *g_in, const void *g_out, const void *R1, const void *L1,
               const void *R2, const void *L2, const void *dy, void *du, float *dK, void *dg_in, void *dg_out, float *dR1,
               float *dL1, float *dR2, float *dL2, int64_t B, int H, int bs, monarch_dtype dt, void *ws, hipStream_t st)
{
    const size_t N = (size_t)bs * bs, HN = (size_t)H * N, n = (size_t)B * HN;
    const int64_t rows = B * H;
    const size_t arr = ((n * sizeof(T) + 255) / 256) * 256;
    unsigned char *w8 = static_cast<unsigned char *>(ws);
    T *a = (T *)w8, *s = (T *)(w8 + arr), *t = (T *)(w8 + 2 * arr), *w = (T *)(w8 + 3 * arr), *x1 = (T *)(w8 + 4 * arr);
    const bool vec = N % 4 == 0;
    const unsigned g = blocks_for(vec ? n / 4 : n);
    auto launch_product = [&](const T *p, const T *q, const T *q2, T *out, T *out2) {
        if (vec) hipLaunchKernelGGL((product_kernel<T, 4>), dim3(g), dim3(THREADS), 0, st, p, q, q2, out, out2, n);
        else hipLaunchKernelGGL((product_kernel<T, 1>), dim3(g), dim3(THREADS), 0, st, p, q, q2, out, out2, n);
    };
    int rc;
    // forward again (nothing to do for an empty batch: the gradient kernels below then only clear their sums)
    const T *a_in = (const T *)u;
    if (rows > 0 && g_in) {
        launch_product((const T *)u, (const T *)g_in, (const T *)nullptr, a, (T *)nullptr);
        a_in = a;
    }
    if (rows > 0) {
        if ((rc = product(a_in, R1, L1, s, rows, bs, dt, st))) return rc;
        if (vec) hipLaunchKernelGGL((kernel_product_kernel<T, 4>), dim3(g), dim3(THREADS), 0, st, (const T *)s, (const T *)K, t, n, HN);
        else hipLaunchKernelGGL((kernel_product_kernel<T, 1>), dim3(g), dim3(THREADS), 0, st, (const T *)s, (const T *)K, t, n, HN);
    }
    const T *dw = (const T *)dy;
    if (rows > 0 && g_out) {
        if (dg_out)
            if ((rc = product(t, R2, L2, w, rows, bs, dt, st))) return rc;
        // dw = dy o g_out, dg_out = dy o w
        launch_product((const T *)dy, (const T *)g_out, dg_out ? (const T *)w : (const T *)nullptr, x1,
                       dg_out ? (T *)dg_out : (T *)nullptr);
        dw = x1;
    }
    // through M2: dt (into w's array), dR2, dL2
    if ((rc = launch_matmul_backward(t, R2, L2, dw, w, dR2, dL2, rows, bs, bs, bs, bs, bs, bs, dt, st))) return rc;
    // dK and ds = dt o K (in place).  An empty batch reads nothing (its inputs may be NULL): dK is only cleared.
    if (rows == 0) {
        if (dK) hipLaunchKernelGGL(clear_kernel, dim3(blocks_for(HN)), dim3(THREADS), 0, st, dK, HN);
    } else if (vec)
        hipLaunchKernelGGL((kernel_gradient_kernel<T, 4>), dim3((unsigned)((HN / 4 + 63) / 64)), dim3(64), 0, st, w, (const T *)s,
                           (const T *)K, dK, B, HN);
    else
        hipLaunchKernelGGL((kernel_gradient_kernel<T, 1>), dim3((unsigned)((HN + THREADS - 1) / THREADS)), dim3(THREADS), 0, st, w,
                           (const T *)s, (const T *)K, dK, B, HN);
    // through M1: da (into t's array, or straight into du without an input gate), dR1, dL1
    const bool need_da = du || dg_in;
    T *da = g_in ? t : (T *)du;
    if ((rc = launch_matmul_backward(a_in, R1, L1, w, need_da ? da : nullptr, dR1, dL1, rows, bs, bs, bs, bs, bs, bs, dt, st)))
        return rc;
    if (rows > 0 && g_in && need_da)
        launch_product((const T *)da, du ? (const T *)g_in : (const T *)nullptr, dg_in ? (const T *)u : (const T *)nullptr,
                       du ? (T *)du : (T *)nullptr, dg_in ? (T *)dg_in : (T *)nullptr);
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

}  // namespace mixb

size_t mixer_backward_workspace_bytes(int64_t B, int H, int bs, monarch_dtype dt)
{
    const size_t n = (size_t)B * H * bs * bs, es = dt == MONARCH_F32 ? 4 : 2;
    return 5 * (((n * es + 255) / 256) * 256);
}

int launch_mixer_backward(const void *u, const void *K, const void *g_in, const void *g_out, const void *R1,
                          const void *L1, const void *R2, const void *L2, const void *dy, void *du, float *dK, void *dg_in,
                          void *dg_out, float *dR1, float *dL1, float *dR2, float *dL2, int64_t B, int H, int bs,
                          monarch_dtype dt, void *ws, hipStream_t s)
{
    if (dt == MONARCH_F32)
        return mixb::run<float>(u, K, g_in, g_out, R1, L1, R2, L2, dy, du, dK, dg_in, dg_out, dR1, dL1, dR2, dL2, B, H, bs, dt, ws, s);
    return mixb::run<bf16_t>(u, K, g_in, g_out, R1, L1, R2, L2, dy, du, dK, dg_in, dg_out, dR1, dL1, dR2, dL2, B, H, bs, dt, ws, s);
}

}  // namespace monarch
