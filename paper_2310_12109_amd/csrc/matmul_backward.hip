// Gradients of the order-2 Monarch product y = P3 L P2 R P1 x (Sec. 3.1) with respect to x, R and L, given
// dy, by the chain rule through the five steps of the product:
//   forward   t0 = P1 x,  t1 = R t0,  t2 = P2 t1,  (t3 = L t2,  y = P3 t3)
//   backward  g3 = P3^T dy,  dL_k += g3_k t2_k^T,  g2 = L^T g3,  g1 = P2^T g2,  dR_k += g1_k t0_k^T,
//             dx = P1^T R^T g1
// fp32 arithmetic on tiles of vectors held in LDS; the permutations are LDS index maps (t0 and g3 are
// written permuted, t2 and g1 are produced permuted).  Workgroups are persistent and walk over the tiles;
// the parameter gradients, sums over the whole batch, are accumulated per workgroup (in registers when a
// thread's share of the entries is at most EPT, else added to memory after every tile) and leave with one
// floating-point atomic add per entry.  The caller's dR / dL are cleared by a fill kernel first.
#include "kernels.h"

namespace monarch {

namespace mmb {

constexpr int THREADS = 256, EPT = 32;

__global__ void fill_zero_kernel(float *a, size_t na, float *b, size_t nb)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < na + nb; i += stride) {
        if (i < na) a[i] = 0.0f;
        else b[i - na] = 0.0f;
    }
}

struct Dims {
    int nbR, r_out, r_in, nbL, l_out, l_in;
};

// KEEP: this thread's entries of dR / dL stay in registers over all tiles of the workgroup.
template <typename T, int TV, bool KEEP>
__global__ __launch_bounds__(THREADS) void matmul_backward_kernel(
    const T *__restrict__ x, const T *__restrict__ R, const T *__restrict__ L, const T *__restrict__ dy,
    T *__restrict__ dx, float *__restrict__ dR, float *__restrict__ dL, int64_t batch, const Dims d)
{
    extern __shared__ float lds[];
    const int nbR = d.nbR, r_out = d.r_out, r_in = d.r_in, nbL = d.nbL, l_out = d.l_out, l_in = d.l_in;
    const int d_in = nbR * r_in, d_mid = nbR * r_out, d_out = nbL * l_out;
    float *t0 = lds;                  // [TV][d_in]   t0[k r_in + c]  = x[c nbR + k]
    float *g3 = t0 + TV * d_in;       // [TV][d_out]  g3[k l_out + r] = dy[r nbL + k]
    float *t2 = g3 + TV * d_out;      // [TV][d_mid]  input of L: t2[r nbR + k] = (R t0)[k r_out + r]
    float *g1 = t2 + TV * d_mid;      // [TV][d_mid]  gradient of R's output: g1[k r_out + r] = (L^T g3)[r nbR + k]
    const int tid = threadIdx.x;
    const int nR = nbR * r_out * r_in, nL = nbL * l_out * l_in;
    const int nRw = dR ? nR : 0, nLw = dL ? nL : 0;   // entries wanted
    const int64_t ntiles = (batch + TV - 1) / TV;

    float keep[KEEP ? EPT : 1];
#pragma unroll
    for (int i = 0; i < (KEEP ? EPT : 1); ++i) keep[i] = 0.0f;

    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t v0 = tile * TV;
        for (int idx = tid; idx < TV * d_in; idx += THREADS) {
            const int v = idx / d_in, j = idx - v * d_in;   // j = c nbR + k
            const int c = j / nbR, k = j - c * nbR;
            t0[v * d_in + k * r_in + c] = v0 + v < batch ? to_f32(x[(v0 + v) * d_in + j]) : 0.0f;
        }
        for (int idx = tid; idx < TV * d_out; idx += THREADS) {
            const int v = idx / d_out, i = idx - v * d_out;   // i = r nbL + k
            const int r = i / nbL, k = i - r * nbL;
            g3[v * d_out + k * l_out + r] = v0 + v < batch ? to_f32(dy[(v0 + v) * d_out + i]) : 0.0f;
        }
        __syncthreads();
        for (int o = tid; o < d_mid; o += THREADS) {   // o = k r_out + r
            const int k = o / r_out, r = o - k * r_out;
            float acc[TV];
#pragma unroll
            for (int v = 0; v < TV; ++v) acc[v] = 0.0f;
            const T *w = R + (size_t)o * r_in;
            for (int c = 0; c < r_in; ++c) {
                const float wv = to_f32(w[c]);
#pragma unroll
                for (int v = 0; v < TV; ++v) acc[v] = fmaf(wv, t0[v * d_in + k * r_in + c], acc[v]);
            }
#pragma unroll
            for (int v = 0; v < TV; ++v) t2[v * d_mid + r * nbR + k] = acc[v];
        }
        for (int o = tid; o < d_mid; o += THREADS) {   // o = k' l_in + a = r nbR + k
            const int kk = o / l_in, a = o - kk * l_in;
            float acc[TV];
#pragma unroll
            for (int v = 0; v < TV; ++v) acc[v] = 0.0f;
            const T *w = L + (size_t)kk * l_out * l_in + a;
            for (int r = 0; r < l_out; ++r) {
                const float wv = to_f32(w[(size_t)r * l_in]);
#pragma unroll
                for (int v = 0; v < TV; ++v) acc[v] = fmaf(wv, g3[v * d_out + kk * l_out + r], acc[v]);
            }
            const int r = o / nbR, k = o - r * nbR;
#pragma unroll
            for (int v = 0; v < TV; ++v) g1[v * d_mid + k * r_out + r] = acc[v];
        }
        __syncthreads();
        if (dx) {
            for (int o = tid; o < d_in; o += THREADS) {   // o = k r_in + c
                const int k = o / r_in, c = o - k * r_in;
                float acc[TV];
#pragma unroll
                for (int v = 0; v < TV; ++v) acc[v] = 0.0f;
                const T *w = R + (size_t)k * r_out * r_in + c;
                for (int r = 0; r < r_out; ++r) {
                    const float wv = to_f32(w[(size_t)r * r_in]);
#pragma unroll
                    for (int v = 0; v < TV; ++v) acc[v] = fmaf(wv, g1[v * d_mid + k * r_out + r], acc[v]);
                }
#pragma unroll
                for (int v = 0; v < TV; ++v)
                    if (v0 + v < batch) dx[(v0 + v) * d_in + c * nbR + k] = from_f32<T>(acc[v]);
            }
        }
        // entry e < nRw: dR[k][r][c] (e = (k r_out + r) r_in + c); then dL[k][r][a]
        int slot = 0;
        for (int e = tid; e < nRw + nLw; e += THREADS, ++slot) {
            float s = 0.0f;
            if (e < nRw) {
                const int o = e / r_in, c = e - o * r_in, k = o / r_out;
#pragma unroll
                for (int v = 0; v < TV; ++v) s = fmaf(g1[v * d_mid + o], t0[v * d_in + k * r_in + c], s);
            } else {
                const int el = e - nRw, o = el / l_in, a = el - o * l_in, k = o / l_out;
#pragma unroll
                for (int v = 0; v < TV; ++v) s = fmaf(g3[v * d_out + o], t2[v * d_mid + k * l_in + a], s);
            }
            if (KEEP) {
#pragma unroll
                for (int i = 0; i < EPT; ++i)   // (constant register index: no scratch memory)
                    if (i == slot) keep[i] += s;
            } else {
                atomicAdd(e < nRw ? dR + e : dL + (e - nRw), s);
            }
        }
        __syncthreads();
    }
    if (KEEP) {
#pragma unroll
        for (int i = 0; i < EPT; ++i) {
            const int e = tid + i * THREADS;
            if (e < nRw + nLw) atomicAdd(e < nRw ? dR + e : dL + (e - nRw), keep[i]);
        }
    }
}

static size_t lds_bytes(const Dims &d, int tv)
{
    return (size_t)tv * ((size_t)d.nbR * d.r_in + (size_t)d.nbL * d.l_out + 2 * (size_t)d.nbR * d.r_out) * sizeof(float);
}

template <typename T>
static int launch_typed(const void *x, const void *R, const void *L, const void *dy, void *dx, float *dR, float *dL,
                        int64_t batch, const Dims &d, hipStream_t s)
{
    int tv = 8;
    while (tv > 1 && lds_bytes(d, tv) > 64 * 1024) tv >>= 1;
    const size_t lds = lds_bytes(d, tv);
    if (lds > 160 * 1024) return fail(MONARCH_ESHAPE, "a row of the backward pass does not fit in LDS");
    int dev = 0, ncu = 0;
    MONARCH_HIP_CHECK(hipGetDevice(&dev));
    MONARCH_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
    const int64_t ntiles = (batch + tv - 1) / tv;
    int64_t grid = (int64_t)ncu * (lds <= 40 * 1024 ? 4 : lds <= 80 * 1024 ? 2 : 1);
    if (grid > ntiles) grid = ntiles;
    const size_t nR = dR ? (size_t)d.nbR * d.r_out * d.r_in : 0, nL = dL ? (size_t)d.nbL * d.l_out * d.l_in : 0;
    if (nR + nL) {
        hipLaunchKernelGGL(fill_zero_kernel, dim3(64), dim3(256), 0, s, dR, nR, dL, nL);
        MONARCH_HIP_CHECK(hipGetLastError());
    }
    if (ntiles == 0) return MONARCH_OK;   // empty batch: the parameter gradients are the zeros just written
    const bool keep = nR + nL <= (size_t)EPT * THREADS;
#define MONARCH_LAUNCH_MMB(TVV, KEEPV)                                                                              \
    do {                                                                                                            \
        auto kern = matmul_backward_kernel<T, TVV, KEEPV>;                                                          \
        if (lds > 64 * 1024)                                                                                        \
            MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,   \
                                                  (int)lds));                                                       \
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(THREADS), lds, s, (const T *)x, (const T *)R,           \
                           (const T *)L, (const T *)dy, (T *)dx, dR, dL, batch, d);                                 \
    } while (0)
#define MONARCH_LAUNCH_MMB_TV(KEEPV)                     \
    do {                                                 \
        switch (tv) {                                    \
        case 8: MONARCH_LAUNCH_MMB(8, KEEPV); break;     \
        case 4: MONARCH_LAUNCH_MMB(4, KEEPV); break;     \
        case 2: MONARCH_LAUNCH_MMB(2, KEEPV); break;     \
        default: MONARCH_LAUNCH_MMB(1, KEEPV); break;    \
        }                                                \
    } while (0)
    if (keep) MONARCH_LAUNCH_MMB_TV(true);
    else MONARCH_LAUNCH_MMB_TV(false);
#undef MONARCH_LAUNCH_MMB_TV
#undef MONARCH_LAUNCH_MMB
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

}  // namespace mmb

bool matmul_backward_fits(int nbR, int r_out, int r_in, int nbL, int l_out, int l_in)
{
    const mmb::Dims d = {nbR, r_out, r_in, nbL, l_out, l_in};
    return mmb::lds_bytes(d, 1) <= 160 * 1024;
}

int launch_matmul_backward(const void *x, const void *R, const void *L, const void *dy, void *dx, float *dR,
                           float *dL, int64_t batch, int nbR, int r_out, int r_in, int nbL, int l_out, int l_in,
                           monarch_dtype dt, hipStream_t s)
{
    const mmb::Dims d = {nbR, r_out, r_in, nbL, l_out, l_in};
    if (dt == MONARCH_F32) return mmb::launch_typed<float>(x, R, L, dy, dx, dR, dL, batch, d, s);
    return mmb::launch_typed<bf16_t>(x, R, L, dy, dx, dR, dL, batch, d, s);
}

}  // namespace monarch
