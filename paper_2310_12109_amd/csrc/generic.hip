// Shape-generic kernels with fp32 arithmetic: the fall-back path of every entry point.
//
//  * matmul_generic_kernel: order-2 Monarch product (Sec. 3.1) or a single block-diagonal
//    factor on a tile of vectors held in LDS; the permutations P are LDS index maps.
//  * fft_pass_kernel: one block-diagonal factor of the Monarch DFT (appendix, DFT corollary)
//    with the twiddle diagonal folded in, reading and writing complex fp32 rows in global
//    memory.  Chaining nf of them gives F_N; conjugating on load/store gives the inverse.
#include "kernels.h"

namespace monarch {

// ------------------------------------------------------------------------------------------
// Order-2 Monarch / block-diagonal product on LDS tiles
// ------------------------------------------------------------------------------------------

// One block-diagonal factor W = [nb][rout][rin] applied to TV vectors in LDS.
// in : element (v, block k, col c) at in [v*in_ld  + c*cs_in  + k*ks_in ]
// out: element (v, block k, row r) at out[v*out_ld + r*rs_out + k*ks_out]
// The two stride pairs are how the permutations of M = P L P R P are realised.
template <typename TW, int TV>
__device__ __forceinline__ void blockdiag_apply(const float *in, int in_ld, int cs_in, int ks_in,
                                                float *out, int out_ld, int rs_out, int ks_out,
                                                const TW *W, int nb, int rout, int rin,
                                                const TW *bias, int act)
{
    const int total = nb * rout;
    for (int o = threadIdx.x; o < total; o += blockDim.x) {
        const int k = o / rout, r = o - k * rout;
        float acc[TV];
#pragma unroll
        for (int v = 0; v < TV; ++v) acc[v] = 0.0f;
        const TW *w = W + (size_t)o * rin;
        const float *src = in + k * ks_in;
        for (int c = 0; c < rin; ++c) {
            const float wv = to_f32(w[c]);
#pragma unroll
            for (int v = 0; v < TV; ++v) acc[v] = fmaf(wv, src[v * in_ld + c * cs_in], acc[v]);
        }
        const int pos = r * rs_out + k * ks_out;
        const float bv = bias ? to_f32(bias[pos]) : 0.0f;
#pragma unroll
        for (int v = 0; v < TV; ++v) out[v * out_ld + pos] = activate(acc[v] + bv, act);
    }
}

template <typename TI, typename TW, typename TO, int TV>
__global__ __launch_bounds__(256) void matmul_generic_kernel(
    const TI *__restrict__ x, const TW *__restrict__ R, const TW *__restrict__ L,
    const TW *__restrict__ bias, TO *__restrict__ y, int64_t batch, int nbR, int r_out, int r_in,
    int nbL, int l_out, int l_in, int order, int act)
{
    extern __shared__ float lds[];
    const int d_in = nbR * r_in;
    const int d_mid = nbR * r_out;
    const int d_out = order == 1 ? d_mid : nbL * l_out;
    const int dA = d_in > d_out ? d_in : d_out;
    float *xs = lds;             // TV x dA : input tile, later the output staging tile
    float *ts = lds + TV * dA;   // TV x d_mid (order 2 only)
    const int64_t v0 = (int64_t)blockIdx.x * TV;

    for (int idx = threadIdx.x; idx < TV * d_in; idx += blockDim.x) {
        const int v = idx / d_in, j = idx - v * d_in;
        xs[v * dA + j] = (v0 + v < batch) ? to_f32(x[(v0 + v) * d_in + j]) : 0.0f;
    }
    __syncthreads();
    if (order == 1) {
        // y[k*r_out + r] = sum_c R_k[r,c] x[k*r_in + c]; result staged in ts then copied out.
        blockdiag_apply<TW, TV>(xs, dA, 1, r_in, ts, d_mid, 1, r_out, R, nbR, r_out, r_in, bias, act);
        __syncthreads();
        for (int idx = threadIdx.x; idx < TV * d_out; idx += blockDim.x) {
            const int v = idx / d_out, j = idx - v * d_out;
            if (v0 + v < batch) y[(v0 + v) * d_out + j] = from_f32<TO>(ts[v * d_mid + j]);
        }
        return;
    }
    // P1 = P_(r_in,d_in): block k reads x[c*nbR + k];  P2 = P_(nbR,d_mid): result to [r*nbR + k].
    blockdiag_apply<TW, TV>(xs, dA, nbR, 1, ts, d_mid, nbR, 1, R, nbR, r_out, r_in, (const TW *)nullptr, 0);
    __syncthreads();
    // L block k' reads ts[k'*l_in + a];  P3 = P_(nbL,d_out): result to [r'*nbL + k'].
    blockdiag_apply<TW, TV>(ts, d_mid, 1, l_in, xs, dA, nbL, 1, L, nbL, l_out, l_in, bias, act);
    __syncthreads();
    for (int idx = threadIdx.x; idx < TV * d_out; idx += blockDim.x) {
        const int v = idx / d_out, j = idx - v * d_out;
        if (v0 + v < batch) y[(v0 + v) * d_out + j] = from_f32<TO>(xs[v * dA + j]);
    }
}

static const size_t kLdsSoftLimit = 64 * 1024;    // no attribute needed below this
static const size_t kLdsHardLimit = 160 * 1024;   // LDS of one gfx950 compute unit

static size_t matmul_generic_lds(int d_in, int d_mid, int d_out, int tv)
{
    int dA = d_in > d_out ? d_in : d_out;
    return (size_t)tv * ((size_t)dA + d_mid) * sizeof(float);
}

bool matmul_generic_fits(int d_in, int d_mid, int d_out)
{
    return matmul_generic_lds(d_in, d_mid, d_out, 1) <= kLdsHardLimit;
}

template <typename TI, typename TW, typename TO>
static int launch_matmul_typed(const void *x, const void *R, const void *L, const void *bias, void *y,
                               int64_t batch, int nbR, int r_out, int r_in, int nbL, int l_out,
                               int l_in, int order, int act, hipStream_t s)
{
    const int d_in = nbR * r_in, d_mid = nbR * r_out, d_out = order == 1 ? d_mid : nbL * l_out;
    int tv = 8;
    while (tv > 1 && matmul_generic_lds(d_in, d_mid, d_out, tv) > kLdsSoftLimit) tv >>= 1;
    const size_t lds = matmul_generic_lds(d_in, d_mid, d_out, tv);
    if (lds > kLdsHardLimit) return fail(MONARCH_ESHAPE, "row of %d+%d floats does not fit in LDS", d_in, d_mid);
    const int64_t grid = (batch + tv - 1) / tv;
    if (grid > 0x7fffffffLL) return fail(MONARCH_ESHAPE, "batch too large");
#define MONARCH_LAUNCH_TV(TVV)                                                                        \
    do {                                                                                              \
        auto kern = matmul_generic_kernel<TI, TW, TO, TVV>;                                           \
        if (lds > kLdsSoftLimit)                                                                      \
            MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern,                                 \
                                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)); \
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, s, (const TI *)x, (const TW *)R, \
                           (const TW *)L, (const TW *)bias, (TO *)y, batch, nbR, r_out, r_in, nbL,    \
                           l_out, l_in, order, act);                                                  \
    } while (0)
    switch (tv) {
    case 8: MONARCH_LAUNCH_TV(8); break;
    case 4: MONARCH_LAUNCH_TV(4); break;
    case 2: MONARCH_LAUNCH_TV(2); break;
    default: MONARCH_LAUNCH_TV(1); break;
    }
#undef MONARCH_LAUNCH_TV
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

int launch_matmul_generic(const void *x, const void *R, const void *L, const void *bias, void *y,
                          int64_t batch, int nbR, int r_out, int r_in, int nbL, int l_out, int l_in,
                          int order, int act, monarch_dtype dt_in, monarch_dtype dt_w,
                          monarch_dtype dt_out, hipStream_t s)
{
    if (batch == 0) return MONARCH_OK;
#define MONARCH_ARGS x, R, L, bias, y, batch, nbR, r_out, r_in, nbL, l_out, l_in, order, act, s
    if (dt_in == MONARCH_F32 && dt_w == MONARCH_F32 && dt_out == MONARCH_F32)
        return launch_matmul_typed<float, float, float>(MONARCH_ARGS);
    if (dt_in == MONARCH_BF16 && dt_w == MONARCH_BF16 && dt_out == MONARCH_BF16)
        return launch_matmul_typed<bf16_t, bf16_t, bf16_t>(MONARCH_ARGS);
    if (dt_in == MONARCH_BF16 && dt_w == MONARCH_BF16 && dt_out == MONARCH_F32)
        return launch_matmul_typed<bf16_t, bf16_t, float>(MONARCH_ARGS);
    if (dt_in == MONARCH_F32 && dt_w == MONARCH_BF16 && dt_out == MONARCH_BF16)
        return launch_matmul_typed<float, bf16_t, bf16_t>(MONARCH_ARGS);
    if (dt_in == MONARCH_F16 && dt_w == MONARCH_F16 && dt_out == MONARCH_F16)
        return launch_matmul_typed<f16_t, f16_t, f16_t>(MONARCH_ARGS);
    if (dt_in == MONARCH_F16 && dt_w == MONARCH_F16 && dt_out == MONARCH_F32)
        return launch_matmul_typed<f16_t, f16_t, float>(MONARCH_ARGS);
    if (dt_in == MONARCH_F32 && dt_w == MONARCH_F16 && dt_out == MONARCH_F16)
        return launch_matmul_typed<float, f16_t, f16_t>(MONARCH_ARGS);
#undef MONARCH_ARGS
    return fail(MONARCH_EDTYPE, "unsupported element type combination");
}

// ------------------------------------------------------------------------------------------
// One factor of the Monarch DFT over rows in global memory
// ------------------------------------------------------------------------------------------

template <typename T>
__device__ __forceinline__ float2 fft_load(const FftPass &p, int64_t row, int pos)
{
    switch (p.load) {
    case LD_C32: return ((const float2 *)p.in)[row * p.N + pos];
    case LD_C32_CONJ: {
        float2 v = ((const float2 *)p.in)[row * p.N + pos];
        return make_float2(v.x, -v.y);
    }
    case LD_C32_CONJ_MULK: {
        float2 v = ((const float2 *)p.in)[row * p.N + pos];
        float2 w = p.kf[(row % p.H) * (int64_t)p.N + pos];
        float2 m = cmul(v, w);
        return make_float2(m.x, -m.y);
    }
    case LD_REAL: {
        if (pos >= p.n_valid) return make_float2(0.0f, 0.0f);
        const int64_t at = row * p.n_valid + pos;
        float v = to_f32(((const T *)p.in)[at]);
        if (p.gate) v *= to_f32(((const T *)p.gate)[at]);
        return make_float2(v, 0.0f);
    }
    default: {  // LD_CPLX
        const int64_t at = (row * p.N + pos) * 2;
        return make_float2(to_f32(((const T *)p.in)[at]), to_f32(((const T *)p.in)[at + 1]));
    }
    }
}

// Natural output index of the last pass: the digits produced so far sit in o with the first
// one most significant; the DFT output wants them least significant first (sub-index reversal).
__device__ __forceinline__ int natural_index(const FftPass &p, int o, int k)
{
    int rev = 0, rem = o;
    for (int q = p.nf - 2; q >= 0; --q) {
        const int fq = p.factors[q];
        const int digit = rem % fq;
        rem /= fq;
        int w = 1;
        for (int r = 0; r < q; ++r) w *= p.factors[r];
        rev += digit * w;
    }
    return k * p.O + rev;
}

template <typename T>
__global__ __launch_bounds__(256) void fft_pass_kernel(const FftPass p)
{
    __shared__ float2 tab[1024];
    const bool use_tab = p.f <= 1024;
    if (use_tab)
        for (int e = threadIdx.x; e < p.f; e += blockDim.x) tab[e] = omega(e, p.f);
    __syncthreads();

    const int64_t total = p.rows * p.N;
    const int fS = p.f * p.S;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t row = e / p.N;
        const int idx = (int)(e - row * p.N);
        const int o = idx / fS;
        const int rem = idx - o * fS;
        const int i = rem / p.S;
        const int a = rem - i * p.S;
        float2 acc = make_float2(0.0f, 0.0f);
        int ph = 0;  // (i*c) mod f
        const int base = o * fS + a;
        for (int c = 0; c < p.f; ++c) {
            const float2 w = use_tab ? tab[ph] : omega(ph, p.f);
            const float2 v = fft_load<T>(p, row, base + c * p.S);
            acc.x = fmaf(w.x, v.x, fmaf(-w.y, v.y, acc.x));
            acc.y = fmaf(w.x, v.y, fmaf(w.y, v.x, acc.y));
            ph += i;
            if (ph >= p.f) ph -= p.f;
        }
        if (p.S > 1) acc = cmul(acc, omega(i * a, fS));   // twiddle diagonal omega_(f*S)^(i*a)
        switch (p.store) {
        case ST_C32: ((float2 *)p.out)[row * p.N + idx] = acc; break;
        case ST_C32_NATURAL: ((float2 *)p.out)[row * p.N + natural_index(p, o, i)] = acc; break;
        case ST_CPLX_CONJ_SCALE: {
            const int64_t at = (row * p.N + natural_index(p, o, i)) * 2;
            ((T *)p.out)[at] = from_f32<T>(acc.x * p.scale);
            ((T *)p.out)[at + 1] = from_f32<T>(-acc.y * p.scale);
            break;
        }
        default: {  // ST_REAL_SCALE_GATE
            const int m = natural_index(p, o, i);
            if (m < p.n_valid) {
                const int64_t at = row * p.n_valid + m;
                float v = acc.x * p.scale;
                if (p.gate) v *= to_f32(((const T *)p.gate)[at]);
                ((T *)p.out)[at] = from_f32<T>(v);
            }
            break;
        }
        }
    }
}

int launch_fft_pass(const FftPass &p, hipStream_t s)
{
    if (p.rows == 0) return MONARCH_OK;
    const int64_t total = p.rows * p.N;
    int64_t grid = (total + 255) / 256;
    if (grid > 1 << 20) grid = 1 << 20;
    if (p.dt == MONARCH_F32)
        hipLaunchKernelGGL(fft_pass_kernel<float>, dim3((unsigned)grid), dim3(256), 0, s, p);
    else if (p.dt == MONARCH_F16)
        hipLaunchKernelGGL(fft_pass_kernel<f16_t>, dim3((unsigned)grid), dim3(256), 0, s, p);
    else
        hipLaunchKernelGGL(fft_pass_kernel<bf16_t>, dim3((unsigned)grid), dim3(256), 0, s, p);
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

}  // namespace monarch
