// Fused gated causal Monarch-FFT convolution, nfft = 2048 = 64 x 32, fp32 I/O and fp32 arithmetic on the matrix
// cores (v_mfma_f32_16x16x4_f32): the fp32 twin of the 16-bit kernel of conv_mfma_2048.hip.
//
// A workgroup (4 waves) takes a work item (channel h, up to 4 pairs of batch rows).  It first turns k[h] into its
// spectrum k_f / N (kept in LDS), then runs, for every pair of rows z = x0 + i x1 (the kernel is real, so the
// convolution of z is conv(x0) + i conv(x1)),
//   gate -> pad -> Monarch DFT -> (.) k_f -> inverse Monarch DFT -> truncate -> gate
// on a 64 x 32 complex tile that ping-pongs between two LDS buffers:
//   the row is the matrix x[c 32 + a]; n = 32 c + a, frequency f = i + 64 k:
//   X : T1[i][a] = sum_c F_64[i][c] x[c][a]       (rows c >= 32 are padding and never multiplied)
//       T1[i][a] *= w_2048^(i a)
//   Y : Z[i][k]  = sum_a T1[i][a] F_32[a][k];     V = conj(Z (.) k_f / N)
//   Y': W[i][a]  = sum_k V[i][k] F_32[k][a];      W[i][a] *= w_2048^(i a)        (the inverse as conj o F o conj,
//   X': o[c][a]  = sum_i F_64[c][i] W[i][a], c < 32 only (truncation)             factors in the opposite order)
//   y0 = Re o, y1 = -Im o, times the output gates.
// Every contraction is a chain of 16x16x4 fp32 MFMAs (a complex product = four real chains); the DFT matrices
// are read from LDS tables of 64 and 32 roots by index arithmetic, the twiddles from a compile-time table of the
// 2048 roots in global memory.  The rows of the next pair and the output gates of this one are requested before
// the stages of the current pair.
//
// Appendix DFT corollary (Monarch form of F_N), Sec. 3.2 Eq. 2 with gating, Thm 3 (padding).
#include "const_roots.h"
#include "kernels.h"

namespace monarch {

namespace c2048f {

typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int N1 = 64, N2 = 32, NFFT = N1 * N2, NHALF = NFFT / 2;
constexpr int P = 34;   // float2 per tile row: rows stay 16-byte aligned, neighbouring rows 4 banks apart

struct RootTable {
    float2 w[NFFT];
};
constexpr RootTable make_roots()
{
    RootTable t{};
    for (int e = 0; e < NFFT; ++e) {
        const croots::CosSin r = croots::unit_root(e, NFFT);
        t.w[e] = float2{(float)r.c, (float)r.s};
    }
    return t;
}
__device__ const RootTable g_roots = make_roots();   // w[e] = exp(+2 pi i e / 2048)
// the twiddles w^(i a) by (i, a): the 16 lanes of a group read 128 contiguous bytes (gathered from the table of roots at
// index i a every lane asked for a cache line of its own, eight times per thread at the head of the kernel)
struct TwiddleTable { float2 v[N1][N2]; };
constexpr TwiddleTable make_twiddles()
{
    TwiddleTable t{};
    for (int i = 0; i < N1; ++i)
        for (int a = 0; a < N2; ++a) {
            const croots::CosSin r = croots::unit_root(i * a, NFFT);
            t.v[i][a].x = (float)r.c;
            t.v[i][a].y = (float)r.s;
        }
    return t;
}
__device__ const TwiddleTable g_twiddles = make_twiddles();

struct Smem {
    float2 tile[2][N1 * P];
    float2 kf[N1 * N2];     // k_f / N at [i][k]
    float2 r64[N1], r32[N2];
};

__device__ __forceinline__ f32x4 mfma(float a, float b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0); }

// One complex k-step: (dr - ds) + i di += (ar + i ai) (br + i bi)
__device__ __forceinline__ void cstep(float2 a, float2 b, f32x4 &dr, f32x4 &ds, f32x4 &di)
{
    dr = mfma(a.x, b.x, dr);
    ds = mfma(a.y, b.y, ds);
    di = mfma(a.x, b.y, di);
    di = mfma(a.y, b.x, di);
}

// Stage X or X': out[j][a] = sum_c F_64[j][c] in[c][a] for the row tile jt (16 rows) and both column tiles of a
// (NA = 2) or one (NA = 1, column tile at0); KSTEPS k-steps of 4 rows of `in`.  Lane (l16, kg) holds, per
// column tile, rows j = 16 jt + 4 kg + r of column a = 16 at + l16.
template <int NA, int KSTEPS>
__device__ __forceinline__ void stage_x(const Smem &sm, const float2 *in, int jt, int at0, int l16, int kg, f32x4 (&zr)[NA], f32x4 (&zi)[NA])
{
    f32x4 dr[NA], ds[NA], di[NA];
#pragma unroll
    for (int t = 0; t < NA; ++t) dr[t] = ds[t] = di[t] = f32x4{0, 0, 0, 0};
    const int j = 16 * jt + l16;
    int e = j * kg;                 // exponent of F_64[j][c], c = c0 + kg
#pragma unroll 4
    for (int s = 0; s < KSTEPS; ++s) {
        const float2 a = sm.r64[e & 63];
        e += 4 * j;
#pragma unroll
        for (int t = 0; t < NA; ++t) cstep(a, in[(4 * s + kg) * P + 16 * (at0 + t) + l16], dr[t], ds[t], di[t]);
    }
#pragma unroll
    for (int t = 0; t < NA; ++t) {
        zr[t] = dr[t] - ds[t];
        zi[t] = di[t];
    }
}

// Stage Y or Y': out[i][k] = sum_a in[i][a] F_32[a][k] for the row tile it and both column tiles of k.
__device__ __forceinline__ void stage_y(const Smem &sm, const float2 *in, int it, int l16, int kg, f32x4 (&zr)[2], f32x4 (&zi)[2])
{
    f32x4 dr[2], ds[2], di[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) dr[t] = ds[t] = di[t] = f32x4{0, 0, 0, 0};
    const float2 *row = in + (16 * it + l16) * P + kg;
#pragma unroll 4
    for (int s = 0; s < N2 / 4; ++s) {
        const float2 a = row[4 * s];
        const int aa = 4 * s + kg;
#pragma unroll
        for (int t = 0; t < 2; ++t) cstep(a, sm.r32[(aa * (16 * t + l16)) & 31], dr[t], ds[t], di[t]);
    }
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        zr[t] = dr[t] - ds[t];
        zi[t] = di[t];
    }
}

// GIN / GOUT: the gates are present.  n, klen: multiples of 4, at most 1024.
template <bool GIN, bool GOUT>
__global__ __launch_bounds__(256, 3) void conv2048_f32_kernel(const float *__restrict__ u, const float *__restrict__ k,
                                                               const float *__restrict__ g_in, const float *__restrict__ g_out,
                                                               float *__restrict__ y, int B, int H, int n, int klen)
{
    __shared__ Smem sm;
    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, kg = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = blockIdx.x % H;
    const int p0 = 4 * (blockIdx.x / H);                // first pair of this work item
    const int npairs = min(4, (B + 1) / 2 - p0);

    if (tid < N1) sm.r64[tid] = g_roots.w[tid * (NFFT / N1)];
    if (tid < N2) sm.r32[tid] = g_roots.w[tid * (NFFT / N2)];

    // this thread's 4 consecutive elements of a row: n0 = 4 tid -> tile position (c, a .. a + 3)
    const int n0 = 4 * tid, c_of = n0 / N2, a_of = n0 % N2;
    const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
    // rows are read once per launch and y written once: streaming accesses
    auto load4 = [&](const float *row, int len) {
        if (n0 >= len) return zero4;
        const uint4 w = load_stream16(row + n0);
        return make_float4(__uint_as_float(w.x), __uint_as_float(w.y), __uint_as_float(w.z), __uint_as_float(w.w));
    };
    auto deposit = [&](float2 *tile, float4 re, float4 im) {
        float4 *dst = reinterpret_cast<float4 *>(tile + c_of * P + a_of);
        dst[0] = make_float4(re.x, im.x, re.y, im.y);
        dst[1] = make_float4(re.z, im.z, re.w, im.w);
    };
    // twiddles of this lane's outputs of stages X and Y': rows i = 16 wave + 4 kg + r, columns a = 16 t + l16
    float2 tw[2][4];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) tw[t][r] = g_twiddles.v[16 * wave + 4 * kg + r][16 * t + l16];

    float2 *tA = sm.tile[0], *tB = sm.tile[1];
    f32x4 zr[2], zi[2];

    // ---- spectrum of the kernel
    {
        const float4 kv = load4(k + (size_t)h * klen, klen);
        if (tid < NHALF / 4) deposit(tA, kv, zero4);   // rows c < 32; the padded rows are never read
    }
    // rows of the first pair, in flight during the kernel's transform
    float4 xa = zero4, xb = zero4, ga = zero4, gb = zero4;
    auto request = [&](int p) {
        const int b0 = 2 * p, b1 = b0 + 1 < B ? b0 + 1 : b0;   // a missing second row reads the first (ignored below)
        const size_t r0 = ((size_t)b0 * H + h) * n, r1 = ((size_t)b1 * H + h) * n;
        xa = load4(u + r0, n);
        xb = load4(u + r1, n);
        if (GIN) {
            ga = load4(g_in + r0, n);
            gb = load4(g_in + r1, n);
        }
    };
    if (npairs > 0) request(p0);
    __syncthreads();
    stage_x<2, NHALF / N2 / 4>(sm, tA, wave, 0, l16, kg, zr, zi);
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) tB[(16 * wave + 4 * kg + r) * P + 16 * t + l16] = cmul(make_float2(zr[t][r], zi[t][r]), tw[t][r]);
    __syncthreads();
    stage_y(sm, tB, wave, l16, kg, zr, zi);
    {
        const float inv = 1.0f / (float)NFFT;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                sm.kf[(16 * wave + 4 * kg + r) * N2 + 16 * t + l16] = make_float2(zr[t][r] * inv, zi[t][r] * inv);
    }

    for (int q = 0; q < npairs; ++q) {
        const int p = p0 + q, b0 = 2 * p;
        const bool two = b0 + 1 < B;
        const size_t r0 = ((size_t)b0 * H + h) * n, r1 = r0 + (size_t)H * n;
        // ---- gate, pad, deposit (tile A is free: the previous pair's store has passed its barrier)
        {
            float4 re = xa, im = two ? xb : zero4;
            if (GIN) {
                re = make_float4(re.x * ga.x, re.y * ga.y, re.z * ga.z, re.w * ga.w);
                im = make_float4(im.x * gb.x, im.y * gb.y, im.z * gb.z, im.w * gb.w);
            }
            if (tid < NHALF / 4) deposit(tA, re, im);
        }
        __syncthreads();   // (also: k_f complete, first pair)
        if (q + 1 < npairs) request(p + 1);
        float4 oa = zero4, ob = zero4;
        if (GOUT) {
            oa = load4(g_out + r0, n);
            ob = load4(g_out + (two ? r1 : r0), n);
        }

        stage_x<2, NHALF / N2 / 4>(sm, tA, wave, 0, l16, kg, zr, zi);
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) tB[(16 * wave + 4 * kg + r) * P + 16 * t + l16] = cmul(make_float2(zr[t][r], zi[t][r]), tw[t][r]);
        __syncthreads();
        stage_y(sm, tB, wave, l16, kg, zr, zi);
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int i = 16 * wave + 4 * kg + r, kk = 16 * t + l16;
                const float2 m = cmul(make_float2(zr[t][r], zi[t][r]), sm.kf[i * N2 + kk]);
                tA[i * P + kk] = make_float2(m.x, -m.y);
            }
        __syncthreads();
        stage_y(sm, tA, wave, l16, kg, zr, zi);
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) tB[(16 * wave + 4 * kg + r) * P + 16 * t + l16] = cmul(make_float2(zr[t][r], zi[t][r]), tw[t][r]);
        __syncthreads();
        {
            // rows c < 32 only: row tile wave / 2, column tile wave % 2; the result goes through tile A so that
            // the stores are 16 bytes per lane like the loads
            f32x4 orr[1], oi[1];
            stage_x<1, N1 / 4>(sm, tB, wave >> 1, wave & 1, l16, kg, orr, oi);
#pragma unroll
            for (int r = 0; r < 4; ++r)
                tA[(16 * (wave >> 1) + 4 * kg + r) * P + 16 * (wave & 1) + l16] = make_float2(orr[0][r], -oi[0][r]);
        }
        __syncthreads();
        if (n0 < n) {
            const float4 *src = reinterpret_cast<const float4 *>(tA + c_of * P + a_of);
            const float4 v0 = src[0], v1 = src[1];   // (y0, y1) of four neighbouring positions
            float4 ya = make_float4(v0.x, v0.z, v1.x, v1.z), yb = make_float4(v0.y, v0.w, v1.y, v1.w);
            if (GOUT) {
                ya = make_float4(ya.x * oa.x, ya.y * oa.y, ya.z * oa.z, ya.w * oa.w);
                yb = make_float4(yb.x * ob.x, yb.y * ob.y, yb.z * ob.z, yb.w * ob.w);
            }
            store_stream16(y + r0 + n0, make_uint4(__float_as_uint(ya.x), __float_as_uint(ya.y), __float_as_uint(ya.z), __float_as_uint(ya.w)));
            if (two) store_stream16(y + r1 + n0, make_uint4(__float_as_uint(yb.x), __float_as_uint(yb.y), __float_as_uint(yb.z), __float_as_uint(yb.w)));
        }
        __syncthreads();
    }
}

}  // namespace c2048f

bool conv_f32_2048_supported(int n, int klen, const int *factors, int nf, monarch_dtype dt)
{
    return dt == MONARCH_F32 && nf == 2 && factors[0] == c2048f::N1 && factors[1] == c2048f::N2 && n >= 1 && klen >= 1 &&
           n <= c2048f::NHALF && klen <= c2048f::NHALF && n % 4 == 0 && klen % 4 == 0;
}

int launch_conv_f32_2048(const void *u, const void *k, const void *g_in, const void *g_out, void *y,
                         int B, int H, int n, int klen, hipStream_t s)
{
    // One workgroup per (channel, group of 4 batch pairs); with B <= 8 that is one per channel.
    const int64_t groups = ((B + 1) / 2 + 3) / 4;
    const int64_t grid = (int64_t)H * groups;
    if (grid > 0x7fffffffLL) return fail(MONARCH_ESHAPE, "B*H too large for one launch");
#define MONARCH_LAUNCH_C2048F(GINV, GOUTV)                                                                       \
    hipLaunchKernelGGL((c2048f::conv2048_f32_kernel<GINV, GOUTV>), dim3((unsigned)grid), dim3(256), 0, s,        \
                       (const float *)u, (const float *)k, (const float *)g_in, (const float *)g_out, (float *)y, B, H, n, klen)
    switch ((g_in ? 2 : 0) | (g_out ? 1 : 0)) {
    case 3: MONARCH_LAUNCH_C2048F(true, true); break;
    case 2: MONARCH_LAUNCH_C2048F(true, false); break;
    case 1: MONARCH_LAUNCH_C2048F(false, true); break;
    default: MONARCH_LAUNCH_C2048F(false, false); break;
    }
#undef MONARCH_LAUNCH_C2048F
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

}  // namespace monarch
