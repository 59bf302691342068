// Fused gated causal Monarch-FFT convolution, nfft = 2048 = 64 x 32, bf16 I/O, fp32 accumulate.
//
// One workgroup (4 waves) owns one channel h.  It first turns k[h] into its spectrum k_f
// (kept in LDS), then every wave takes PAIRS of batch rows of that channel and runs the whole
// chain  pad -> Monarch DFT -> (.) k_f -> inverse Monarch DFT -> truncate -> gate  in registers:
//
//   * two real rows ride as one complex row z = x0 + i x1 (the kernel is real, so the
//     convolution of z is conv(x0) + i conv(x1)): half the transforms;
//   * the row is the N1 x N2 = 64 x 32 matrix x[c*32 + a]; the Monarch factors are
//     R = I (x) F_64 (contract c), twiddle w_2048^(i a), L = F_32 blocks (contract a);
//     the zero-padded half (c >= 32) is never multiplied and only outputs c < 32 are formed;
//   * every factor is a bf16 MFMA (32x32x16) with the constant DFT matrix as one operand and
//     the previous stage's accumulators, re-rounded to bf16, as the other.  An accumulator
//     tile (rows in registers, columns on lanes) is a valid B operand (contract its rows,
//     keep columns on lanes) and equally a valid A operand (contract its rows, its lane index
//     becomes the new row index), so no stage needs a transpose: the permutations P of
//     M = P L P R P never exist as data movement, not even in LDS;
//   * twiddles, the spectrum product and the gates are fp32 on the accumulators.
//
// Appendix DFT corollary (Monarch form of F_N), Sec. 3.2 Eq. 2 with gating, Thm 3 (padding).
#include "kernels.h"

namespace monarch {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

namespace c2048 {

constexpr int N1 = 64, N2 = 32, NFFT = 2048, NHALF = 1024;
constexpr int TW_LD = 34;   // padded row length (complex) of the twiddle table

struct Smem {
    float2 tw[N1][TW_LD];          // w_2048^(i*a), i < 64, a < 32
    float4 kf_re[2][4][64];        // k_f / NFFT in accumulator layout [tile][quad][lane]
    float4 kf_im[2][4][64];
    uint32_t stage[4][NHALF];      // per wave: (re bf16 | im bf16 << 16) at [c*32 + a]
};

union Pack8 {
    bf16x8 v;
    uint32_t d[4];
    uint4 q;
};

struct COp { bf16x8 r, i, ni; };   // constant complex operand: real, imag, -imag

// cos/sin of 2*pi*e/N through the hardware units (argument in revolutions, 0 <= e < N).
__device__ __forceinline__ float2 hw_omega(int e, int N)
{
    const float x = (float)e / (float)N;
    return make_float2(__builtin_amdgcn_cosf(x), __builtin_amdgcn_sinf(x));
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    bf16x2 p = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, p);
}

__device__ __forceinline__ float bf16_lo(uint32_t d) { return __uint_as_float(d << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t d) { return __uint_as_float(d & 0xffff0000u); }

// Contraction index carried by operand slot (kstep s, lane group g, element j) when the operand
// is made from accumulator registers 8s..8s+7: the accumulator row 8*(r/4) + 4*g + r%4.
__device__ __forceinline__ int slot_index(int s, int g, int j) { return 16 * s + 8 * (j >> 2) + 4 * g + (j & 3); }

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16x8 pack_acc(const f32x16 &v, int s)
{
    Pack8 p;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) p.d[jj] = pack_bf16(v[8 * s + 2 * jj], v[8 * s + 2 * jj + 1]);
    return p.v;
}

// 8 consecutive bf16 of a row (chunk ch), zero past the end of the row.
__device__ __forceinline__ uint4 load_chunk(const bf16_t *row, int ch, int len)
{
    if (ch * 8 < len) return *reinterpret_cast<const uint4 *>(row + ch * 8);
    return make_uint4(0u, 0u, 0u, 0u);
}

__device__ __forceinline__ uint32_t mul_pack(uint32_t a, uint32_t b)
{
    return pack_bf16(bf16_lo(a) * bf16_lo(b), bf16_hi(a) * bf16_hi(b));
}

// Writes rows x0 (real part) and x1 (imaginary part, may be absent) of one pair into the
// wave's staging tile, gated by g0/g1 when given.  Lane handles chunks lane and lane+64.
__device__ __forceinline__ void stage_pair(uint32_t *stage, int lane, const bf16_t *x0, const bf16_t *x1,
                                           const bf16_t *g0, const bf16_t *g1, int len)
{
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const int ch = lane + 64 * half;
        uint4 re = load_chunk(x0, ch, len);
        uint4 im = x1 ? load_chunk(x1, ch, len) : make_uint4(0u, 0u, 0u, 0u);
        if (g0) {
            const uint4 ga = load_chunk(g0, ch, len);
            re.x = mul_pack(re.x, ga.x); re.y = mul_pack(re.y, ga.y);
            re.z = mul_pack(re.z, ga.z); re.w = mul_pack(re.w, ga.w);
            if (x1) {
                const uint4 gb = load_chunk(g1, ch, len);
                im.x = mul_pack(im.x, gb.x); im.y = mul_pack(im.y, gb.y);
                im.z = mul_pack(im.z, gb.z); im.w = mul_pack(im.w, gb.w);
            }
        }
        const uint32_t r[4] = {re.x, re.y, re.z, re.w}, m[4] = {im.x, im.y, im.z, im.w};
        uint4 o0, o1;
        // element e: (re_e | im_e << 16)
        o0.x = __builtin_amdgcn_perm(m[0], r[0], 0x05040100u); o0.y = __builtin_amdgcn_perm(m[0], r[0], 0x07060302u);
        o0.z = __builtin_amdgcn_perm(m[1], r[1], 0x05040100u); o0.w = __builtin_amdgcn_perm(m[1], r[1], 0x07060302u);
        o1.x = __builtin_amdgcn_perm(m[2], r[2], 0x05040100u); o1.y = __builtin_amdgcn_perm(m[2], r[2], 0x07060302u);
        o1.z = __builtin_amdgcn_perm(m[3], r[3], 0x05040100u); o1.w = __builtin_amdgcn_perm(m[3], r[3], 0x07060302u);
        uint4 *dst = reinterpret_cast<uint4 *>(stage + ch * 8);
        dst[0] = o0;
        dst[1] = o1;
    }
}

// A operands of the first factor: lane (a = lane%32, g) holds x[c][a] for the 8 c of each kstep.
__device__ __forceinline__ void read_stage_operands(const uint32_t *stage, int il, int g, bf16x8 (&xr)[2], bf16x8 (&xi)[2])
{
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        Pack8 pr, pi;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const uint32_t d0 = stage[slot_index(s, g, 2 * jj) * 32 + il];
            const uint32_t d1 = stage[slot_index(s, g, 2 * jj + 1) * 32 + il];
            pr.d[jj] = __builtin_amdgcn_perm(d1, d0, 0x05040100u);
            pi.d[jj] = __builtin_amdgcn_perm(d1, d0, 0x07060302u);
        }
        xr[s] = pr.v;
        xi[s] = pi.v;
    }
}

// Forward transform of tile t (spectrum columns i = 32t + lane%32):
//   Z1[a,i] = sum_c x[c,a] F64[c,i];  Z1 *= w_2048^(i a);  Z2[k,i] = sum_a F32[k,a] Z1[a,i].
// Result rows k sit in registers (accumulator layout), columns i on lanes.
template <bool HAS_IM>
__device__ __forceinline__ void forward_tile(const Smem &sm, int t, int il, int g, const bf16x8 (&xr)[2],
                                             const bf16x8 (&xi)[2], const COp (&Fb)[2], const COp (&G)[2],
                                             f32x16 &z2r, f32x16 &z2i)
{
    f32x16 zr = {0}, zi = {0};
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        zr = mfma(xr[s], Fb[s].r, zr);
        zi = mfma(xr[s], Fb[s].i, zi);
        if (HAS_IM) {
            zr = mfma(xi[s], Fb[s].ni, zr);
            zi = mfma(xi[s], Fb[s].r, zi);
        }
    }
    // twiddle: rows a = 8q + 4g + rr in registers, column i on the lane
    const float2 *trow = sm.tw[32 * t + il];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const float4 t01 = *reinterpret_cast<const float4 *>(trow + 8 * q + 4 * g);
        const float4 t23 = *reinterpret_cast<const float4 *>(trow + 8 * q + 4 * g + 2);
        const float tr[4] = {t01.x, t01.z, t23.x, t23.z}, ti[4] = {t01.y, t01.w, t23.y, t23.w};
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
            const float a = zr[4 * q + rr], b = zi[4 * q + rr];
            zr[4 * q + rr] = a * tr[rr] - b * ti[rr];
            zi[4 * q + rr] = a * ti[rr] + b * tr[rr];
        }
    }
    z2r = (f32x16){0};
    z2i = (f32x16){0};
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const bf16x8 br = pack_acc(zr, s), bi = pack_acc(zi, s);
        z2r = mfma(G[s].r, br, z2r);
        z2r = mfma(G[s].ni, bi, z2r);
        z2i = mfma(G[s].i, br, z2i);
        z2i = mfma(G[s].r, bi, z2i);
    }
}

__global__ __launch_bounds__(256) void conv2048_bf16_kernel(
    const bf16_t *__restrict__ u, const bf16_t *__restrict__ k, const bf16_t *__restrict__ g_in,
    const bf16_t *__restrict__ g_out, bf16_t *__restrict__ y, int B, int H, int n, int klen)
{
    __shared__ Smem sm;
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, il = lane & 31, g = lane >> 5;
    const int h = blockIdx.x;
    uint32_t *stage = sm.stage[wave];

    // twiddle table w_2048^(i*a); i*a <= 63*31 < 2048
    for (int idx = tid; idx < N1 * N2; idx += 256) {
        const int i = idx >> 5, a = idx & 31;
        sm.tw[i][a] = hw_omega(i * a, NFFT);
    }

    // per-lane constant operands
    COp Fb[2][2];   // F64[c][i], c = slot, i = 32t + il         (first factor, B operand; last factor t=0, A operand)
    COp Hb[2];      // F64[il][32 + slot]                        (last factor, A operand, contraction rows 32..63)
    COp G[2];       // F32[il][slot]                             (second factor A operand / third factor B operand)
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        Pack8 fr[2], fi[2], fn[2], hr, hi, hn, gr, gi, gn;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            float2 w[2][2], wh[2], wg[2];
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int cm = slot_index(s, g, 2 * jj + e);
                w[0][e] = hw_omega((cm * il) & 63, 64);
                w[1][e] = hw_omega((cm * (32 + il)) & 63, 64);
                wh[e] = hw_omega((il * (32 + cm)) & 63, 64);
                wg[e] = hw_omega((il * cm) & 31, 32);
            }
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                fr[t].d[jj] = pack_bf16(w[t][0].x, w[t][1].x);
                fi[t].d[jj] = pack_bf16(w[t][0].y, w[t][1].y);
                fn[t].d[jj] = pack_bf16(-w[t][0].y, -w[t][1].y);
            }
            hr.d[jj] = pack_bf16(wh[0].x, wh[1].x);
            hi.d[jj] = pack_bf16(wh[0].y, wh[1].y);
            hn.d[jj] = pack_bf16(-wh[0].y, -wh[1].y);
            gr.d[jj] = pack_bf16(wg[0].x, wg[1].x);
            gi.d[jj] = pack_bf16(wg[0].y, wg[1].y);
            gn.d[jj] = pack_bf16(-wg[0].y, -wg[1].y);
        }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            Fb[t][s].r = fr[t].v; Fb[t][s].i = fi[t].v; Fb[t][s].ni = fn[t].v;
        }
        Hb[s].r = hr.v; Hb[s].i = hi.v; Hb[s].ni = hn.v;
        G[s].r = gr.v; G[s].i = gi.v; G[s].ni = gn.v;
    }
    __syncthreads();   // twiddle table complete

    // spectrum of the kernel: waves 0 and 1 take one tile of spectrum columns each
    if (wave < 2) {
        stage_pair(stage, lane, k + (size_t)h * klen, nullptr, nullptr, nullptr, klen);
        __builtin_amdgcn_wave_barrier();
        bf16x8 xr[2], xi[2];
        read_stage_operands(stage, il, g, xr, xi);
        f32x16 zr, zi;
        if (wave == 0) forward_tile<false>(sm, 0, il, g, xr, xi, Fb[0], G, zr, zi);
        else forward_tile<false>(sm, 1, il, g, xr, xi, Fb[1], G, zr, zi);
        const float inv = 1.0f / (float)NFFT;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            sm.kf_re[wave][q][lane] = make_float4(zr[4 * q] * inv, zr[4 * q + 1] * inv, zr[4 * q + 2] * inv, zr[4 * q + 3] * inv);
            sm.kf_im[wave][q][lane] = make_float4(zi[4 * q] * inv, zi[4 * q + 1] * inv, zi[4 * q + 2] * inv, zi[4 * q + 3] * inv);
        }
    }
    __syncthreads();   // k_f complete; staging tiles of waves 0/1 free again

    const int npairs = (B + 1) >> 1;
    for (int p = wave; p < npairs; p += 4) {
        const int b0 = 2 * p;
        const bool two = b0 + 1 < B;
        const size_t row0 = ((size_t)b0 * H + h) * n, row1 = ((size_t)(b0 + 1) * H + h) * n;
        __builtin_amdgcn_wave_barrier();
        stage_pair(stage, lane, u + row0, two ? u + row1 : nullptr, g_in ? g_in + row0 : nullptr,
                   g_in ? g_in + row1 : nullptr, n);
        __builtin_amdgcn_wave_barrier();
        bf16x8 xr[2], xi[2];
        read_stage_operands(stage, il, g, xr, xi);

        // forward transform and spectrum product, then third factor, per tile of columns i
        bf16x8 wr_op[2][2], wi_op[2][2];   // [tile][kstep] operands of the last factor
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            f32x16 zr, zi;
            forward_tile<true>(sm, t, il, g, xr, xi, Fb[t], G, zr, zi);
            // Y = Z2 (.) k_f   (rows k in registers, column i on the lane)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 kr = sm.kf_re[t][q][lane], ki = sm.kf_im[t][q][lane];
                const float kre[4] = {kr.x, kr.y, kr.z, kr.w}, kim[4] = {ki.x, ki.y, ki.z, ki.w};
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    const float a = zr[4 * q + rr], b = zi[4 * q + rr];
                    zr[4 * q + rr] = a * kre[rr] - b * kim[rr];
                    zi[4 * q + rr] = a * kim[rr] + b * kre[rr];
                }
            }
            // third factor: W[i,a] = sum_k Y[i,k] conj(F32)[k,a]; Y's lane index i becomes the row index
            f32x16 wr = {0}, wi = {0};
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const bf16x8 ar = pack_acc(zr, s), ai = pack_acc(zi, s);
                wr = mfma(ar, G[s].r, wr);
                wr = mfma(ai, G[s].i, wr);
                wi = mfma(ar, G[s].ni, wi);
                wi = mfma(ai, G[s].r, wi);
            }
            // conjugate twiddle: rows i = 32t + 8q + 4g + rr in registers, column a on the lane
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int i = 32 * t + 8 * (r >> 2) + 4 * g + (r & 3);
                const float2 w = sm.tw[i][il];
                const float a = wr[r], b = wi[r];
                wr[r] = a * w.x + b * w.y;
                wi[r] = b * w.x - a * w.y;
            }
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                wr_op[t][s] = pack_acc(wr, s);
                wi_op[t][s] = pack_acc(wi, s);
            }
        }
        // last factor: y[c,a] = sum_i conj(F64)[c,i] W[i,a], c < 32 only (truncation to n)
        f32x16 yr = {0}, yi = {0};
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            yr = mfma(Fb[0][s].r, wr_op[0][s], yr);
            yr = mfma(Fb[0][s].i, wi_op[0][s], yr);
            yi = mfma(Fb[0][s].r, wi_op[0][s], yi);
            yi = mfma(Fb[0][s].ni, wr_op[0][s], yi);
            yr = mfma(Hb[s].r, wr_op[1][s], yr);
            yr = mfma(Hb[s].i, wi_op[1][s], yr);
            yi = mfma(Hb[s].r, wi_op[1][s], yi);
            yi = mfma(Hb[s].ni, wr_op[1][s], yi);
        }
        // rows c = 8q + 4g + rr, column a = il  ->  staging tile, then coalesced gated stores
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int c = 8 * (r >> 2) + 4 * g + (r & 3);
            stage[c * 32 + il] = pack_bf16(yr[r], yi[r]);
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int ch = lane + 64 * half;
            if (ch * 8 >= n) continue;
            const uint4 *src = reinterpret_cast<const uint4 *>(stage + ch * 8);
            const uint4 s0 = src[0], s1 = src[1];
            const uint32_t d[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
            uint32_t re[4], im[4];
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                re[jj] = __builtin_amdgcn_perm(d[2 * jj + 1], d[2 * jj], 0x05040100u);
                im[jj] = __builtin_amdgcn_perm(d[2 * jj + 1], d[2 * jj], 0x07060302u);
            }
            if (g_out) {
                const uint4 ga = load_chunk(g_out + row0, ch, n);
                re[0] = mul_pack(re[0], ga.x); re[1] = mul_pack(re[1], ga.y);
                re[2] = mul_pack(re[2], ga.z); re[3] = mul_pack(re[3], ga.w);
                if (two) {
                    const uint4 gb = load_chunk(g_out + row1, ch, n);
                    im[0] = mul_pack(im[0], gb.x); im[1] = mul_pack(im[1], gb.y);
                    im[2] = mul_pack(im[2], gb.z); im[3] = mul_pack(im[3], gb.w);
                }
            }
            *reinterpret_cast<uint4 *>(y + row0 + ch * 8) = make_uint4(re[0], re[1], re[2], re[3]);
            if (two) *reinterpret_cast<uint4 *>(y + row1 + ch * 8) = make_uint4(im[0], im[1], im[2], im[3]);
        }
    }
}

}  // namespace c2048

bool conv_mfma_2048_supported(int n, int klen, const int *factors, int nf, monarch_dtype dt)
{
    return dt == MONARCH_BF16 && nf == 2 && factors[0] == 64 && factors[1] == 32 && n <= 1024 && klen <= 1024 &&
           n % 8 == 0 && klen % 8 == 0;
}

int launch_conv_mfma_2048(const void *u, const void *k, const void *g_in, const void *g_out, void *y,
                          int B, int H, int n, int klen, hipStream_t s)
{
    hipLaunchKernelGGL(c2048::conv2048_bf16_kernel, dim3((unsigned)H), dim3(256), 0, s, (const bf16_t *)u,
                       (const bf16_t *)k, (const bf16_t *)g_in, (const bf16_t *)g_out, (bf16_t *)y, B, H, n, klen);
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

}  // namespace monarch
