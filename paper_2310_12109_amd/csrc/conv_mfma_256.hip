// Fused gated causal convolution for nfft = 256 = 16 x 16, n <= 128, klen <= 256, bf16 I/O
// (Sec. 3.1 Monarch DFT, Sec. 3.2 Eq. 2 / Thm 3 convolution, gates fused).
//
// One wave per (channel, group of four row pairs); two real rows of a channel are transformed as one
// complex row.  A 16 x 16 complex tile is one MFMA accumulator pair (re, im), and every stage is a
// complex 16 x 16 product done as two real MFMAs with the contraction index stacked (re rows, im rows):
//   S1  Tt[a, i]  = sum_c x[c, a] F[i, c]          data as A operand (loaded straight from global)
//       Tt       *= omega_256^(i a)                fp32, on the accumulators
//   S2  U[k, i]   = sum_a F[k, a] Tt[a, i]         accumulators re-enter as B operand (rows = contraction)
//       P         = U o k_f                        k_f made by the same two stages, kept in registers
//   S3  Vt[i, a'] = sum_k P[k, i] conj F[a', k]    accumulators re-enter as A operand (lane = row)
//       Vt       *= conj omega_256^(i a')
//   S4  Y[c', a'] = sum_i conj F[c', i] Vt[i, a']  accumulators re-enter as B operand
// so no value ever passes through LDS.  The input x[c, a] = x[16 c + a] has c < 8 (zero padding), so
// S1 is a K = 16 MFMA; of Y only c' < 8 is stored, and the rows of the last constant operand are
// ordered so that every lane group holds two of those rows.
#include "kernels.h"

namespace monarch {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

namespace c256 {

constexpr int PAIRS = 4;   // row pairs per wave

__device__ __forceinline__ uint32_t pack2(float lo, float hi)
{
    bf16x2 v = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ f32x4 mfma32(u32x4 a, u32x4 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mfma16(u32x2 a, u32x2 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, a), __builtin_bit_cast(s16x4, b), c, 0, 0, 0);
}
__device__ __forceinline__ float bf(const bf16_t *p, int64_t at, bool ok)
{
    const float v = (float)p[ok ? at : 0];
    return ok ? v : 0.0f;
}
// accumulator tiles (re, im) -> stacked-contraction operand: slots 0..3 = re rows, 4..7 = im rows
__device__ __forceinline__ u32x4 stack(const f32x4 &re, const f32x4 &im)
{
    return u32x4{pack2(re[0], re[1]), pack2(re[2], re[3]), pack2(im[0], im[1]), pack2(im[2], im[3])};
}

// F16 entries of one matrix row for four consecutive columns, as bf16 pairs
struct Quad {
    u32x2 re, im, nim;
};
__device__ __forceinline__ Quad dft_quad(int row, int col0)
{
    // hardware sine / cosine of an exact fraction of a turn (error ~1e-6, far below bf16 resolution);
    // the library sincospif would cost more instructions here than the five transforms of the wave
    float c[4], s[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float turn = (float)((row * (col0 + e)) & 15) * 0.0625f;
        s[e] = __builtin_amdgcn_sinf(turn);
        c[e] = __builtin_amdgcn_cosf(turn);
    }
    Quad q;
    q.re = u32x2{pack2(c[0], c[1]), pack2(c[2], c[3])};
    q.im = u32x2{pack2(s[0], s[1]), pack2(s[2], s[3])};
    q.nim = q.im ^ 0x80008000u;
    return q;
}
__device__ __forceinline__ u32x4 cat(u32x2 a, u32x2 b) { return u32x4{a[0], a[1], b[0], b[1]}; }

// VEC (n a multiple of 8): the rows of the wave's four pairs travel between global memory and the wave's own LDS
// staging area 16 bytes per lane (8 rows of 256 bytes per stream = two accesses of the wave), and the 2-byte
// operand gathers and result scatters of the layouts below happen in LDS; otherwise every element is a 2-byte
// global access of its own.
template <bool GIN, bool GOUT, bool VEC>
__global__ __launch_bounds__(256) void conv256_bf16_kernel(const bf16_t *__restrict__ u, const bf16_t *__restrict__ k,
                                                           const bf16_t *__restrict__ g_in, const bf16_t *__restrict__ g_out,
                                                           bf16_t *__restrict__ y, int B, int H, int n, int klen)
{
    const int lane = threadIdx.x & 63, l16 = lane & 15, kg = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int h = blockIdx.x;
    const int npairs = (B + 1) / 2;
    const int p0 = (blockIdx.y * 4 + wave) * PAIRS;
    if (p0 >= npairs) return;

    // ---- requests first: the kernel row and this wave's inputs
    float kv[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int t = (4 * kg + e) * 16 + l16;
        kv[e] = bf(k, (int64_t)h * klen + t, t < klen);
    }
    // S1 data operand: lane (a = l16, kg): lane groups 0, 1 carry the first row of the pair (re) at
    // c = 4 kg + e, groups 2, 3 the second (im) at c = 4 (kg - 2) + e
    const int member = kg >> 1, cb = 4 * (kg & 1);
    float xin[PAIRS][4], gout[PAIRS][2][2];
    // VEC: [stream: u, g_in, g_out / y][row 2 p + member][128] per wave, rows of 256 bytes
    __shared__ __attribute__((aligned(16))) uint16_t staging[VEC ? 4 : 1][3][VEC ? 2 * PAIRS * 128 : 8];
    uint16_t (*st)[2 * PAIRS * 128] = reinterpret_cast<uint16_t (*)[2 * PAIRS * 128]>(&staging[VEC ? wave : 0][0][0]);
    if constexpr (VEC) {
        uint4 ld[3][PAIRS / 2];
#pragma unroll
        for (int it = 0; it < PAIRS / 2; ++it) {
            const int r = 4 * it + (lane >> 4), b = 2 * (p0 + (r >> 1)) + (r & 1), e0 = 8 * l16;
            const bool ok = b < B && e0 < n;
            const int64_t at = ok ? ((int64_t)b * H + h) * n + e0 : 0;
            const uint4 zero4 = make_uint4(0u, 0u, 0u, 0u);
            ld[0][it] = load_stream16(u + at);   // rows touched once per launch: streaming accesses
            if (GIN) ld[1][it] = load_stream16(g_in + at);
            if (GOUT) ld[2][it] = load_stream16(g_out + at);
            if (!ok) ld[0][it] = zero4;   // (the gates of a missing element meet a zero or are never used)
        }
#pragma unroll
        for (int it = 0; it < PAIRS / 2; ++it) {
            const int off = (4 * it + (lane >> 4)) * 128 + 8 * l16;
            *reinterpret_cast<uint4 *>(&st[0][off]) = ld[0][it];
            if (GIN) *reinterpret_cast<uint4 *>(&st[1][off]) = ld[1][it];
            if (GOUT) *reinterpret_cast<uint4 *>(&st[2][off]) = ld[2][it];
        }
        __builtin_amdgcn_wave_barrier();
        auto f32_of = [](uint16_t h) { return __uint_as_float((uint32_t)h << 16); };
#pragma unroll
        for (int p = 0; p < PAIRS; ++p) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int at = (2 * p + member) * 128 + (cb + e) * 16 + l16;
                float v = f32_of(st[0][at]);
                if (GIN) v *= f32_of(st[1][at]);
                xin[p][e] = v;
            }
#pragma unroll
            for (int m = 0; m < 2; ++m)
#pragma unroll
                for (int r = 0; r < 2; ++r) gout[p][m][r] = GOUT ? f32_of(st[2][(2 * p + m) * 128 + (2 * kg + r) * 16 + l16]) : 1.0f;
        }
    }
#pragma unroll
    for (int p = 0; p < PAIRS && !VEC; ++p) {
        const int b = 2 * (p0 + p) + member;
        const int64_t row = ((int64_t)b * H + h) * n;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int t = (cb + e) * 16 + l16;
            const bool ok = b < B && t < n;
            float v = bf(u, row + t, ok);
            if (GIN) v *= bf(g_in, row + t, ok);
            xin[p][e] = v;
        }
        // outputs this lane stores: rows c' = 2 kg + r (r = 0, 1), column a' = l16, both members
#pragma unroll
        for (int m = 0; m < 2; ++m)
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                const int bb = 2 * (p0 + p) + m, t = (2 * kg + r) * 16 + l16;
                gout[p][m][r] = GOUT ? bf(g_out, ((int64_t)bb * H + h) * n + t, bb < B && t < n) : 1.0f;
            }
    }

    // ---- constants: F16 rows in the operand layouts of the four stages, twiddles
    const Quad q = dft_quad(l16, 4 * kg);
    const u32x4 opA = cat(q.re, q.nim), opB = cat(q.im, q.re);   // S2 (A operand) and S1 of the kernel (B operand)
    const u32x4 opC = cat(q.re, q.im), opD = cat(q.nim, q.re);   // S3 (B operand)
    const int crow = (l16 & 2) ? 8 + 2 * (l16 >> 2) + (l16 & 1) : 2 * (l16 >> 2) + (l16 & 1);   // S4: tile row l16 computes c'
    const Quad q4 = dft_quad(crow, 4 * kg);
    const u32x4 opC4 = cat(q4.re, q4.im), opD4 = cat(q4.nim, q4.re);
    const Quad q1 = dft_quad(l16, cb);   // S1 of the data: K = 16, slots = (member, c)
    const u32x2 s1re = member ? q1.nim : q1.re, s1im = member ? q1.re : q1.im;
    float2 tw[4];   // omega_256^((4 kg + r) l16)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const float turn = (float)(((4 * kg + r) * l16) & 255) * (1.0f / 256.0f);
        tw[r] = make_float2(__builtin_amdgcn_cosf(turn), __builtin_amdgcn_sinf(turn));
    }
    const f32x4 zero = {0, 0, 0, 0};

    // ---- k_f = F k' / 256 in the accumulator layout of U: lane (i = l16), rows k = 4 kg + r
    f32x4 kfr, kfi;
    {
        const u32x4 ka = {pack2(kv[0], kv[1]), pack2(kv[2], kv[3]), 0u, 0u};   // real input: im slots empty
        f32x4 tr = mfma32(ka, opA, zero), ti = mfma32(ka, opB, zero);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float a = tr[r], b = ti[r];
            tr[r] = a * tw[r].x - b * tw[r].y;
            ti[r] = a * tw[r].y + b * tw[r].x;
        }
        const u32x4 tb = stack(tr, ti);
        kfr = mfma32(opA, tb, zero);
        kfi = mfma32(opB, tb, zero);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            kfr[r] *= 1.0f / 256.0f;
            kfi[r] *= 1.0f / 256.0f;
        }
    }

#pragma unroll
    for (int p = 0; p < PAIRS; ++p) {   // (pairs past the end compute on zeros and store nothing: one block of code, so
                                        // that the independent chains of the four pairs can be interleaved)
        const u32x2 xa = {pack2(xin[p][0], xin[p][1]), pack2(xin[p][2], xin[p][3])};
        f32x4 tr = mfma16(xa, s1re, zero), ti = mfma16(xa, s1im, zero);           // S1
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float a = tr[r], b = ti[r];
            tr[r] = a * tw[r].x - b * tw[r].y;
            ti[r] = a * tw[r].y + b * tw[r].x;
        }
        const u32x4 tb = stack(tr, ti);
        f32x4 ur = mfma32(opA, tb, zero), ui = mfma32(opB, tb, zero);              // S2
#pragma unroll
        for (int r = 0; r < 4; ++r) {                                              // spectrum product
            const float a = ur[r], b = ui[r];
            ur[r] = a * kfr[r] - b * kfi[r];
            ui[r] = a * kfi[r] + b * kfr[r];
        }
        const u32x4 pa = stack(ur, ui);
        f32x4 vr = mfma32(pa, opC, zero), vi = mfma32(pa, opD, zero);              // S3
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float a = vr[r], b = vi[r];
            vr[r] = a * tw[r].x + b * tw[r].y;
            vi[r] = b * tw[r].x - a * tw[r].y;
        }
        const u32x4 vb = stack(vr, vi);
        const f32x4 yr = mfma32(opC4, vb, zero), yi = mfma32(opD4, vb, zero);      // S4
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            const int b = 2 * (p0 + p) + m;
            if constexpr (VEC) {   // into the staging rows of the output gates (read above), stored below
#pragma unroll
                for (int r = 0; r < 2; ++r)
                    st[2][(2 * p + m) * 128 + (2 * kg + r) * 16 + l16] = __builtin_bit_cast(uint16_t, (bf16_t)((m ? yi[r] : yr[r]) * gout[p][m][r]));
            } else if (b < B) {
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                    const int t = (2 * kg + r) * 16 + l16;
                    if (t < n) y[((int64_t)b * H + h) * n + t] = (bf16_t)((m ? yi[r] : yr[r]) * gout[p][m][r]);
                }
            }
        }
    }
    if constexpr (VEC) {
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int it = 0; it < PAIRS / 2; ++it) {
            const int r = 4 * it + (lane >> 4), b = 2 * (p0 + (r >> 1)) + (r & 1), e0 = 8 * l16;
            if (p0 + (r >> 1) < npairs && b < B && e0 < n)
                store_stream16(y + ((int64_t)b * H + h) * n + e0, *reinterpret_cast<const uint4 *>(&st[2][r * 128 + e0]));
        }
    }
}

}  // namespace c256

bool conv_mfma_256_supported(int n, int klen, const int *factors, int nf, monarch_dtype dt)
{
    return dt == MONARCH_BF16 && nf == 2 && factors[0] == 16 && factors[1] == 16 && n >= 1 && n <= 128 && klen >= 1 && klen <= 256;
}

int launch_conv_mfma_256(const void *u, const void *k, const void *g_in, const void *g_out, void *y, int B, int H, int n,
                         int klen, hipStream_t s)
{
    const int npairs = (B + 1) / 2;
    const int groups = (npairs + c256::PAIRS - 1) / c256::PAIRS;
    const dim3 grid((unsigned)H, (unsigned)((groups + 3) / 4));
    if (grid.y > 65535) return fail(MONARCH_ESHAPE, "batch too large for one launch");
    const bool vec = n % 8 == 0;
#define MONARCH_LAUNCH_C256(GI, GO)                                                                                  \
    do {                                                                                                             \
        if (vec)                                                                                                     \
            hipLaunchKernelGGL((c256::conv256_bf16_kernel<GI, GO, true>), grid, dim3(256), 0, s, (const bf16_t *)u,  \
                               (const bf16_t *)k, (const bf16_t *)g_in, (const bf16_t *)g_out, (bf16_t *)y, B, H, n, klen); \
        else                                                                                                         \
            hipLaunchKernelGGL((c256::conv256_bf16_kernel<GI, GO, false>), grid, dim3(256), 0, s, (const bf16_t *)u, \
                               (const bf16_t *)k, (const bf16_t *)g_in, (const bf16_t *)g_out, (bf16_t *)y, B, H, n, klen); \
    } while (0)
    if (g_in && g_out) MONARCH_LAUNCH_C256(true, true);
    else if (g_in) MONARCH_LAUNCH_C256(true, false);
    else if (g_out) MONARCH_LAUNCH_C256(false, true);
    else MONARCH_LAUNCH_C256(false, false);
#undef MONARCH_LAUNCH_C256
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

}  // namespace monarch
