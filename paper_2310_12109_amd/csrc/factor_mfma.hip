// One block-diagonal factor of a rectangular order-2 Monarch matrix (Sec. 3.1) together with the
// permutations on both of its sides, bf16 I/O, fp32 accumulate:
//   out[t][P_out(k, r)] = sum_c W_k[r, c] * in[t][P_in(k, c)]  (+ bias[P_out(k, r)])
// FIRST factor  (R of M = P L P R P):  P_in(k, c) = c nb + k          (the right-most P)
//                                      P_out(k, r) = r nb + k          (the middle P)
// SECOND factor (L):                   P_in(k, a) = k r_in + a         (input already permuted)
//                                      P_out(k, r) = r nb + k          (the left-most P)
// SECOND_GATHER (L fed with the natural block order [block][row] of the previous factor's
// output, i.e. the middle P is applied here): with j = k r_in + a,
//                                      P_in(k, a) = (j mod nb) (d_in / nb) + j / nb.
//
// One workgroup takes 16 tokens and every block: the token rows are read and written whole
// (coalesced 16-byte accesses) through LDS tiles, the permutations are 2-byte LDS index maps, the
// weights are 16-byte loads (8 consecutive inputs of one row) served by L2.  Tokens sit on the MFMA
// column index; wave w takes blocks w, w + 4, ...
#include "kernels.h"

namespace monarch {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

namespace fac {

constexpr int TOK = 16;

union Pack8 {
    bf16x8 v;
    uint32_t d[4];
    uint4 q;
};

enum { IN_FIRST = 0, IN_SECOND = 1, IN_SECOND_GATHER = 2 };

// KS = r_in / 32 k-steps.
template <int KS, int MODE>
__global__ __launch_bounds__(256, 2) void factor_kernel(const bf16_t *__restrict__ in, bf16_t *__restrict__ out,
                                                        int64_t tokens, int nb, int r_out, const bf16_t *__restrict__ W,
                                                        const bf16_t *__restrict__ bias)
{
    constexpr int RIN = 32 * KS;
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    const int d_in = nb * RIN, d_out = nb * r_out;
    const int ld_in = d_in + 8, ld_out = d_out + 8;   // row pitch: 16-byte aligned, 4 words off a bank multiple
    uint16_t *tin = lds, *tout = lds + TOK * ld_in;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, l16 = lane & 15, kg = lane >> 4;
    const int64_t t0 = (int64_t)blockIdx.x * TOK;

    // token rows -> LDS, 16 bytes per access
    const int pin = d_in / 8;
    for (int idx = tid; idx < TOK * pin; idx += 256) {
        const int t = idx / pin, o = (idx - t * pin) * 8;
        int64_t tt = t0 + t;
        if (tt >= tokens) tt = tokens - 1;   // clamp: computed, never stored
        *reinterpret_cast<uint4 *>(tin + t * ld_in + o) = *reinterpret_cast<const uint4 *>(in + tt * d_in + o);
    }
    __syncthreads();

    const uint16_t *row = tin + l16 * ld_in;
    for (int k = wave; k < nb; k += 4) {
        // B operands: slot e of k-step ks is input c = 32 ks + 8 kg + e of block k
        Pack8 xop[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                uint32_t w[2];
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const int c = 32 * ks + 8 * kg + 2 * h + q;
                    int pos;
                    if (MODE == IN_FIRST) pos = c * nb + k;
                    else if (MODE == IN_SECOND) pos = k * RIN + c;
                    else {
                        const int j = k * RIN + c;
                        pos = (j % nb) * RIN + j / nb;   // d_in / nb = RIN
                    }
                    w[q] = row[pos];
                }
                xop[ks].d[h] = w[0] | (w[1] << 16);
            }
        const bf16_t *Wk = W + (size_t)k * r_out * RIN;
        for (int mt = 0; mt < r_out / 16; ++mt) {
            Pack8 a[KS];
            const bf16_t *wrow = Wk + (size_t)(16 * mt + l16) * RIN + 8 * kg;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) a[ks].q = *reinterpret_cast<const uint4 *>(wrow + 32 * ks);
            f32x4 acc = {0, 0, 0, 0};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[ks].v, xop[ks].v, acc, 0, 0, 0);
            // rows r = 16 mt + 4 kg + i of block k, token l16  ->  output position r nb + k
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int pos = (16 * mt + 4 * kg + i) * nb + k;
                float v = acc[i];
                if (bias) v += (float)bias[pos];
                tout[l16 * ld_out + pos] = __builtin_bit_cast(uint16_t, (__bf16)v);
            }
        }
    }
    __syncthreads();

    const int pout = d_out / 8;
    for (int idx = tid; idx < TOK * pout; idx += 256) {
        const int t = idx / pout, o = (idx - t * pout) * 8;
        if (t0 + t < tokens)
            *reinterpret_cast<uint4 *>(out + (t0 + t) * d_out + o) = *reinterpret_cast<const uint4 *>(tout + t * ld_out + o);
    }
}

}  // namespace fac

bool factor_mfma_supported(int nb, int r_out, int r_in, monarch_dtype dt)
{
    if (dt != MONARCH_BF16 || nb < 1) return false;
    if (r_in % 32 || r_in > 192 || r_out % 16) return false;
    const size_t lds = (size_t)fac::TOK * ((size_t)nb * r_in + 8 + (size_t)nb * r_out + 8) * 2;
    return lds <= 160 * 1024;
}

int launch_factor_mfma(const void *in, void *out, int64_t tokens, int nb, int r_out, int r_in, const void *W,
                       const void *bias, int mode, hipStream_t s)
{
    if (tokens == 0) return MONARCH_OK;
    const int64_t grid = (tokens + fac::TOK - 1) / fac::TOK;
    if (grid > 0x7fffffffLL) return fail(MONARCH_ESHAPE, "too many tokens for one launch");
    const size_t lds = (size_t)fac::TOK * ((size_t)nb * r_in + 8 + (size_t)nb * r_out + 8) * 2;
#define MONARCH_LAUNCH_FAC(KSV, MODEV)                                                                            \
    do {                                                                                                          \
        auto kern = fac::factor_kernel<KSV, MODEV>;                                                               \
        if (lds > 48 * 1024)                                                                                      \
            MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,  \
                                                  (int)lds));                                                     \
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, s, (const bf16_t *)in, (bf16_t *)out,      \
                           tokens, nb, r_out, (const bf16_t *)W, (const bf16_t *)bias);                           \
    } while (0)
#define MONARCH_LAUNCH_FAC_MODE(KSV)                                         \
    do {                                                                     \
        if (mode == fac::IN_FIRST) MONARCH_LAUNCH_FAC(KSV, fac::IN_FIRST);   \
        else if (mode == fac::IN_SECOND) MONARCH_LAUNCH_FAC(KSV, fac::IN_SECOND); \
        else MONARCH_LAUNCH_FAC(KSV, fac::IN_SECOND_GATHER);                 \
    } while (0)
    switch (r_in / 32) {
    case 1: MONARCH_LAUNCH_FAC_MODE(1); break;
    case 2: MONARCH_LAUNCH_FAC_MODE(2); break;
    case 3: MONARCH_LAUNCH_FAC_MODE(3); break;
    case 4: MONARCH_LAUNCH_FAC_MODE(4); break;
    case 5: MONARCH_LAUNCH_FAC_MODE(5); break;
    default: MONARCH_LAUNCH_FAC_MODE(6); break;
    }
#undef MONARCH_LAUNCH_FAC_MODE
#undef MONARCH_LAUNCH_FAC
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

}  // namespace monarch
