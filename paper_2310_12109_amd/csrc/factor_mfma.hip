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
// (coalesced 16-byte accesses) through LDS tiles.  P_in is applied while the rows are copied into
// LDS (2-byte scatter), so that a block's inputs are contiguous and an MFMA operand is one 16-byte
// read; P_out is a 2-byte scatter of the accumulators into the output tile; the bias is added
// when the tile is copied out.  The weights are 16-byte loads (8 consecutive inputs of one row)
// served by L2.  Tokens sit on the MFMA column index.  The workgroup has 16 waves and the (block,
// row tile) units are dealt round-robin to them, each wave requesting the weights of its first units
// before it waits for the token tile: one trip to HBM and one to L2 per workgroup, overlapped.
#include "half16.h"
#include "kernels.h"

namespace monarch {

using h16::f32x4;
using h16::op8;

namespace fac {

constexpr int THREADS = 1024, WAVES = THREADS / 64;

union Pack8 {
    op8 v;
    uint32_t d[4];
    uint16_t h[8];
    uint4 q;
};

enum { IN_FIRST = 0, IN_SECOND = 1, IN_SECOND_GATHER = 2 };

// the input and the output tile, bf16, rows padded by 8 elements
static inline size_t lds_bytes(int tok, int nb, int r_out, int r_in)
{
    return (size_t)tok * ((size_t)nb * r_in + 8 + (size_t)nb * r_out + 8) * 2;
}

// KS = r_in / 32 k-steps; NTK column tiles of 16 tokens per workgroup.
template <typename E, int KS, int MODE, int NTK>
__global__ __launch_bounds__(1024) void factor_kernel(const E *__restrict__ in, E *__restrict__ out,
                                                        int64_t tokens, int nb, int r_out, const E *__restrict__ W,
                                                        const E *__restrict__ bias)
{
    constexpr int RIN = 32 * KS, TOK = 16 * NTK;
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    const int d_in = nb * RIN, d_out = nb * r_out;
    const int ld_in = d_in + 8, ld_out = d_out + 8;   // row pitch: 16-byte aligned, 4 words off a bank multiple
    uint16_t *tin = lds, *tout = lds + TOK * ld_in;   // tin: [token][block][input], tout: natural output order
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, l16 = lane & 15, kg = lane >> 4;
    const int64_t t0 = (int64_t)blockIdx.x * TOK;

    // unit u = (block k, row tile mt) = (u / mts, u % mts); this wave takes units wave, wave + 16, ...,
    // UB at a time, with all their weight loads in flight together
    constexpr int UB = KS > 3 ? 2 : 4;
    const int mts = r_out / 16, units = nb * mts;
    Pack8 a[UB][KS];
    auto request = [&](int u0) {
#pragma unroll
        for (int b = 0; b < UB; ++b) {
            int u = u0 + b * WAVES;
            if (u >= units) u = u0;
            const int k = u / mts, mt = u - k * mts;
            const E *wrow = W + ((size_t)k * r_out + 16 * mt + l16) * RIN + 8 * kg;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) a[b][ks].q = *reinterpret_cast<const uint4 *>(wrow + 32 * ks);
        }
    };
    if (wave < units) request(wave);

    // token rows -> LDS, 16 bytes per global access, two accesses in flight per thread; element i of
    // a row goes to its block-major position
    const int pin = d_in / 8, npieces = TOK * pin;
    for (int base = tid; base < npieces; base += 2 * THREADS) {
        Pack8 v[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = base + u * THREADS < npieces ? base + u * THREADS : base;
            const int t = idx / pin, o = (idx - t * pin) * 8;
            int64_t tt = t0 + t;
            if (tt >= tokens) tt = tokens - 1;   // clamp: computed, never stored
            v[u].q = *reinterpret_cast<const uint4 *>(in + tt * d_in + o);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = base + u * THREADS;
            if (idx >= npieces) break;
            const int t = idx / pin, o = (idx - t * pin) * 8;
            uint16_t *dst = tin + t * ld_in;
            if (MODE == IN_SECOND) {
                *reinterpret_cast<uint4 *>(dst + o) = v[u].q;
            } else if (MODE == IN_FIRST) {        // i = c nb + k  ->  k RIN + c
                int c = o / nb, k = o - c * nb;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    dst[k * RIN + c] = v[u].h[e];
                    if (++k == nb) {
                        k = 0;
                        ++c;
                    }
                }
            } else {                               // i = kk RIN + r (previous factor's block kk, row r)  ->  r nb + kk
                const int kk = o / RIN, r = o - kk * RIN;
#pragma unroll
                for (int e = 0; e < 8; ++e) dst[(r + e) * nb + kk] = v[u].h[e];
            }
        }
    }
    __syncthreads();

    const uint16_t *row = tin + l16 * ld_in + 8 * kg;
    for (int u0 = wave; u0 < units; u0 += UB * WAVES) {
        if (u0 != wave) request(u0);   // (the first batch was requested before the barrier)
#pragma unroll
        for (int b = 0; b < UB; ++b) {
            const int u = u0 + b * WAVES;
            if (u < units) {
                const int k = u / mts, mt = u - k * mts;
                // B operands: slot e of k-step ks is input c = 32 ks + 8 kg + e of block k
#pragma unroll
                for (int nt = 0; nt < NTK; ++nt) {
                    f32x4 acc = {0, 0, 0, 0};
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
                        Pack8 xop;
                        xop.q = *reinterpret_cast<const uint4 *>(row + 16 * nt * ld_in + k * RIN + 32 * ks);
                        acc = h16::mfma<E>(a[b][ks].v, xop.v, acc);
                    }
                    // rows r = 16 mt + 4 kg + i of block k, token 16 nt + l16  ->  output position r nb + k
                    // (rounded to bf16 here; the bias is added to that value at copy-out and the sum
                    // rounded again: at most half a bf16 ulp more than a single rounding)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        tout[(16 * nt + l16) * ld_out + (16 * mt + 4 * kg + i) * nb + k] = __builtin_bit_cast(uint16_t, (E)acc[i]);
                }
            }
        }
    }
    __syncthreads();

    const int pout = d_out / 8, nout = TOK * pout;
    for (int base = tid; base < nout; base += 2 * THREADS) {
        Pack8 v[2], bv[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = base + u * THREADS < nout ? base + u * THREADS : base;
            const int t = idx / pout, o = (idx - t * pout) * 8;
            v[u].q = *reinterpret_cast<const uint4 *>(tout + t * ld_out + o);
            bv[u].q = make_uint4(0u, 0u, 0u, 0u);
            if (bias) bv[u].q = *reinterpret_cast<const uint4 *>(bias + o);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = base + u * THREADS;
            if (idx >= nout) break;
            const int t = idx / pout, o = (idx - t * pout) * 8;
            if (t0 + t >= tokens) continue;
            if (bias) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float sum = (float)__builtin_bit_cast(E, v[u].h[e]) + (float)__builtin_bit_cast(E, bv[u].h[e]);
                    v[u].h[e] = __builtin_bit_cast(uint16_t, (E)sum);
                }
            }
            *reinterpret_cast<uint4 *>(out + (t0 + t) * d_out + o) = v[u].q;
        }
    }
}

}  // namespace fac

bool factor_mfma_supported(int nb, int r_out, int r_in, monarch_dtype dt)
{
    if ((dt != MONARCH_BF16 && dt != MONARCH_F16) || nb < 1) return false;
    if (r_in % 32 || r_in > 192 || r_out % 16) return false;
    return fac::lds_bytes(16, nb, r_out, r_in) <= 160 * 1024;
}

namespace {

template <typename E>
int launch_typed(const void *in, void *out, int64_t tokens, int nb, int r_out, int r_in, const void *W,
                 const void *bias, int mode, hipStream_t s)
{
    if (tokens == 0) return MONARCH_OK;
    // 16 tokens per workgroup: measured faster than 32 (which halves the weight traffic out of L2
    // but leaves one workgroup per compute unit with twice the serial copy-in / copy-out time)
    const int tok = 16;
    const int64_t grid = (tokens + tok - 1) / tok;
    if (grid > 0x7fffffffLL) return fail(MONARCH_ESHAPE, "too many tokens for one launch");
    const size_t lds = fac::lds_bytes(tok, nb, r_out, r_in);
#define MONARCH_LAUNCH_FAC(KSV, MODEV, NTKV)                                                                            \
    do {                                                                                                          \
        auto kern = fac::factor_kernel<E, KSV, MODEV, NTKV>;                                                             \
        if (lds > 48 * 1024)                                                                                      \
            MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,  \
                                                  (int)lds));                                                     \
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(fac::THREADS), lds, s, (const E *)in, (E *)out, \
                           tokens, nb, r_out, (const E *)W, (const E *)bias);                           \
    } while (0)
#define MONARCH_LAUNCH_FAC_MODE(KSV)                                         \
    do {                                                                     \
        if (tok == 32) {                                                     \
            if (mode == fac::IN_FIRST) MONARCH_LAUNCH_FAC(KSV, fac::IN_FIRST, 2);   \
            else if (mode == fac::IN_SECOND) MONARCH_LAUNCH_FAC(KSV, fac::IN_SECOND, 2); \
            else MONARCH_LAUNCH_FAC(KSV, fac::IN_SECOND_GATHER, 2);          \
        } else {                                                             \
            if (mode == fac::IN_FIRST) MONARCH_LAUNCH_FAC(KSV, fac::IN_FIRST, 1);   \
            else if (mode == fac::IN_SECOND) MONARCH_LAUNCH_FAC(KSV, fac::IN_SECOND, 1); \
            else MONARCH_LAUNCH_FAC(KSV, fac::IN_SECOND_GATHER, 1);          \
        }                                                                    \
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

}  // namespace

int launch_factor_mfma(const void *in, void *out, int64_t tokens, int nb, int r_out, int r_in, const void *W,
                       const void *bias, int mode, monarch_dtype dt, hipStream_t s)
{
    if (dt == MONARCH_F16) return launch_typed<f16_t>(in, out, tokens, nb, r_out, r_in, W, bias, mode, s);
    return launch_typed<bf16_t>(in, out, tokens, nb, r_out, r_in, W, bias, mode, s);
}

}  // namespace monarch
