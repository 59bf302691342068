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

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;   // (arrays of HIP's uint4 struct can end up in scratch memory)
union Pack8 {
    op8 v;
    uint32_t d[4];
    uint16_t h[8];
    u32x4 q;
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
            for (int ks = 0; ks < KS; ++ks) a[b][ks].q = *reinterpret_cast<const u32x4 *>(wrow + 32 * ks);
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
            v[u].q = *reinterpret_cast<const u32x4 *>(in + tt * d_in + o);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = base + u * THREADS;
            if (idx >= npieces) break;
            const int t = idx / pin, o = (idx - t * pin) * 8;
            uint16_t *dst = tin + t * ld_in;
            if (MODE == IN_SECOND) {
                *reinterpret_cast<u32x4 *>(dst + o) = v[u].q;
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
                        xop.q = *reinterpret_cast<const u32x4 *>(row + 16 * nt * ld_in + k * RIN + 32 * ks);
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
            v[u].q = *reinterpret_cast<const u32x4 *>(tout + t * ld_out + o);
            bv[u].q = u32x4{0u, 0u, 0u, 0u};
            if (bias) bv[u].q = *reinterpret_cast<const u32x4 *>(bias + o);
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
            *reinterpret_cast<u32x4 *>(out + (t0 + t) * d_out + o) = v[u].q;
        }
    }
}


// The same factor with resident weights: a workgroup keeps going over tiles of 16 tokens (tile blockIdx.x,
// + gridDim.x, ...).  Every wave owns the same UPW units (block, row tile) in each tile, so their weights are
// loaded once per workgroup and stay in registers; the token rows of the next tile are requested before the
// current tile is multiplied; each thread's pieces of the rows sit at the same places in every tile, so the
// piece arithmetic and the bias are computed once.  NPI / NPO: 16-byte pieces per thread of a tile's input /
// output rows (16 d / 8 pieces over 1024 threads; d <= 1024).
// Position of element pos of a token row inside its LDS tile row: the 16-byte pieces of a row are permuted (piece index
// XOR three higher bits of itself) so that the 2-byte scatters of a wave, whose targets lie a multiple of 128 bytes
// apart, spread over the banks; SH: which bits (4 for the input tile, 3 for the output tile).
template <int SH> __device__ __forceinline__ int swz8(int pos)
{
    const int piece = pos >> 3;
    return ((piece ^ ((piece >> SH) & 7)) << 3) | (pos & 7);
}

template <typename E, int KS, int MODE, int UPW>
__global__ __launch_bounds__(1024) void factor_resident_kernel(const E *__restrict__ in, E *__restrict__ out,
                                                                 int64_t tokens, int nb, int r_out, const E *__restrict__ W,
                                                                 const E *__restrict__ bias, int ntiles)
{
    constexpr int RIN = 32 * KS, TOK = 16, NPI = 2, NPO = 2;
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    const int d_in = nb * RIN, d_out = nb * r_out;
    const int ld_in = d_in + 8, ld_out = d_out + 8;
    uint16_t *tin = lds, *tout = lds + TOK * ld_in;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, l16 = lane & 15, kg = lane >> 4;

    const int mts = r_out / 16, units = nb * mts;
    Pack8 a[UPW][KS];
    int uk[UPW], umt[UPW];
#pragma unroll
    for (int b = 0; b < UPW; ++b) {
        int u = wave + b * WAVES;
        if (u >= units) u = units - 1;   // (computed and dropped)
        uk[b] = u / mts;
        umt[b] = u - uk[b] * mts;
        const E *wrow = W + ((size_t)uk[b] * r_out + 16 * umt[b] + l16) * RIN + 8 * kg;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) a[b][ks].q = *reinterpret_cast<const u32x4 *>(wrow + 32 * ks);
    }

    // this thread's pieces of a tile: input piece q covers elements o .. o + 7 of token t
    const int pin = d_in / 8, npin = TOK * pin, pout = d_out / 8, npout = TOK * pout;
    int it[NPI], io[NPI], ot[NPO], oo[NPO];
    Pack8 bv[NPO];
#pragma unroll
    for (int q = 0; q < NPI; ++q) {
        const int idx = tid + q * THREADS < npin ? tid + q * THREADS : tid;   // (tid < npin: d_in >= 512)
        it[q] = idx / pin;
        io[q] = (idx - it[q] * pin) * 8;
    }
#pragma unroll
    for (int q = 0; q < NPO; ++q) {
        const int idx = tid + q * THREADS < npout ? tid + q * THREADS : tid;
        ot[q] = idx / pout;
        oo[q] = (idx - ot[q] * pout) * 8;
        bv[q].q = u32x4{0u, 0u, 0u, 0u};
        if (bias) bv[q].q = *reinterpret_cast<const u32x4 *>(bias + oo[q]);
    }

    Pack8 v[NPI];
    auto request = [&](int tile) {
#pragma unroll
        for (int q = 0; q < NPI; ++q)
            if (q == 0 || tid + q * THREADS < npin) {
                int64_t tt = (int64_t)tile * TOK + it[q];
                if (tt >= tokens) tt = tokens - 1;   // clamp: computed, never stored
                v[q].q = MODE == IN_FIRST ? __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(in + tt * d_in + io[q]))
                                          : *reinterpret_cast<const u32x4 *>(in + tt * d_in + io[q]);
            }
    };

    int tile = blockIdx.x;
    if (tile < ntiles) request(tile);
    const uint16_t *row = tin + l16 * ld_in;
    for (; tile < ntiles; tile += gridDim.x) {
        // token rows -> LDS, element i of a row to its block-major position
#pragma unroll
        for (int q = 0; q < NPI; ++q)
            if (tid + q * THREADS < npin) {
                uint16_t *dst = tin + it[q] * ld_in;
                const int o = io[q];
                if (MODE == IN_SECOND) {
                    *reinterpret_cast<u32x4 *>(dst + swz8<4>(o)) = v[q].q;
                } else if (MODE == IN_FIRST) {        // i = c nb + k  ->  k RIN + c
                    int c = o / nb, k = o - c * nb;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        dst[swz8<4>(k * RIN + c)] = v[q].h[e];
                        if (++k == nb) {
                            k = 0;
                            ++c;
                        }
                    }
                } else {                               // i = kk RIN + r (previous factor's block kk, row r)  ->  r nb + kk
                    const int kk = o / RIN, r = o - kk * RIN;
#pragma unroll
                    for (int e = 0; e < 8; ++e) dst[swz8<4>((r + e) * nb + kk)] = v[q].h[e];
                }
            }
        __syncthreads();
        if (tile + (int)gridDim.x < ntiles) request(tile + gridDim.x);

#pragma unroll
        for (int b = 0; b < UPW; ++b)
            if (wave + b * WAVES < units) {
                f32x4 acc = {0, 0, 0, 0};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    Pack8 xop;
                    xop.q = *reinterpret_cast<const u32x4 *>(row + swz8<4>(uk[b] * RIN + 32 * ks + 8 * kg));
                    acc = h16::mfma<E>(a[b][ks].v, xop.v, acc);
                }
                // rows r = 16 mt + 4 kg + i of block k, token l16  ->  output position r nb + k (rounded here; the
                // bias is added to that value at copy-out and the sum rounded again)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    tout[l16 * ld_out + swz8<3>((16 * umt[b] + 4 * kg + i) * nb + uk[b])] = __builtin_bit_cast(uint16_t, (E)acc[i]);
            }
        __syncthreads();

#pragma unroll
        for (int q = 0; q < NPO; ++q)
            if (tid + q * THREADS < npout) {
                const int64_t tt = (int64_t)tile * TOK + ot[q];
                Pack8 r;
                r.q = *reinterpret_cast<const u32x4 *>(tout + ot[q] * ld_out + swz8<3>(oo[q]));
                if (bias) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float sum = (float)__builtin_bit_cast(E, r.h[e]) + (float)__builtin_bit_cast(E, bv[q].h[e]);
                        r.h[e] = __builtin_bit_cast(uint16_t, (E)sum);
                    }
                }
                if (tt < tokens) {
                    if (MODE == IN_FIRST) *reinterpret_cast<u32x4 *>(out + tt * d_out + oo[q]) = r.q;
                    else __builtin_nontemporal_store(r.q, reinterpret_cast<u32x4 *>(out + tt * d_out + oo[q]));
                }
            }
        // (the next tile's rows go to tin, which nobody reads any more; tout is rewritten only after the next barrier)
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

template <typename E, int KS, int MODE, int UPW>
int launch_resident_one(const void *in, void *out, int64_t tokens, int nb, int r_out, const void *W, const void *bias,
                        hipStream_t s)
{
    const size_t lds = fac::lds_bytes(16, nb, r_out, 32 * KS);
    const int64_t ntiles = (tokens + 15) / 16;
    if (ntiles > 0x7fffffffLL) return fail(MONARCH_ESHAPE, "too many tokens for one launch");
    int dev = 0, ncu = 0;
    MONARCH_HIP_CHECK(hipGetDevice(&dev));
    MONARCH_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
    auto kern = fac::factor_resident_kernel<E, KS, MODE, UPW>;
    if (lds > 48 * 1024)
        MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    int per_cu = 1;   // workgroups that fit a compute unit at once (registers and LDS): the grid is exactly one round
    MONARCH_HIP_CHECK(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void *)kern, fac::THREADS, lds));
    if (per_cu < 1) per_cu = 1;
    const int64_t cap = (int64_t)ncu * per_cu;
    const int64_t grid = ntiles < cap ? ntiles : cap;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(fac::THREADS), lds, s, (const E *)in, (E *)out, tokens, nb, r_out,
                       (const E *)W, (const E *)bias, (int)ntiles);
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

template <typename E, int KS, int UPW>
int launch_resident_mode(const void *in, void *out, int64_t tokens, int nb, int r_out, const void *W, const void *bias,
                         int mode, hipStream_t s)
{
    if (mode == fac::IN_FIRST) return launch_resident_one<E, KS, fac::IN_FIRST, UPW>(in, out, tokens, nb, r_out, W, bias, s);
    if (mode == fac::IN_SECOND) return launch_resident_one<E, KS, fac::IN_SECOND, UPW>(in, out, tokens, nb, r_out, W, bias, s);
    return launch_resident_one<E, KS, fac::IN_SECOND_GATHER, UPW>(in, out, tokens, nb, r_out, W, bias, s);
}

template <typename E>
int launch_resident(const void *in, void *out, int64_t tokens, int nb, int r_out, int r_in, const void *W, const void *bias,
                    int mode, int upw, hipStream_t s)
{
#define MONARCH_RES(KSV)                                                                                      \
    case KSV:                                                                                                 \
        if constexpr (KSV * 2 <= 12) {                                                                        \
            if (upw == 2) return launch_resident_mode<E, KSV, 2>(in, out, tokens, nb, r_out, W, bias, mode, s); \
        }                                                                                                     \
        if constexpr (KSV * 4 <= 12) {                                                                        \
            if (upw == 4) return launch_resident_mode<E, KSV, 4>(in, out, tokens, nb, r_out, W, bias, mode, s); \
        }                                                                                                     \
        break;
    switch (r_in / 32) {
        MONARCH_RES(1)
        MONARCH_RES(2)
        MONARCH_RES(3)
        MONARCH_RES(4)
        MONARCH_RES(5)
        MONARCH_RES(6)
    default: break;
    }
#undef MONARCH_RES
    return fail(MONARCH_EINVAL, "internal: resident factor kernel %d x %d units not built", r_in / 32, upw);
}

template <typename E>
int launch_typed(const void *in, void *out, int64_t tokens, int nb, int r_out, int r_in, const void *W,
                 const void *bias, int mode, hipStream_t s)
{
    if (tokens == 0) return MONARCH_OK;
    const int tok = 16;   // tokens per tile
    {
        // resident weights when a wave's share of them fits in registers and a thread has at most two pieces of a
        // tile's rows on either side
        const int units = nb * (r_out / 16), upw = (units + fac::WAVES - 1) / fac::WAVES, ks = r_in / 32;
        const int d_in = nb * r_in, d_out = nb * r_out;
        const int built = upw <= 2 ? 2 : 4;   // units per wave of the instantiated kernels
        // (rows of a multiple of 64 elements: the tiles permute 16-byte pieces within groups of eight)
        if (upw <= 4 && built * ks <= 12 && d_in >= 512 && d_in <= 1024 && d_out >= 512 && d_out <= 1024 && d_in % 64 == 0 && d_out % 64 == 0)
            return launch_resident<E>(in, out, tokens, nb, r_out, r_in, W, bias, mode, built, s);
    }
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
        if (mode == fac::IN_FIRST) MONARCH_LAUNCH_FAC(KSV, fac::IN_FIRST, 1);   \
        else if (mode == fac::IN_SECOND) MONARCH_LAUNCH_FAC(KSV, fac::IN_SECOND, 1); \
        else MONARCH_LAUNCH_FAC(KSV, fac::IN_SECOND_GATHER, 1);              \
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
