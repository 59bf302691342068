// One block-diagonal factor of the Monarch DFT (appendix, DFT corollary) on the matrix cores, for
// bf16 transforms whose factor is 16, 32, 64 or 128.
//
// The row is viewed as [O][f][S] and the middle digit is contracted with F_f; the result is
// multiplied by the twiddle diagonal omega_(fS)^(j s) and written back.  As a GEMM: A = F_f
// (bf16, built once per workgroup in LDS in MFMA operand order), B = 16 "columns" (one (o, s)
// each) by f contraction values, loaded straight from global memory into operand registers,
// D = fp32 accumulators.  Complex arithmetic is four real MFMA chains per output tile:
//   Dr = Fr Br + Fi (-Bi),   Di = Fi Br + Fr Bi.
// Between passes a row is stored as packed bf16 pairs (re, im): the next pass would round its
// operands to bf16 anyway, so this halves the traffic at no cost in accuracy.
//
// Column tiles: when S >= 16 a tile is 16 consecutive s (loads and stores are 16-lane contiguous
// runs); the last pass (S = 1) takes 16 consecutive *natural output* positions, so that its
// stores are contiguous, and each lane reads its own contiguous run of f inputs.
#include "kernels.h"

namespace monarch {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

namespace fpm {

__device__ __forceinline__ uint32_t pack2(float lo, float hi)
{
    bf16x2 v = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ float lo_f32(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float hi_f32(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }

__device__ __forceinline__ f32x4 mfma(u32x4 a, u32x4 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// Real rows of complex row rc when two real rows of the same channel are packed as (re, im):
// complex row b2 * H + h holds real rows (2 b2) * H + h and (2 b2 + 1) * H + h.
__device__ __forceinline__ int64_t pair_first_row(const FftPass &p, int64_t rc) { return rc + (rc / p.H) * p.H; }

// One input element as a complex number, with the load mode's conjugation / gating / spectrum
// product applied.  pos is the position inside the row.
template <int LOAD>
__device__ __forceinline__ float2 load_value(const FftPass &p, int64_t rc, int pos)
{
    typedef bf16_t T;
    if constexpr (LOAD == LD_C32_CONJ) {
        const float2 v = ((const float2 *)p.in)[rc * p.N + pos];
        return make_float2(v.x, -v.y);
    } else if constexpr (LOAD == LD_CPLX) {
        const uint32_t w = ((const uint32_t *)p.in)[rc * p.N + pos];
        return make_float2(lo_f32(w), hi_f32(w));
    } else if constexpr (LOAD == LD_C16_CONJ_MULK) {
        const uint32_t w = ((const uint32_t *)p.in)[rc * p.N + pos];
        const float2 k = p.kf[(rc % p.H) * (int64_t)p.N + pos];
        const float2 m = cmul(make_float2(lo_f32(w), hi_f32(w)), k);
        return make_float2(m.x, -m.y);
    } else if constexpr (LOAD == LD_REAL) {
        const bool ok = pos < p.n_valid;
        const int64_t at = rc * p.n_valid + (ok ? pos : 0);
        float v = to_f32(((const T *)p.in)[at]);
        if (p.gate) v *= to_f32(((const T *)p.gate)[at]);
        return make_float2(ok ? v : 0.0f, 0.0f);
    } else {  // LD_REAL_PAIR
        const bool ok = pos < p.n_valid;
        const int64_t ra = pair_first_row(p, rc);
        const bool okb = ok && ra + p.H < p.real_rows;
        const int64_t at = ra * p.n_valid + (ok ? pos : 0);
        const int64_t bt = okb ? at + (int64_t)p.H * p.n_valid : at;
        float va = to_f32(((const T *)p.in)[at]), vb = to_f32(((const T *)p.in)[bt]);
        if (p.gate) {
            va *= to_f32(((const T *)p.gate)[at]);
            vb *= to_f32(((const T *)p.gate)[bt]);
        }
        return make_float2(ok ? va : 0.0f, okb ? vb : 0.0f);
    }
}

template <int F, int LOAD, int STORE, bool CONTIG>
__global__ __launch_bounds__(256, 2) void fft_pass_mfma_kernel(const FftPass p)
{
    constexpr int JT = F / 16, KS = (F + 31) / 32;
    constexpr bool REAL_B = LOAD == LD_REAL;                   // imaginary part of the input is zero
    constexpr bool REAL_D = STORE == ST_REAL_SCALE_GATE;       // only the real part is kept
    extern __shared__ __attribute__((aligned(16))) u32x4 ftab[];   // [JT][KS][re, im][lane]
    __shared__ float2 roots[F];
    for (int e = threadIdx.x; e < F; e += 256) roots[e] = omega(e, F);
    __syncthreads();
    // A operand of row tile jt, k-step ks: lane (row l16, group kg) holds F[16 jt + l16][32 ks + 8 kg + e]
    for (int idx = threadIdx.x; idx < JT * KS * 64; idx += 256) {
        const int ln = idx & 63, ks = (idx >> 6) % KS, jt = idx / (64 * KS);
        const int j = 16 * jt + (ln & 15), c0 = 32 * ks + 8 * (ln >> 4);
        u32x4 re, im;
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            float2 w0 = make_float2(0.0f, 0.0f), w1 = w0;
            if (c0 + 2 * h < F) w0 = roots[(j * (c0 + 2 * h)) % F];
            if (c0 + 2 * h + 1 < F) w1 = roots[(j * (c0 + 2 * h + 1)) % F];
            re[h] = pack2(w0.x, w1.x);
            im[h] = pack2(w0.y, w1.y);
        }
        ftab[(idx >> 6) * 128 + ln] = re;
        ftab[(idx >> 6) * 128 + 64 + ln] = im;
    }
    __syncthreads();

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63, l16 = lane & 15, kg = lane >> 4;
    const int S = p.S, O = p.O;
    const int tiles_per_unit = CONTIG ? O / 16 : S / 16;           // unit: a row (CONTIG) or one (row, o)
    const int64_t ntiles = p.rows * (CONTIG ? 1 : O) * tiles_per_unit;
    const float inv_fs = 1.0f / (float)((int64_t)F * S);

    for (int64_t tile = (int64_t)blockIdx.x * 4 + wave; tile < ntiles; tile += (int64_t)gridDim.x * 4) {
        int64_t rc;
        int col, base;   // col: s (S >= 16) or natural low index rho (S == 1); base: position of (o, c = 0, s)
        if constexpr (CONTIG) {
            rc = tile / tiles_per_unit;
            col = (int)(tile - rc * tiles_per_unit) * 16 + l16;
            int o = col;   // two factors: the digit itself; three: swap the two digits already produced
            if (p.nf == 3) o = (col % p.factors[0]) * p.factors[1] + col / p.factors[0];
            base = o * F;
        } else {
            const int64_t unit = tile / tiles_per_unit;
            col = (int)(tile - unit * tiles_per_unit) * 16 + l16;
            rc = unit / O;
            base = (int)(unit - rc * O) * F * S + col;
        }

        // ---- B operands: k-step ks, slot e  <->  c = 32 ks + 8 kg + e
        u32x4 br[KS], bi[KS], nbi[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int c0 = 32 * ks + 8 * kg;
            if constexpr (CONTIG) {   // packed bf16 pairs, 8 consecutive elements per lane
                u32x4 w0 = {0, 0, 0, 0}, w1 = w0;
                if (c0 < F) {
                    const u32x4 *src = (const u32x4 *)((const uint32_t *)p.in + rc * p.N + base + c0);
                    w0 = src[0];
                    w1 = src[1];
                }
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    br[ks][h] = (w0[2 * h] & 0xffffu) | (w0[2 * h + 1] << 16);
                    bi[ks][h] = (w0[2 * h] >> 16) | (w0[2 * h + 1] & 0xffff0000u);
                    br[ks][2 + h] = (w1[2 * h] & 0xffffu) | (w1[2 * h + 1] << 16);
                    bi[ks][2 + h] = (w1[2 * h] >> 16) | (w1[2 * h + 1] & 0xffff0000u);
                }
            } else if constexpr (LOAD == LD_C16) {
                uint32_t w[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const bool ok = c0 + e < F;
                    const uint32_t v = ((const uint32_t *)p.in)[rc * p.N + base + (ok ? (c0 + e) * S : 0)];
                    w[e] = ok ? v : 0u;
                }
#pragma unroll
                for (int h = 0; h < 4; ++h) {
                    br[ks][h] = (w[2 * h] & 0xffffu) | (w[2 * h + 1] << 16);
                    bi[ks][h] = (w[2 * h] >> 16) | (w[2 * h + 1] & 0xffff0000u);
                }
            } else {
                // inputs past n_valid are zero: a k-step wholly past it is skipped (wave-uniform)
                const bool live = !(LOAD == LD_REAL || LOAD == LD_REAL_PAIR) || (int64_t)32 * ks * S < p.n_valid;
                float2 v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    v[e] = make_float2(0.0f, 0.0f);
                    if (live) {
                        const bool ok = c0 + e < F;
                        const float2 t = load_value<LOAD>(p, rc, base + (ok ? (c0 + e) * S : 0));
                        if (ok) v[e] = t;
                    }
                }
#pragma unroll
                for (int h = 0; h < 4; ++h) {
                    br[ks][h] = pack2(v[2 * h].x, v[2 * h + 1].x);
                    bi[ks][h] = pack2(v[2 * h].y, v[2 * h + 1].y);
                }
            }
#pragma unroll
            for (int h = 0; h < 4; ++h) nbi[ks][h] = bi[ks][h] ^ 0x80008000u;
        }

        // ---- twiddle seeds: omega_(fS)^(j s) for j = 4 kg + r, stepped by omega_(fS)^(16 s) per row tile
        float2 tw[4], step;
        if constexpr (!CONTIG) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float rev = (float)((4 * kg + r) * col) * inv_fs;   // exact: j s < f S <= 2^24
                tw[r] = make_float2(__builtin_amdgcn_cosf(rev), __builtin_amdgcn_sinf(rev));
            }
            const float rev = (float)(16 * col) * inv_fs;
            step = make_float2(__builtin_amdgcn_cosf(rev), __builtin_amdgcn_sinf(rev));
        }

        // ---- row tiles of the output digit j (kept as a loop: unrolled, the operand reads of all
        // tiles are hoisted and the register file overflows)
#pragma unroll 1
        for (int jt = 0; jt < JT; ++jt) {
            const bool wanted = !(STORE == ST_REAL_SCALE_GATE || STORE == ST_REAL_PAIR) || (int64_t)16 * jt * O < p.n_valid;
            if (wanted) {
                f32x4 dr = {0, 0, 0, 0}, di = {0, 0, 0, 0};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const bool live = !(LOAD == LD_REAL || LOAD == LD_REAL_PAIR) || (int64_t)32 * ks * S < p.n_valid;
                    if (live) {
                        const u32x4 ar = ftab[(jt * KS + ks) * 128 + lane], ai = ftab[(jt * KS + ks) * 128 + 64 + lane];
                        dr = mfma(ar, br[ks], dr);
                        if constexpr (!REAL_B) dr = mfma(ai, nbi[ks], dr);
                        if constexpr (!REAL_D) {
                            di = mfma(ai, br[ks], di);
                            if constexpr (!REAL_B) di = mfma(ar, bi[ks], di);
                        }
                    }
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int j = 16 * jt + 4 * kg + r;
                    float2 z = make_float2(dr[r], di[r]);
                    if constexpr (!CONTIG) {
                        z = cmul(z, tw[r]);
                        const int64_t at = rc * p.N + base + (int64_t)j * S;
                        if constexpr (STORE == ST_C16) ((uint32_t *)p.out)[at] = pack2(z.x, z.y);
                        else ((float2 *)p.out)[at] = z;   // ST_C32
                    } else {
                        const int m = j * O + col;   // natural output index
                        if constexpr (STORE == ST_C32_NATURAL) {
                            ((float2 *)p.out)[rc * p.N + m] = z;
                        } else if constexpr (STORE == ST_C16_NATURAL) {
                            ((uint32_t *)p.out)[rc * p.N + m] = pack2(z.x, z.y);
                        } else if constexpr (STORE == ST_CPLX_CONJ_SCALE) {
                            ((uint32_t *)p.out)[rc * p.N + m] = pack2(z.x * p.scale, -z.y * p.scale);
                        } else if constexpr (STORE == ST_REAL_SCALE_GATE) {
                            if (m < p.n_valid) {
                                const int64_t at = rc * p.n_valid + m;
                                float v = z.x * p.scale;
                                if (p.gate) v *= to_f32(((const bf16_t *)p.gate)[at]);
                                ((bf16_t *)p.out)[at] = (bf16_t)v;
                            }
                        } else {   // ST_REAL_PAIR: F^-1 = conj(F conj(.)) / N, so the second row is -Im
                            if (m < p.n_valid) {
                                const int64_t ra = pair_first_row(p, rc);
                                const int64_t at = ra * p.n_valid + m, bt = at + (int64_t)p.H * p.n_valid;
                                const bool hasb = ra + p.H < p.real_rows;
                                float va = z.x * p.scale, vb = -z.y * p.scale;
                                if (p.gate) {
                                    va *= to_f32(((const bf16_t *)p.gate)[at]);
                                    if (hasb) vb *= to_f32(((const bf16_t *)p.gate)[bt]);
                                }
                                ((bf16_t *)p.out)[at] = (bf16_t)va;
                                if (hasb) ((bf16_t *)p.out)[bt] = (bf16_t)vb;
                            }
                        }
                    }
                }
            }
            if constexpr (!CONTIG) {
#pragma unroll
                for (int r = 0; r < 4; ++r) tw[r] = cmul(tw[r], step);
            }
        }
    }
}

template <int F, int LOAD, int STORE, bool CONTIG>
static int launch_one(const FftPass &p, hipStream_t s)
{
    constexpr int JT = F / 16, KS = (F + 31) / 32;
    const size_t lds = (size_t)JT * KS * 2 * 64 * 16;
    int dev = 0, ncu = 0;
    MONARCH_HIP_CHECK(hipGetDevice(&dev));
    MONARCH_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
    const int64_t ntiles = p.rows * (int64_t)p.N / F / 16;
    int64_t grid = (ntiles + 3) / 4;
    const int64_t cap = (int64_t)ncu * (F == 128 ? 2 : 4);
    if (grid > cap) grid = cap;
    auto kern = fft_pass_mfma_kernel<F, LOAD, STORE, CONTIG>;
    if (lds > 48 * 1024)
        MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, s, p);
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

template <int F>
static int launch_f(const FftPass &p, hipStream_t s)
{
    if (p.S == 1) {
        switch (p.store) {
        case ST_C32_NATURAL: return launch_one<F, LD_C16, ST_C32_NATURAL, true>(p, s);
        case ST_C16_NATURAL: return launch_one<F, LD_C16, ST_C16_NATURAL, true>(p, s);
        case ST_CPLX_CONJ_SCALE: return launch_one<F, LD_C16, ST_CPLX_CONJ_SCALE, true>(p, s);
        case ST_REAL_SCALE_GATE: return launch_one<F, LD_C16, ST_REAL_SCALE_GATE, true>(p, s);
        case ST_REAL_PAIR: return launch_one<F, LD_C16, ST_REAL_PAIR, true>(p, s);
        default: break;
        }
    } else {
        switch (p.load) {
        case LD_C16: return launch_one<F, LD_C16, ST_C16, false>(p, s);
        case LD_C16_CONJ_MULK: return launch_one<F, LD_C16_CONJ_MULK, ST_C16, false>(p, s);
        case LD_C32_CONJ: return launch_one<F, LD_C32_CONJ, ST_C16, false>(p, s);
        case LD_REAL: return launch_one<F, LD_REAL, ST_C16, false>(p, s);
        case LD_REAL_PAIR: return launch_one<F, LD_REAL_PAIR, ST_C16, false>(p, s);
        case LD_CPLX: return launch_one<F, LD_CPLX, ST_C16, false>(p, s);
        default: break;
        }
    }
    return fail(MONARCH_EINVAL, "internal: pass modes %d/%d not built for the MFMA path", p.load, p.store);
}

}  // namespace fpm

bool fft_mfma_supported(int N, const int *factors, int nf, monarch_dtype dt)
{
    if (dt != MONARCH_BF16 || nf < 2 || nf > 3 || N > (1 << 24)) return false;
    for (int q = 0; q < nf; ++q)
        if (factors[q] != 16 && factors[q] != 32 && factors[q] != 64 && factors[q] != 128) return false;
    return true;
}

int launch_fft_pass_mfma(const FftPass &p, hipStream_t s)
{
    if (p.rows == 0) return MONARCH_OK;
    // shapes the kernel's indexing relies on
    const bool last = p.S == 1;
    if (last ? (p.O % 16 != 0 || p.load != LD_C16) : (p.S % 16 != 0 || p.store != ST_C16))
        return fail(MONARCH_EINVAL, "internal: MFMA pass geometry O=%d f=%d S=%d load=%d store=%d", p.O, p.f, p.S, p.load, p.store);
    if ((int64_t)p.O * p.f * p.S != p.N) return fail(MONARCH_EINVAL, "internal: pass geometry does not multiply to N");
    switch (p.f) {
    case 16: return fpm::launch_f<16>(p, s);
    case 32: return fpm::launch_f<32>(p, s);
    case 64: return fpm::launch_f<64>(p, s);
    case 128: return fpm::launch_f<128>(p, s);
    default: return fail(MONARCH_EINVAL, "internal: factor %d not built for the MFMA path", p.f);
    }
}

}  // namespace monarch
