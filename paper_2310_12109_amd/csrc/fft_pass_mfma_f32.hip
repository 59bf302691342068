// One block-diagonal factor of the Monarch DFT (appendix, DFT corollary) on the fp32 matrix cores
// (16x16x4 MFMA: fp32 products, fp32 accumulation), for fp32 transforms whose factor is 16, 32, 64 or 128.
//
// Same decomposition as the bf16 pass: the row is viewed as [O][f][S], the middle digit is
// contracted with F_f, the result is multiplied by omega_(fS)^(j s).  A = F_f: every entry is one
// of the f roots of unity, kept exact in a 1 KB LDS table and fetched by (j c) mod f; B = 16
// columns by f contraction values in registers, loaded straight from global memory; rows travel
// between passes as complex fp32.  Four real MFMA chains per output tile (two for real input or
// real output).  Twiddles: four exact seeds per lane (sincospif) stepped by omega^(16 s) per row tile.
#include "kernels.h"

namespace monarch {

typedef __attribute__((ext_vector_type(4))) float f32x4;

namespace fpf {

__device__ __forceinline__ f32x4 mfma(float a, float b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// first of the two real rows packed as (re, im) in complex row rc; the second is pair_stride rows on
__device__ __forceinline__ int64_t pair_first_row(const FftPass &p, int64_t rc)
{
    return rc + (rc / p.pair_stride) * p.pair_stride;   // (rc / ps) * 2 ps + rc % ps
}

template <int LOAD>
__device__ __forceinline__ float2 load_value(const FftPass &p, int64_t rc, int pos)
{
    if constexpr (LOAD == LD_C32) {
        return ((const float2 *)p.in)[rc * p.N + pos];
    } else if constexpr (LOAD == LD_C32_CONJ) {
        const float2 v = ((const float2 *)p.in)[rc * p.N + pos];
        return make_float2(v.x, -v.y);
    } else if constexpr (LOAD == LD_CPLX) {
        return ((const float2 *)p.in)[rc * p.N + pos];
    } else if constexpr (LOAD == LD_C32_CONJ_MULK) {
        const float2 v = ((const float2 *)p.in)[rc * p.N + pos];
        const float2 m = cmul(v, p.kf[(rc % p.H) * (int64_t)p.N + pos]);
        return make_float2(m.x, -m.y);
    } else if constexpr (LOAD == LD_REAL) {
        const bool ok = pos < p.n_valid;
        const int64_t at = rc * p.n_valid + (ok ? pos : 0);
        float v = ((const float *)p.in)[at];
        if (p.gate) v *= ((const float *)p.gate)[at];
        return make_float2(ok ? v : 0.0f, 0.0f);
    } else {  // LD_REAL_PAIR
        const bool ok = pos < p.n_valid;
        const int64_t ra = pair_first_row(p, rc);
        const bool okb = ok && ra + p.pair_stride < p.real_rows;
        const int64_t at = ra * p.n_valid + (ok ? pos : 0);
        const int64_t bt = okb ? at + (int64_t)p.pair_stride * p.n_valid : at;
        float va = ((const float *)p.in)[at], vb = ((const float *)p.in)[bt];
        if (p.gate) {
            va *= ((const float *)p.gate)[at];
            vb *= ((const float *)p.gate)[bt];
        }
        return make_float2(ok ? va : 0.0f, okb ? vb : 0.0f);
    }
}

// Contraction value of lane group kg in k-step ks.  Strided columns: c = 4 ks + kg, so k-steps wholly
// inside the zero padding can be skipped.  Last pass: c = kg f/4 + ks, so a lane reads one contiguous run.
template <int F, bool CONTIG>
__device__ __forceinline__ int c_of(int ks, int kg)
{
    return CONTIG ? kg * (F / 4) + ks : 4 * ks + kg;
}

template <int F, int LOAD, int STORE, bool CONTIG>
__global__ __launch_bounds__(256, 2) void fft_pass_f32_kernel(const FftPass p)
{
    constexpr int JT = F / 16, KS = F / 4;
    constexpr bool REAL_IN = LOAD == LD_REAL || LOAD == LD_REAL_PAIR;
    constexpr bool REAL_OUT = STORE == ST_REAL_SCALE_GATE || STORE == ST_REAL_PAIR;
    constexpr bool REAL_B = LOAD == LD_REAL;               // imaginary part of the input is zero
    constexpr bool REAL_D = STORE == ST_REAL_SCALE_GATE;   // only the real part is kept
    __shared__ float2 roots[F];
    for (int e = threadIdx.x; e < F; e += 256) roots[e] = omega(e, F);
    __syncthreads();

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63, l16 = lane & 15, kg = lane >> 4;
    const int S = p.S, O = p.O;
    const int tiles_per_unit = (CONTIG ? O : S) / 16;   // unit: a row (CONTIG) or one (row, o)
    const int64_t ntiles = p.rows * (CONTIG ? 1 : O) * tiles_per_unit;
    const float inv_fs = 2.0f / (float)((int64_t)F * S);

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

        // ---- B operands
        float br[KS], bi[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bool live = !REAL_IN || (int64_t)4 * ks * S < p.n_valid;   // wave-uniform
            float2 v = make_float2(0.0f, 0.0f);
            if (live) v = load_value<LOAD>(p, rc, base + c_of<F, CONTIG>(ks, kg) * (CONTIG ? 1 : S));
            br[ks] = v.x;
            bi[ks] = v.y;
        }

        // ---- twiddle seeds: omega_(fS)^(j s) for j = 4 kg + r, stepped by omega_(fS)^(16 s) per row tile
        float2 tw[4], step;
        if constexpr (!CONTIG) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float sn, cs;
                sincospif((float)((4 * kg + r) * col) * inv_fs, &sn, &cs);   // exact argument: j s < f S <= 2^24
                tw[r] = make_float2(cs, sn);
            }
            float sn, cs;
            sincospif((float)(16 * col) * inv_fs, &sn, &cs);
            step = make_float2(cs, sn);
        }

#pragma unroll 1
        for (int jt = 0; jt < JT; ++jt) {
            const bool wanted = !REAL_OUT || (int64_t)16 * jt * O < p.n_valid;
            if (wanted) {
                f32x4 dr = {0, 0, 0, 0}, di = {0, 0, 0, 0};
                const int j = 16 * jt + l16;   // A operand row of this lane
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const bool live = !REAL_IN || (int64_t)4 * ks * S < p.n_valid;
                    if (live) {
                        const float2 a = roots[(j * c_of<F, CONTIG>(ks, kg)) & (F - 1)];
                        dr = mfma(a.x, br[ks], dr);
                        if constexpr (!REAL_B) dr = mfma(-a.y, bi[ks], dr);
                        if constexpr (!REAL_D) {
                            di = mfma(a.y, br[ks], di);
                            if constexpr (!REAL_B) di = mfma(a.x, bi[ks], di);
                        }
                    }
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int jo = 16 * jt + 4 * kg + r;
                    float2 z = make_float2(dr[r], di[r]);
                    if constexpr (!CONTIG) {   // ST_C32
                        z = cmul(z, tw[r]);
                        ((float2 *)p.out)[rc * p.N + base + (int64_t)jo * S] = z;
                    } else {
                        const int m = jo * O + col;   // natural output index
                        if constexpr (STORE == ST_C32_NATURAL) {
                            ((float2 *)p.out)[rc * p.N + m] = z;
                        } else if constexpr (STORE == ST_CPLX_CONJ_SCALE) {
                            ((float2 *)p.out)[rc * p.N + m] = make_float2(z.x * p.scale, -z.y * p.scale);
                        } else if constexpr (STORE == ST_REAL_SCALE_GATE) {
                            if (m < p.n_valid) {
                                const int64_t at = rc * p.n_valid + m;
                                float v = z.x * p.scale;
                                if (p.gate) v *= ((const float *)p.gate)[at];
                                ((float *)p.out)[at] = v;
                            }
                        } else {   // ST_REAL_PAIR: F^-1 = conj(F conj(.)) / N, so the second row is -Im
                            if (m < p.n_valid) {
                                const int64_t ra = pair_first_row(p, rc);
                                const int64_t at = ra * p.n_valid + m, bt = at + (int64_t)p.pair_stride * p.n_valid;
                                const bool hasb = ra + p.pair_stride < p.real_rows;
                                float va = z.x * p.scale, vb = -z.y * p.scale;
                                if (p.gate) {
                                    va *= ((const float *)p.gate)[at];
                                    if (hasb) vb *= ((const float *)p.gate)[bt];
                                }
                                ((float *)p.out)[at] = va;
                                if (hasb) ((float *)p.out)[bt] = vb;
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
    int dev = 0, ncu = 0;
    MONARCH_HIP_CHECK(hipGetDevice(&dev));
    MONARCH_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
    const int64_t ntiles = p.rows * (int64_t)p.N / F / 16;
    int64_t grid = (ntiles + 3) / 4;
    const int64_t cap = (int64_t)ncu * 4;
    if (grid > cap) grid = cap;
    hipLaunchKernelGGL((fft_pass_f32_kernel<F, LOAD, STORE, CONTIG>), dim3((unsigned)grid), dim3(256), 0, s, p);
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

template <int F>
static int launch_f(const FftPass &p, hipStream_t s)
{
    if (p.S == 1) {
        switch (p.store) {
        case ST_C32_NATURAL: return launch_one<F, LD_C32, ST_C32_NATURAL, true>(p, s);
        case ST_CPLX_CONJ_SCALE: return launch_one<F, LD_C32, ST_CPLX_CONJ_SCALE, true>(p, s);
        case ST_REAL_SCALE_GATE: return launch_one<F, LD_C32, ST_REAL_SCALE_GATE, true>(p, s);
        case ST_REAL_PAIR: return launch_one<F, LD_C32, ST_REAL_PAIR, true>(p, s);
        default: break;
        }
    } else {
        switch (p.load) {
        case LD_C32: return launch_one<F, LD_C32, ST_C32, false>(p, s);
        case LD_C32_CONJ_MULK: return launch_one<F, LD_C32_CONJ_MULK, ST_C32, false>(p, s);
        case LD_C32_CONJ: return launch_one<F, LD_C32_CONJ, ST_C32, false>(p, s);
        case LD_REAL: return launch_one<F, LD_REAL, ST_C32, false>(p, s);
        case LD_REAL_PAIR: return launch_one<F, LD_REAL_PAIR, ST_C32, false>(p, s);
        case LD_CPLX: return launch_one<F, LD_CPLX, ST_C32, false>(p, s);
        default: break;
        }
    }
    return fail(MONARCH_EINVAL, "internal: pass modes %d/%d not built for the fp32 MFMA path", p.load, p.store);
}

}  // namespace fpf

bool fft_mfma_f32_supported(int N, const int *factors, int nf, monarch_dtype dt)
{
    if (dt != MONARCH_F32 || nf < 2 || nf > 3 || N > (1 << 24)) return false;
    for (int q = 0; q < nf; ++q)
        if (factors[q] != 16 && factors[q] != 32 && factors[q] != 64 && factors[q] != 128) return false;
    return true;
}

int launch_fft_pass_mfma_f32(const FftPass &p, hipStream_t s)
{
    if (p.rows == 0) return MONARCH_OK;
    const bool last = p.S == 1;
    if (last ? (p.O % 16 != 0 || p.load != LD_C32) : (p.S % 16 != 0 || p.store != ST_C32))
        return fail(MONARCH_EINVAL, "internal: fp32 MFMA pass geometry O=%d f=%d S=%d load=%d store=%d", p.O, p.f, p.S, p.load, p.store);
    if ((int64_t)p.O * p.f * p.S != p.N) return fail(MONARCH_EINVAL, "internal: pass geometry does not multiply to N");
    switch (p.f) {
    case 16: return fpf::launch_f<16>(p, s);
    case 32: return fpf::launch_f<32>(p, s);
    case 64: return fpf::launch_f<64>(p, s);
    case 128: return fpf::launch_f<128>(p, s);
    default: return fail(MONARCH_EINVAL, "internal: factor %d not built for the fp32 MFMA path", p.f);
    }
}

}  // namespace monarch
