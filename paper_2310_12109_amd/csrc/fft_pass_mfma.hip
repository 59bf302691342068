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
// Column tiles: when S >= 16 a tile is 16 or 32 consecutive s (loads and stores are 16-lane
// contiguous runs of one or two elements per lane); the last pass (S = 1) takes 16 or 32 consecutive
// *natural output* positions, so that its stores are contiguous, and each lane reads its own
// contiguous run of f inputs per column.
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

// First of the two real rows packed as (re, im) in complex row rc; the second is pair_stride rows on.
__device__ __forceinline__ int64_t pair_first_row(const FftPass &p, int64_t rc)
{
    // 32-bit arithmetic (row counts stay far below 2^31), a shift when the stride is a power of two: a 64-bit
    // division costs a wave some 150 scalar instructions, as much as the rest of a tile's index arithmetic
    const uint32_t r = (uint32_t)rc, ps = (uint32_t)p.pair_stride;
    const uint32_t q = (ps & (ps - 1)) == 0 ? r >> __builtin_ctz(ps) : r / ps;
    return (int64_t)r + (int64_t)q * ps;   // (rc / ps) * 2 ps + rc % ps
}

// NT adjacent 32-bit words / bf16 values with one access (NT = 1 or 2; the callers guarantee the
// natural alignment of the wider access).
template <int NT>
__device__ __forceinline__ void load_words(const uint32_t *src, uint32_t (&w)[NT])
{
    if constexpr (NT == 1) w[0] = src[0];
    else {
        const uint2 v = *(const uint2 *)src;
        w[0] = v.x;
        w[1] = v.y;
    }
}
template <int NT>
__device__ __forceinline__ void store_words(uint32_t *dst, const uint32_t (&w)[NT])
{
    if constexpr (NT == 1) dst[0] = w[0];
    else *(uint2 *)dst = make_uint2(w[0], w[1]);
}
template <int NT>
__device__ __forceinline__ void load_bf16s(const bf16_t *src, float (&v)[NT])
{
    if constexpr (NT == 1) v[0] = (float)src[0];
    else {
        const uint32_t w = *(const uint32_t *)src;
        v[0] = lo_f32(w);
        v[1] = hi_f32(w);
    }
}
template <int NT>
__device__ __forceinline__ void store_bf16s(bf16_t *dst, const float (&v)[NT])
{
    if constexpr (NT == 1) dst[0] = (bf16_t)v[0];
    else *(uint32_t *)dst = pack2(v[0], v[1]);
}

// NT adjacent input elements as complex numbers, with the load mode's conjugation / gating /
// spectrum product applied.  pos is the position of the first one inside the row.
template <int LOAD, int NT>
__device__ __forceinline__ void load_values(const FftPass &p, int64_t rc, int pos, float (&re)[NT], float (&im)[NT])
{
    typedef bf16_t T;
    if constexpr (LOAD == LD_C32_CONJ) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {   // adjacent 8-byte loads: merged by the compiler
            const float2 v = ((const float2 *)p.in)[rc * p.N + pos + t];
            re[t] = v.x;
            im[t] = -v.y;
        }
    } else if constexpr (LOAD == LD_CPLX) {
        uint32_t w[NT];
        load_words<NT>((const uint32_t *)p.in + rc * p.N + pos, w);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            re[t] = lo_f32(w[t]);
            im[t] = hi_f32(w[t]);
        }
    } else if constexpr (LOAD == LD_C16_CONJ_MULK) {
        uint32_t w[NT];
        load_words<NT>((const uint32_t *)p.in + rc * p.N + pos, w);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const float2 k = p.kf[(int64_t)((uint32_t)rc % (uint32_t)p.H) * p.N + pos + t];
            const float2 m = cmul(make_float2(lo_f32(w[t]), hi_f32(w[t])), k);
            re[t] = m.x;
            im[t] = -m.y;
        }
    } else if constexpr (LOAD == LD_C16_HERM_MULK) {
        // z = a + i b with a, b real: A[m] = (Z[m] + conj Z[N-m]) / 2, B[m] = (Z[m] - conj Z[N-m]) / 2i; same for
        // the kernels.  Wanted: conj(A Ka + i B Kb), the spectrum of conv(a, ka) + i conv(b, kb), conjugated.
        const uint32_t *zrow = (const uint32_t *)p.in + rc * p.N, *krow = (const uint32_t *)p.kf + rc * p.N;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int m = pos + t, mr = (p.N - m) & (p.N - 1);   // N is a power of two here
            const uint32_t z0 = zrow[m], z1 = zrow[mr], k0 = krow[m], k1 = krow[mr];
            const float2 za = make_float2(lo_f32(z0), hi_f32(z0)), zb = make_float2(lo_f32(z1), -hi_f32(z1));
            const float2 ka = make_float2(lo_f32(k0), hi_f32(k0)), kb = make_float2(lo_f32(k1), -hi_f32(k1));
            const float2 A = make_float2(0.5f * (za.x + zb.x), 0.5f * (za.y + zb.y));
            const float2 Bv = make_float2(0.5f * (za.y - zb.y), -0.5f * (za.x - zb.x));   // (za - zb) / 2i
            const float2 Ka = make_float2(0.5f * (ka.x + kb.x), 0.5f * (ka.y + kb.y));
            const float2 Kb = make_float2(0.5f * (ka.y - kb.y), -0.5f * (ka.x - kb.x));
            const float2 pa = cmul(A, Ka), pb = cmul(Bv, Kb);
            re[t] = pa.x - pb.y;          // Re(pa + i pb)
            im[t] = -(pa.y + pb.x);       // -Im(pa + i pb)
        }
    } else if constexpr (LOAD == LD_REAL) {
        const bool ok = pos < p.n_valid;   // NT = 2: pos and n_valid are even
        const int64_t at = rc * p.n_valid + (ok ? pos : 0);
        float v[NT], g[NT];
        load_bf16s<NT>((const T *)p.in + at, v);
        if (p.gate) {
            load_bf16s<NT>((const T *)p.gate + at, g);
#pragma unroll
            for (int t = 0; t < NT; ++t) v[t] *= g[t];
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            re[t] = ok ? v[t] : 0.0f;
            im[t] = 0.0f;
        }
    } else {  // LD_REAL_PAIR
        const bool ok = pos < p.n_valid;
        const int64_t ra = pair_first_row(p, rc);
        const bool okb = ok && ra + p.pair_stride < p.real_rows;
        const int64_t at = ra * p.n_valid + (ok ? pos : 0);
        const int64_t bt = okb ? at + (int64_t)p.pair_stride * p.n_valid : at;
        float va[NT], vb[NT], ga[NT], gb[NT];
        load_bf16s<NT>((const T *)p.in + at, va);
        load_bf16s<NT>((const T *)p.in + bt, vb);
        if (p.gate) {
            load_bf16s<NT>((const T *)p.gate + at, ga);
            load_bf16s<NT>((const T *)p.gate + bt, gb);
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                va[t] *= ga[t];
                vb[t] *= gb[t];
            }
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            re[t] = ok ? va[t] : 0.0f;
            im[t] = okb ? vb[t] : 0.0f;
        }
    }
}

// The operands of F_f for the matrix instruction, built once per workgroup: entry [jt][ks][re, im][lane], where
// lane (row l16, group kg) of row tile jt and k-step ks holds F[16 jt + l16][32 ks + 8 kg + e], e < 8, as bf16 pairs.
template <int F, int THREADS>
__device__ __forceinline__ void build_ftab(u32x4 *ftab)
{
    constexpr int JT = F / 16, KS = (F + 31) / 32;
    __shared__ float2 roots[F];
    for (int e = threadIdx.x; e < F; e += THREADS) roots[e] = omega(e, F);
    __syncthreads();
    for (int idx = threadIdx.x; idx < JT * KS * 64; idx += THREADS) {
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
}

// NT column tiles per wave: lane l16 owns the adjacent columns col0 + t, t < NT, so that NT = 2
// doubles the width of every global access and halves the operand reads from LDS.
template <int F, int LOAD, int STORE, bool CONTIG, int NT>
__global__ __launch_bounds__(F == 128 ? 512 : 256, F == 128 ? 4 : 2) void fft_pass_mfma_kernel(const FftPass p)
{
    constexpr int JT = F / 16, KS = (F + 31) / 32;
    constexpr int THREADS = F == 128 ? 512 : 256, WAVES = THREADS / 64;   // the 64 KB table of f = 128 is shared by 8 waves
    constexpr int COLS = 16 * NT;
    constexpr bool REAL_IN = LOAD == LD_REAL || LOAD == LD_REAL_PAIR;
    constexpr bool REAL_OUT = STORE == ST_REAL_SCALE_GATE || STORE == ST_REAL_PAIR;
    constexpr bool REAL_B = LOAD == LD_REAL;                   // imaginary part of the input is zero
    constexpr bool REAL_D = STORE == ST_REAL_SCALE_GATE;       // only the real part is kept
    extern __shared__ __attribute__((aligned(16))) u32x4 ftab[];   // [JT][KS][re, im][lane]
    build_ftab<F, THREADS>(ftab);

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63, l16 = lane & 15, kg = lane >> 4;
    const int S = p.S, O = p.O;
    const int tiles_per_unit = (CONTIG ? O : S) / COLS;           // unit: a row (CONTIG) or one (row, o)
    // O and S are products of the factors 16 .. 128, powers of two: the index arithmetic below is shifts
    const int tpu_shift = __builtin_ctz(tiles_per_unit), o_shift = __builtin_ctz(O);
    const int64_t ntiles = p.rows * (CONTIG ? 1 : O) * tiles_per_unit;
    const float inv_fs = 1.0f / (float)((int64_t)F * S);

    for (int64_t tile = (int64_t)blockIdx.x * WAVES + wave; tile < ntiles; tile += (int64_t)gridDim.x * WAVES) {
        int64_t rc;
        int col0;       // first of this lane's columns: s (S >= 16) or natural low index rho (S == 1)
        int base[NT];   // CONTIG: position of (o(col0 + t), c = 0); else base[0]: position of (o, c = 0, s = col0)
        if constexpr (CONTIG) {
            rc = tile >> tpu_shift;
            col0 = (int)(tile - (rc << tpu_shift)) * COLS + NT * l16;
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                int o = col0 + t;   // two factors: the digit itself; three: swap the two digits already produced
                if (p.nf == 3) o = ((col0 + t) % p.factors[0]) * p.factors[1] + (col0 + t) / p.factors[0];
                base[t] = o * F;
            }
        } else {
            const int64_t unit = tile >> tpu_shift;
            col0 = (int)(tile - (unit << tpu_shift)) * COLS + NT * l16;
            rc = unit >> o_shift;
            base[0] = (int)(unit - (rc << o_shift)) * F * S + col0;
        }

        // ---- B operands: k-step ks, slot e  <->  c = 32 ks + 8 kg + e
        u32x4 br[NT][KS], bi[NT][KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int c0 = 32 * ks + 8 * kg;
            if constexpr (CONTIG) {   // packed bf16 pairs, 8 consecutive elements per lane and column
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    u32x4 w0 = {0, 0, 0, 0}, w1 = w0;
                    if (c0 < F) {
                        const u32x4 *src = (const u32x4 *)((const uint32_t *)p.in + rc * p.N + base[t] + c0);
                        w0 = src[0];
                        w1 = src[1];
                    }
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        br[t][ks][h] = (w0[2 * h] & 0xffffu) | (w0[2 * h + 1] << 16);
                        bi[t][ks][h] = (w0[2 * h] >> 16) | (w0[2 * h + 1] & 0xffff0000u);
                        br[t][ks][2 + h] = (w1[2 * h] & 0xffffu) | (w1[2 * h + 1] << 16);
                        bi[t][ks][2 + h] = (w1[2 * h] >> 16) | (w1[2 * h + 1] & 0xffff0000u);
                    }
                }
            } else if constexpr (LOAD == LD_C16) {
                uint32_t w[8][NT];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const bool ok = c0 + e < F;
                    load_words<NT>((const uint32_t *)p.in + rc * p.N + base[0] + (ok ? (c0 + e) * S : 0), w[e]);
#pragma unroll
                    for (int t = 0; t < NT; ++t) w[e][t] = ok ? w[e][t] : 0u;
                }
#pragma unroll
                for (int t = 0; t < NT; ++t)
#pragma unroll
                    for (int h = 0; h < 4; ++h) {
                        br[t][ks][h] = (w[2 * h][t] & 0xffffu) | (w[2 * h + 1][t] << 16);
                        bi[t][ks][h] = (w[2 * h][t] >> 16) | (w[2 * h + 1][t] & 0xffff0000u);
                    }
            } else {
                // inputs past n_valid are zero: a k-step wholly past it is skipped (wave-uniform)
                const bool live = !REAL_IN || (int64_t)32 * ks * S < p.n_valid;
                float vr[8][NT], vi[8][NT];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
#pragma unroll
                    for (int t = 0; t < NT; ++t) vr[e][t] = vi[e][t] = 0.0f;
                    if (live) {
                        const bool ok = c0 + e < F;
                        float re[NT], im[NT];
                        load_values<LOAD, NT>(p, rc, base[0] + (ok ? (c0 + e) * S : 0), re, im);
#pragma unroll
                        for (int t = 0; t < NT; ++t) {
                            vr[e][t] = ok ? re[t] : 0.0f;
                            vi[e][t] = ok ? im[t] : 0.0f;
                        }
                    }
                }
#pragma unroll
                for (int t = 0; t < NT; ++t)
#pragma unroll
                    for (int h = 0; h < 4; ++h) {
                        br[t][ks][h] = pack2(vr[2 * h][t], vr[2 * h + 1][t]);
                        bi[t][ks][h] = pack2(vi[2 * h][t], vi[2 * h + 1][t]);
                    }
            }
        }

        // ---- twiddle seeds: omega_(fS)^(j s) for j = 4 kg + r, stepped by omega_(fS)^(16 s) per row tile
        float2 tw[NT][4], step[NT];
        if constexpr (!CONTIG) {
#pragma unroll
            for (int t = 0; t < NT; ++t) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float rev = (float)((4 * kg + r) * (col0 + t)) * inv_fs;   // exact: j s < f S <= 2^24
                    tw[t][r] = make_float2(__builtin_amdgcn_cosf(rev), __builtin_amdgcn_sinf(rev));
                }
                const float rev = (float)(16 * (col0 + t)) * inv_fs;
                step[t] = make_float2(__builtin_amdgcn_cosf(rev), __builtin_amdgcn_sinf(rev));
            }
        }

        // ---- row tiles of the output digit j (kept as a loop: unrolled, the operand reads of all
        // tiles are hoisted and the register file overflows)
#pragma unroll 1
        for (int jt = 0; jt < JT; ++jt) {
            const bool wanted = !REAL_OUT || (int64_t)16 * jt * (CONTIG ? O : S) < p.n_valid;
            if (wanted) {
                f32x4 dr[NT], di[NT];
#pragma unroll
                for (int t = 0; t < NT; ++t) dr[t] = di[t] = f32x4{0, 0, 0, 0};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const bool live = !REAL_IN || (int64_t)32 * ks * S < p.n_valid;
                    if (live) {
                        const u32x4 ar = ftab[(jt * KS + ks) * 128 + lane], ai = ftab[(jt * KS + ks) * 128 + 64 + lane];
                        const u32x4 nai = ai ^ 0x80008000u;
#pragma unroll
                        for (int t = 0; t < NT; ++t) {
                            dr[t] = mfma(ar, br[t][ks], dr[t]);
                            if constexpr (!REAL_B) dr[t] = mfma(nai, bi[t][ks], dr[t]);
                            if constexpr (!REAL_D) {
                                di[t] = mfma(ai, br[t][ks], di[t]);
                                if constexpr (!REAL_B) di[t] = mfma(ar, bi[t][ks], di[t]);
                            }
                        }
                    }
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int j = 16 * jt + 4 * kg + r;
                    float zr[NT], zi[NT];
#pragma unroll
                    for (int t = 0; t < NT; ++t) {
                        zr[t] = dr[t][r];
                        zi[t] = di[t][r];
                    }
                    if constexpr (!CONTIG && !REAL_OUT) {   // ST_C16
                        uint32_t w[NT];
#pragma unroll
                        for (int t = 0; t < NT; ++t) {
                            const float2 z = cmul(make_float2(zr[t], zi[t]), tw[t][r]);
                            w[t] = pack2(z.x, z.y);
                        }
                        store_words<NT>((uint32_t *)p.out + rc * p.N + base[0] + (int64_t)j * S, w);
                    } else if constexpr (!CONTIG) {
                        // Last pass of an inverse whose factors run in the opposite order (the first digit is
                        // contracted last, O = 1): no twiddle follows, outputs are in time order j S + s.
                        const int m = j * S + col0;
                        if (m < p.n_valid) {
                            const int64_t ra = STORE == ST_REAL_PAIR ? pair_first_row(p, rc) : rc;
                            const int64_t at = ra * p.n_valid + m, bt = at + (int64_t)p.pair_stride * p.n_valid;
                            const bool hasb = STORE == ST_REAL_PAIR && ra + p.pair_stride < p.real_rows;
                            float va[NT], vb[NT], g[NT];
#pragma unroll
                            for (int t = 0; t < NT; ++t) {
                                va[t] = zr[t] * p.scale;
                                vb[t] = -zi[t] * p.scale;
                            }
                            if (p.gate) {
                                load_bf16s<NT>((const bf16_t *)p.gate + at, g);
#pragma unroll
                                for (int t = 0; t < NT; ++t) va[t] *= g[t];
                            }
                            store_bf16s<NT>((bf16_t *)p.out + at, va);
                            if (hasb) {
                                if (p.gate) {
                                    load_bf16s<NT>((const bf16_t *)p.gate + bt, g);
#pragma unroll
                                    for (int t = 0; t < NT; ++t) vb[t] *= g[t];
                                }
                                store_bf16s<NT>((bf16_t *)p.out + bt, vb);
                            }
                        }
                    } else {
                        const int m = j * O + col0;   // natural output index of the first column
                        if constexpr (STORE == ST_C32_NATURAL) {
#pragma unroll
                            for (int t = 0; t < NT; ++t) ((float2 *)p.out)[rc * p.N + m + t] = make_float2(zr[t], zi[t]);
                        } else if constexpr (STORE == ST_C16_NATURAL || STORE == ST_CPLX_CONJ_SCALE) {
                            uint32_t w[NT];
#pragma unroll
                            for (int t = 0; t < NT; ++t)
                                w[t] = STORE == ST_C16_NATURAL ? pack2(zr[t], zi[t]) : pack2(zr[t] * p.scale, -zi[t] * p.scale);
                            store_words<NT>((uint32_t *)p.out + rc * p.N + m, w);
                        } else if constexpr (STORE == ST_REAL_SCALE_GATE) {
                            if (m < p.n_valid) {   // NT = 2: m and n_valid are even
                                const int64_t at = rc * p.n_valid + m;
                                float v[NT], g[NT];
#pragma unroll
                                for (int t = 0; t < NT; ++t) v[t] = zr[t] * p.scale;
                                if (p.gate) {
                                    load_bf16s<NT>((const bf16_t *)p.gate + at, g);
#pragma unroll
                                    for (int t = 0; t < NT; ++t) v[t] *= g[t];
                                }
                                store_bf16s<NT>((bf16_t *)p.out + at, v);
                            }
                        } else {   // ST_REAL_PAIR: F^-1 = conj(F conj(.)) / N, so the second row is -Im
                            if (m < p.n_valid) {
                                const int64_t ra = pair_first_row(p, rc);
                                const int64_t at = ra * p.n_valid + m, bt = at + (int64_t)p.pair_stride * p.n_valid;
                                const bool hasb = ra + p.pair_stride < p.real_rows;
                                float va[NT], vb[NT], g[NT];
#pragma unroll
                                for (int t = 0; t < NT; ++t) {
                                    va[t] = zr[t] * p.scale;
                                    vb[t] = -zi[t] * p.scale;
                                }
                                if (p.gate) {
                                    load_bf16s<NT>((const bf16_t *)p.gate + at, g);
#pragma unroll
                                    for (int t = 0; t < NT; ++t) va[t] *= g[t];
                                }
                                store_bf16s<NT>((bf16_t *)p.out + at, va);
                                if (hasb) {
                                    if (p.gate) {
                                        load_bf16s<NT>((const bf16_t *)p.gate + bt, g);
#pragma unroll
                                        for (int t = 0; t < NT; ++t) vb[t] *= g[t];
                                    }
                                    store_bf16s<NT>((bf16_t *)p.out + bt, vb);
                                }
                            }
                        }
                    }
                }
            }
            if constexpr (!CONTIG) {
#pragma unroll
                for (int t = 0; t < NT; ++t)
#pragma unroll
                    for (int r = 0; r < 4; ++r) tw[t][r] = cmul(tw[t][r], step[t]);
            }
        }
    }
}

// ---- passes whose real rows move in 16-byte pieces --------------------------------------------
//
// A wave of the kernel above touches a real bf16 row 64 bytes at a time (32 columns), four rows per access:
// half cache lines, which the memory system serves at a fraction of its rate.  The two kernels below take 128
// columns per workgroup; the threads read or write the real rows in 16-byte pieces (256 contiguous bytes per
// row) and the waves exchange operands and results through LDS.  They cover the first pass of a forward
// transform of real rows (rows_in: O = 1, ST_C16) and the last pass of an inverse that ends in time order
// (rows_out: O = 1, LD_C16, S > 1), for S a multiple of 128 and rows of a multiple of 8 elements.

constexpr int RB_COLS = 128;          // columns of a workgroup's block: 32 per wave, 2 per lane
constexpr int RB_PITCH = RB_COLS + 8; // words per LDS row: the four row groups of an access fall on different banks

// First pass.  LDS holds, per plane (real parts; PAIR: imaginary parts = the second real row), the block as
// [row pair][column] words of two bf16 (rows 2 rp, 2 rp + 1): the matrix instruction's operand pairs.
// LS: k-steps (32 rows) that hold input; the rows past n_valid are zero and never read.
template <int F, bool PAIR, int LS>
__global__ __launch_bounds__(256, 2) void fft_pass_rows_in_kernel(const FftPass p)
{
    constexpr int JT = F / 16, KS = (F + 31) / 32, THREADS = 256, NP = PAIR ? 2 : 1;
    static_assert(LS >= 1 && LS <= KS, "live k-steps");
    extern __shared__ __attribute__((aligned(16))) u32x4 ftab[];
    uint32_t *plane = reinterpret_cast<uint32_t *>(ftab + JT * KS * 128);   // [NP][16 LS][RB_PITCH]
    build_ftab<F, THREADS>(ftab);

    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, kg = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int S = p.S, blocks_per_row = S / RB_COLS, bpr_shift = __builtin_ctz(blocks_per_row);   // S is a power of two
    const int64_t nblocks = p.rows * blocks_per_row;
    const float inv_fs = 1.0f / (float)((int64_t)F * S);
    const bool gated = p.gate != nullptr;
    const bf16_t *in = (const bf16_t *)p.in, *gate = gated ? (const bf16_t *)p.gate : in;
    const int piece = tid & 15, rp0 = tid >> 4;   // this thread's pieces: columns 8 piece .. + 7 of row pairs rp0 + 16 st

    u32x4 val[LS][NP][2], gat[LS][NP][2];   // [k-step][real row][row of the pair]
    auto request = [&](int64_t blk) {
        const int64_t rc = blk >> bpr_shift;
        const int s0 = (int)(blk - (rc << bpr_shift)) * RB_COLS + 8 * piece;
        const int64_t ra = PAIR ? pair_first_row(p, rc) : rc;
        const bool hasb = PAIR && ra + p.pair_stride < p.real_rows;
#pragma unroll
        for (int st = 0; st < LS; ++st)
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int c = 2 * (rp0 + 16 * st) + q, pos = c * S + s0;
                const int64_t at = ra * p.n_valid + (c < F && pos < p.n_valid ? pos : 0);   // past the row: any valid address
                // (real rows are read once per launch: streaming loads)
                val[st][0][q] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(in + at));
                if (gated) gat[st][0][q] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(gate + at));
                if constexpr (PAIR) {
                    const int64_t bt = hasb ? at + (int64_t)p.pair_stride * p.n_valid : at;
                    val[st][1][q] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(in + bt));
                    if (gated) gat[st][1][q] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(gate + bt));
                }
            }
    };
    // rounds the (gated) values to bf16 and writes the pairs of rows 2 rp, 2 rp + 1
    auto deposit = [&](int64_t blk) {
        const int64_t rc = blk >> bpr_shift;
        const int s0 = (int)(blk - (rc << bpr_shift)) * RB_COLS + 8 * piece;
        const int64_t ra = PAIR ? pair_first_row(p, rc) : rc;
        const bool hasb = PAIR && ra + p.pair_stride < p.real_rows;
#pragma unroll
        for (int st = 0; st < LS; ++st) {
            const int rp = rp0 + 16 * st;
            bool ok[2];
#pragma unroll
            for (int q = 0; q < 2; ++q) ok[q] = 2 * rp + q < F && (2 * rp + q) * S + s0 < p.n_valid;
#pragma unroll
            for (int np = 0; np < NP; ++np) {
                u32x4 v[2];
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const bool live = ok[q] && (np == 0 || hasb);
#pragma unroll
                    for (int h = 0; h < 4; ++h) v[q][h] = live ? val[st][np][q][h] : 0u;
                }
                u32x4 w0, w1;   // columns 0..3 and 4..7 of the piece
#pragma unroll
                for (int h = 0; h < 4; ++h) {
                    uint32_t even, odd;   // columns 2 h and 2 h + 1: (row 2 rp, row 2 rp + 1)
                    if (gated) {
                        const uint32_t g0 = gat[st][np][0][h], g1 = gat[st][np][1][h];
                        even = pack2(lo_f32(v[0][h]) * lo_f32(g0), lo_f32(v[1][h]) * lo_f32(g1));
                        odd = pack2(hi_f32(v[0][h]) * hi_f32(g0), hi_f32(v[1][h]) * hi_f32(g1));
                    } else {
                        even = __builtin_amdgcn_perm(v[1][h], v[0][h], 0x05040100u);
                        odd = __builtin_amdgcn_perm(v[1][h], v[0][h], 0x07060302u);
                    }
                    if (h < 2) {
                        w0[2 * h] = even;
                        w0[2 * h + 1] = odd;
                    } else {
                        w1[2 * h - 4] = even;
                        w1[2 * h - 3] = odd;
                    }
                }
                uint32_t *dst = plane + (np * 16 * LS + rp) * RB_PITCH + 8 * piece;
                *reinterpret_cast<u32x4 *>(dst) = w0;
                *reinterpret_cast<u32x4 *>(dst + 4) = w1;
            }
        }
    };

    int64_t blk = blockIdx.x;
    if (blk < nblocks) request(blk);
    for (; blk < nblocks; blk += gridDim.x) {
        deposit(blk);
        __syncthreads();
        if (blk + gridDim.x < nblocks) request(blk + gridDim.x);

        // ---- B operands of this wave's 32 columns: k-step ks, slot pair h  <->  rows 32 ks + 8 kg + 2 h, + 1
        u32x4 br[2][LS], bi[2][PAIR ? LS : 1];
#pragma unroll
        for (int ks = 0; ks < LS; ++ks)
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                const uint32_t *src = plane + (16 * ks + 4 * kg + h) * RB_PITCH + 32 * wave + 2 * l16;
                const uint2 r = *reinterpret_cast<const uint2 *>(src);
                br[0][ks][h] = r.x;
                br[1][ks][h] = r.y;
                if constexpr (PAIR) {
                    const uint2 i = *reinterpret_cast<const uint2 *>(src + 16 * LS * RB_PITCH);
                    bi[0][ks][h] = i.x;
                    bi[1][ks][h] = i.y;
                }
            }
        __syncthreads();   // the planes are free for the next block

        const int64_t rc = blk >> bpr_shift;
        const int col0 = (int)(blk - (rc << bpr_shift)) * RB_COLS + 32 * wave + 2 * l16;
        // twiddle seeds: omega_(fS)^(j s) for j = 4 kg + r, stepped by omega_(fS)^(16 s) per row tile
        float2 tw[2][4], step[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float rev = (float)((4 * kg + r) * (col0 + t)) * inv_fs;   // exact: j s < f S <= 2^24
                tw[t][r] = make_float2(__builtin_amdgcn_cosf(rev), __builtin_amdgcn_sinf(rev));
            }
            const float rev = (float)(16 * (col0 + t)) * inv_fs;
            step[t] = make_float2(__builtin_amdgcn_cosf(rev), __builtin_amdgcn_sinf(rev));
        }
        uint32_t *out = (uint32_t *)p.out + rc * p.N + col0;
#pragma unroll 1
        for (int jt = 0; jt < JT; ++jt) {
            f32x4 dr[2], di[2];
#pragma unroll
            for (int t = 0; t < 2; ++t) dr[t] = di[t] = f32x4{0, 0, 0, 0};
#pragma unroll
            for (int ks = 0; ks < LS; ++ks) {
                const u32x4 ar = ftab[(jt * KS + ks) * 128 + lane], ai = ftab[(jt * KS + ks) * 128 + 64 + lane];
                const u32x4 nai = ai ^ 0x80008000u;
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    dr[t] = mfma(ar, br[t][ks], dr[t]);
                    di[t] = mfma(ai, br[t][ks], di[t]);
                    if constexpr (PAIR) {
                        dr[t] = mfma(nai, bi[t][ks], dr[t]);
                        di[t] = mfma(ar, bi[t][ks], di[t]);
                    }
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int j = 16 * jt + 4 * kg + r;
                uint32_t w[2];
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const float2 z = cmul(make_float2(dr[t][r], di[t][r]), tw[t][r]);
                    w[t] = pack2(z.x, z.y);
                }
                store_words<2>(out + (int64_t)j * S, w);
            }
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r) tw[t][r] = cmul(tw[t][r], step[t]);
        }
    }
}

// Last pass.  The results of a block, scaled, go to LDS as fp32 [real row][j][column]; the threads then take them
// in pieces of 8 columns, apply the output gate and store 16 bytes.  wra: rows j kept, a multiple of 16.
// MAXT: bound on the pieces per thread, NP wra / 16.
template <int F, bool PAIR, int MAXT>
__global__ __launch_bounds__(256, MAXT <= 4 ? 3 : 2) void fft_pass_rows_out_kernel(const FftPass p, const int wra)
{
    constexpr int JT = F / 16, KS = (F + 31) / 32, THREADS = 256, NP = PAIR ? 2 : 1;
    extern __shared__ __attribute__((aligned(16))) u32x4 ftab[];
    float *stage = reinterpret_cast<float *>(ftab + JT * KS * 128);   // [NP][wra][RB_PITCH]
    build_ftab<F, THREADS>(ftab);

    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, kg = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int S = p.S, blocks_per_row = S / RB_COLS, bpr_shift = __builtin_ctz(blocks_per_row);   // S is a power of two
    const int64_t nblocks = p.rows * blocks_per_row;
    const bool gated = p.gate != nullptr;
    const int piece = tid & 15, row0 = tid >> 4;   // this thread's pieces: columns 8 piece .. + 7 of rows row0 + 16 i of [NP][wra]
    const int npieces = NP * wra / 16;             // per thread

    for (int64_t blk = blockIdx.x; blk < nblocks; blk += gridDim.x) {
        const int64_t rc = blk >> bpr_shift;
        const int s0 = (int)(blk - (rc << bpr_shift)) * RB_COLS;
        const int col0 = s0 + 32 * wave + 2 * l16;
        const int64_t ra = PAIR ? pair_first_row(p, rc) : rc;
        const bool hasb = PAIR && ra + p.pair_stride < p.real_rows;

        // ---- B operands: k-step ks, slot e  <->  c = 32 ks + 8 kg + e
        u32x4 br[2][KS], bi[2][KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int c0 = 32 * ks + 8 * kg;
            uint32_t w[8][2];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint2 v = load_stream8((const uint32_t *)p.in + rc * p.N + col0 + (c0 + e) * S);   // (c0 + e < F: F is 32 or 64)
                w[e][0] = v.x;
                w[e][1] = v.y;
            }
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int h = 0; h < 4; ++h) {
                    br[t][ks][h] = __builtin_amdgcn_perm(w[2 * h + 1][t], w[2 * h][t], 0x05040100u);
                    bi[t][ks][h] = __builtin_amdgcn_perm(w[2 * h + 1][t], w[2 * h][t], 0x07060302u);
                }
        }
        // ---- the output gates of this thread's pieces, in flight during the products
        u32x4 gat[MAXT];
        if (gated) {
#pragma unroll
            for (int i = 0; i < MAXT; ++i)
                if (i < npieces) {
                    const int row = row0 + 16 * i, np = row / wra, j = row - np * wra;
                    const int m = j * S + s0 + 8 * piece;
                    const bool ok = m < p.n_valid && (np == 0 || hasb);
                    const int64_t at = (ra + (ok ? np : 0) * (int64_t)p.pair_stride) * p.n_valid + (ok ? m : 0);
                    gat[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>((const bf16_t *)p.gate + at));
                }
        }

#pragma unroll 1
        for (int jt = 0; jt < JT; ++jt) {
            if (16 * jt < wra) {
                f32x4 dr[2], di[2];
#pragma unroll
                for (int t = 0; t < 2; ++t) dr[t] = di[t] = f32x4{0, 0, 0, 0};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const u32x4 ar = ftab[(jt * KS + ks) * 128 + lane], ai = ftab[(jt * KS + ks) * 128 + 64 + lane];
                    const u32x4 nai = ai ^ 0x80008000u;
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        dr[t] = mfma(ar, br[t][ks], dr[t]);
                        dr[t] = mfma(nai, bi[t][ks], dr[t]);
                        if constexpr (PAIR) {
                            di[t] = mfma(ai, br[t][ks], di[t]);
                            di[t] = mfma(ar, bi[t][ks], di[t]);
                        }
                    }
                }
                // F^-1 = conj(F conj(.)) / N: the first real row is the real part, the second minus the imaginary part
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float *dst = stage + (16 * jt + 4 * kg + r) * RB_PITCH + 32 * wave + 2 * l16;
                    *reinterpret_cast<float2 *>(dst) = make_float2(dr[0][r] * p.scale, dr[1][r] * p.scale);
                    if constexpr (PAIR)
                        *reinterpret_cast<float2 *>(dst + wra * RB_PITCH) = make_float2(-di[0][r] * p.scale, -di[1][r] * p.scale);
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < MAXT; ++i)
            if (i < npieces) {
                const int row = row0 + 16 * i, np = row / wra, j = row - np * wra;
                const int m = j * S + s0 + 8 * piece;   // time index of the piece's first element
                if (m < p.n_valid && (np == 0 || hasb)) {
                    const f32x4 a = *reinterpret_cast<const f32x4 *>(stage + row * RB_PITCH + 8 * piece);
                    const f32x4 b = *reinterpret_cast<const f32x4 *>(stage + row * RB_PITCH + 8 * piece + 4);
                    u32x4 w;
                    if (gated) {
                        const u32x4 g = gat[i];
                        w[0] = pack2(a[0] * lo_f32(g[0]), a[1] * hi_f32(g[0]));
                        w[1] = pack2(a[2] * lo_f32(g[1]), a[3] * hi_f32(g[1]));
                        w[2] = pack2(b[0] * lo_f32(g[2]), b[1] * hi_f32(g[2]));
                        w[3] = pack2(b[2] * lo_f32(g[3]), b[3] * hi_f32(g[3]));
                    } else {
                        w[0] = pack2(a[0], a[1]);
                        w[1] = pack2(a[2], a[3]);
                        w[2] = pack2(b[0], b[1]);
                        w[3] = pack2(b[2], b[3]);
                    }
                    const int64_t at = (ra + np * (int64_t)p.pair_stride) * p.n_valid + m;
                    __builtin_nontemporal_store(w, reinterpret_cast<u32x4 *>((bf16_t *)p.out + at));   // y: written once
                }
            }
        __syncthreads();   // the stage is free for the next block
    }
}

// over: workgroups per compute unit beyond those that fit at once (the last pass ran faster with twice as many, shorter
// workgroups: 50 -> 45 us at the 64^3 convolution; the first pass did not)
static int rows_kernel_grid(int64_t nblocks, size_t lds, int over, int *grid)
{
    int dev = 0, ncu = 0;
    MONARCH_HIP_CHECK(hipGetDevice(&dev));
    MONARCH_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
    int per_cu = (int)((160 * 1024) / (lds + 1024));
    per_cu = per_cu < 1 ? 1 : per_cu > 4 ? 4 : per_cu;
    const int64_t cap = (int64_t)ncu * per_cu * over;
    *grid = (int)(nblocks < cap ? nblocks : cap);
    return MONARCH_OK;
}

static bool aligned16(const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15) == 0; }   // (a null gate passes)

// k-steps of the first pass that hold input
static int live_ksteps(const FftPass &p) { return (int)(((int64_t)p.n_valid + 32 * (int64_t)p.S - 1) / (32 * (int64_t)p.S)); }

static bool rows_in_applies(const FftPass &p)
{
    return (p.load == LD_REAL || p.load == LD_REAL_PAIR) && p.store == ST_C16 && p.O == 1 && p.S % RB_COLS == 0 && p.n_valid % 8 == 0 &&
           p.n_valid > 0 && (p.f == 32 || p.f == 64) && p.dt == MONARCH_BF16 && aligned16(p.in) && aligned16(p.gate);
}

template <int F, bool PAIR, int LS>
static int launch_rows_in_ls(const FftPass &p, hipStream_t s)
{
    constexpr int JT = F / 16, KS = (F + 31) / 32;
    const size_t lds = (size_t)JT * KS * 2 * 64 * 16 + (size_t)(PAIR ? 2 : 1) * 16 * LS * RB_PITCH * 4;
    int grid = 0;
    const int rc = rows_kernel_grid(p.rows * (p.S / RB_COLS), lds, 1, &grid);
    if (rc != MONARCH_OK) return rc;
    auto kern = fft_pass_rows_in_kernel<F, PAIR, LS>;
    if (lds > 48 * 1024)
        MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, s, p);
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

template <int F>
static int launch_rows_in(const FftPass &p, hipStream_t s)
{
    const bool pair = p.load == LD_REAL_PAIR;
    const int ls = live_ksteps(p);
    if constexpr (F == 64) {
        if (ls >= 2) return pair ? launch_rows_in_ls<F, true, 2>(p, s) : launch_rows_in_ls<F, false, 2>(p, s);
    }
    return pair ? launch_rows_in_ls<F, true, 1>(p, s) : launch_rows_in_ls<F, false, 1>(p, s);
}

static bool rows_out_applies(const FftPass &p)
{
    return p.load == LD_C16 && (p.store == ST_REAL_PAIR || p.store == ST_REAL_SCALE_GATE) && p.O == 1 && p.S % RB_COLS == 0 &&
           p.n_valid % 8 == 0 && p.n_valid > 0 && (p.f == 32 || p.f == 64) && p.dt == MONARCH_BF16 && aligned16(p.out) && aligned16(p.gate);
}

template <int F, bool PAIR>
static int launch_rows_out_np(const FftPass &p, hipStream_t s)
{
    constexpr int JT = F / 16, KS = (F + 31) / 32;
    int64_t want = ((int64_t)p.n_valid + p.S - 1) / p.S;   // rows j with outputs
    if (want > F) want = F;
    const int wra = (int)((want + 15) / 16) * 16;
    const size_t lds = (size_t)JT * KS * 2 * 64 * 16 + (size_t)(PAIR ? 2 : 1) * wra * RB_PITCH * 4;
    int grid = 0;
    const int rc = rows_kernel_grid(p.rows * (p.S / RB_COLS), lds, 2, &grid);
    if (rc != MONARCH_OK) return rc;
    const int npieces = (PAIR ? 2 : 1) * wra / 16;
    auto kern = npieces <= 2 ? fft_pass_rows_out_kernel<F, PAIR, 2> : npieces <= 4 ? fft_pass_rows_out_kernel<F, PAIR, 4> : fft_pass_rows_out_kernel<F, PAIR, 8>;
    if (lds > 48 * 1024)
        MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, s, p, wra);
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

template <int F>
static int launch_rows_out(const FftPass &p, hipStream_t s)
{
    return p.store == ST_REAL_PAIR ? launch_rows_out_np<F, true>(p, s) : launch_rows_out_np<F, false>(p, s);
}

template <int F, int LOAD, int STORE, bool CONTIG, int NT>
static int launch_nt(const FftPass &p, hipStream_t s)
{
    constexpr int JT = F / 16, KS = (F + 31) / 32;
    const size_t lds = (size_t)JT * KS * 2 * 64 * 16;
    int dev = 0, ncu = 0;
    MONARCH_HIP_CHECK(hipGetDevice(&dev));
    MONARCH_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
    const int64_t ntiles = p.rows * (int64_t)p.N / F / (16 * NT);
    constexpr int THREADS = F == 128 ? 512 : 256, WAVES = THREADS / 64;
    int64_t grid = (ntiles + WAVES - 1) / WAVES;
    const int64_t cap = (int64_t)ncu * (F == 128 ? 2 : 4);   // 16 waves per compute unit
    if (grid > cap) grid = cap;
    auto kern = fft_pass_mfma_kernel<F, LOAD, STORE, CONTIG, NT>;
    if (lds > 48 * 1024)
        MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(THREADS), lds, s, p);
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

// Two column tiles per wave whenever the wider accesses are aligned: an even run of columns and,
// for real rows, an even row length.
template <int F, int LOAD, int STORE, bool CONTIG>
static int launch_one(const FftPass &p, hipStream_t s)
{
    const bool real_rows = LOAD == LD_REAL || LOAD == LD_REAL_PAIR || STORE == ST_REAL_SCALE_GATE || STORE == ST_REAL_PAIR;
    // (f = 128 with strided columns runs at 128 registers per lane, where two tiles would spill)
    const bool wide = (CONTIG ? p.O : p.S) % 32 == 0 && (!real_rows || p.n_valid % 2 == 0) && (CONTIG || F < 128);
    return wide ? launch_nt<F, LOAD, STORE, CONTIG, 2>(p, s) : launch_nt<F, LOAD, STORE, CONTIG, 1>(p, s);
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
        if (p.store == ST_REAL_PAIR) return launch_one<F, LD_C16, ST_REAL_PAIR, false>(p, s);
        if (p.store == ST_REAL_SCALE_GATE) return launch_one<F, LD_C16, ST_REAL_SCALE_GATE, false>(p, s);
        switch (p.load) {
        case LD_C16: return launch_one<F, LD_C16, ST_C16, false>(p, s);
        case LD_C16_CONJ_MULK: return launch_one<F, LD_C16_CONJ_MULK, ST_C16, false>(p, s);
        case LD_C16_HERM_MULK: return launch_one<F, LD_C16_HERM_MULK, ST_C16, false>(p, s);
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
    const bool real_out = p.store == ST_REAL_PAIR || p.store == ST_REAL_SCALE_GATE;
    if (last ? (p.O % 16 != 0 || p.load != LD_C16)
             : (p.S % 16 != 0 || (real_out ? (p.O != 1 || p.load != LD_C16) : p.store != ST_C16)))
        return fail(MONARCH_EINVAL, "internal: MFMA pass geometry O=%d f=%d S=%d load=%d store=%d", p.O, p.f, p.S, p.load, p.store);
    if ((int64_t)p.O * p.f * p.S != p.N) return fail(MONARCH_EINVAL, "internal: pass geometry does not multiply to N");
    if ((p.O & (p.O - 1)) || (p.S & (p.S - 1)) || p.rows >= (int64_t)1 << 31)   // the kernels index with shifts and 32-bit row numbers
        return fail(MONARCH_EINVAL, "internal: MFMA pass needs power-of-two digits, got O=%d S=%d", p.O, p.S);
    if (fpm::rows_in_applies(p)) return p.f == 64 ? fpm::launch_rows_in<64>(p, s) : fpm::launch_rows_in<32>(p, s);
    if (fpm::rows_out_applies(p)) return p.f == 64 ? fpm::launch_rows_out<64>(p, s) : fpm::launch_rows_out<32>(p, s);
    switch (p.f) {
    case 16: return fpm::launch_f<16>(p, s);
    case 32: return fpm::launch_f<32>(p, s);
    case 64: return fpm::launch_f<64>(p, s);
    case 128: return fpm::launch_f<128>(p, s);
    default: return fail(MONARCH_EINVAL, "internal: factor %d not built for the MFMA path", p.f);
    }
}

}  // namespace monarch
