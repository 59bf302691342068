// Two factors of the Monarch DFT (appendix, DFT corollary) in one kernel, on a chunk of f1 x f2
// complex numbers held in LDS: bf16 operands, fp32 accumulation, f1, f2 in {16, 32, 64, 128}.
//
// The chunk is the last two digits [c1][c2] of a row (the whole row for two factors).  It is read
// from global memory once with coalesced 16-byte accesses, both block-diagonal factors and the
// twiddle diagonal between them are applied in place in LDS, and it is written back once:
//   forward:  X: contract c1 -> j1, times omega_(f1 f2)^(j1 c2);   Y: contract c2 -> j2
//   inverse (as conj o F o conj, factors in the opposite order):
//             Y: contract j2 -> c2, times omega_(f1 f2)^(j1 c2);   X: contract j1 -> c1
// so the spectrum stays in the order the forward leaves it in, position [j1][j2] holding frequency
// j2 f1 + j1: the element-wise product with the kernel's spectrum needs no reordering, and neither
// transform ever stores with a stride.  Stage X reads operands down the columns of the tile
// (8 x 4 bytes per k-step), stage Y along its rows (2 x 16 bytes per k-step); each wave owns whole
// column tiles (X) or row tiles (Y), so a stage works in place and one barrier separates the stages.
#include "kernels.h"

namespace monarch {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

namespace f2l {

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

constexpr int pitch_of(int f2) { return f2 + 4; }              // words per tile row: 16-byte aligned, 4 banks off
// F_64 keeps only the first 32 columns of its operand table: F[j][32 + c] = (-1)^j F[j][c], and a row tile holds
// rows of one parity (tile jt of F_64: rows 32 (jt / 2) + 2 i + jt % 2, i < 16), so the second k-step of an odd
// tile is the first one on negated data.  Every other factor: row tile jt holds rows 16 jt + i.
constexpr bool half_table(int f) { return f == 64; }
constexpr int table_ks(int f) { return half_table(f) ? 1 : (f + 31) / 32; }
constexpr int table_words(int f) { return (f / 16) * table_ks(f) * 2 * 64 * 4; }
template <int F>
__device__ __forceinline__ constexpr int row_of(int jt, int i)
{
    return half_table(F) ? 32 * (jt >> 1) + 2 * i + (jt & 1) : 16 * jt + i;
}

// A-operand table of F_f in MFMA operand order: piece ((jt * KS + ks) * 2 + part) * 64 + lane, KS = table_ks(f)
template <int F, int THREADS>
__device__ __forceinline__ void build_table(u32x4 *tab, float2 *roots)
{
    constexpr int JT = F / 16, KS = table_ks(F);
    for (int e = threadIdx.x; e < F; e += THREADS) roots[e] = omega(e, F);
    __syncthreads();
    for (int idx = threadIdx.x; idx < JT * KS * 64; idx += THREADS) {
        const int ln = idx & 63, ks = (idx >> 6) % KS, jt = idx / (64 * KS);
        const int j = row_of<F>(jt, ln & 15), c0 = 32 * ks + 8 * (ln >> 4);
        u32x4 re, im;
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            float2 w0 = make_float2(0.0f, 0.0f), w1 = w0;
            if (c0 + 2 * h < F) w0 = roots[(j * (c0 + 2 * h)) % F];
            if (c0 + 2 * h + 1 < F) w1 = roots[(j * (c0 + 2 * h + 1)) % F];
            re[h] = pack2(w0.x, w1.x);
            im[h] = pack2(w0.y, w1.y);
        }
        tab[(idx >> 6) * 128 + ln] = re;
        tab[(idx >> 6) * 128 + 64 + ln] = im;
    }
    __syncthreads();
}

// The data operands of one stage_tile call: the real parts (br) and the imaginary parts (bi) of the 16 columns'
// values along the contracted digit, paired for the matrix instruction.
template <int F>
struct StageOps {
    u32x4 br[(F + 31) / 32], bi[(F + 31) / 32];
};

// First half of stage_tile: reads the operands of column tile `col` from the tile.
// SWZ: the tile keeps element (row, col) at column col ^ 16 when bits 3 and 4 of row differ (swz_bit), so that the
// row groups kg and kg + 1 of a strided access (rows 8 kg + e, a multiple of 32 words apart) fall on different
// halves of the 32 banks; a row's 16-byte pieces move together, so row-wise accesses are unchanged.
__device__ __forceinline__ constexpr int swz_bit(int row) { return (((row >> 3) ^ (row >> 4)) & 1) << 4; }
template <int F, int PITCH, bool STRIDED, bool SWZ = false>
__device__ __forceinline__ void stage_load(const uint32_t *tile, int col, int lane, int live_ks, StageOps<F> &ops)
{
    constexpr int KS = (F + 31) / 32;
    const int kg = lane >> 4;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        const int c0 = 32 * ks + 8 * kg;
        uint32_t w[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) w[e] = 0u;
        if (ks < live_ks && c0 < F) {
            if constexpr (STRIDED) {
#pragma unroll
                for (int e = 0; e < 8; ++e) w[e] = tile[(c0 + e) * PITCH + (SWZ ? col ^ swz_bit(8 * kg) : col)];
            } else {
                const int cx = SWZ ? c0 ^ swz_bit(col) : c0;
                const u32x4 v0 = *reinterpret_cast<const u32x4 *>(tile + col * PITCH + cx);
                const u32x4 v1 = *reinterpret_cast<const u32x4 *>(tile + col * PITCH + cx + 4);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    w[e] = v0[e];
                    w[4 + e] = v1[e];
                }
            }
        }
#pragma unroll
        for (int h = 0; h < 4; ++h) {   // low halves (real parts) of two words into one, high halves into another
            ops.br[ks][h] = __builtin_amdgcn_perm(w[2 * h + 1], w[2 * h], 0x05040100u);
            ops.bi[ks][h] = __builtin_amdgcn_perm(w[2 * h + 1], w[2 * h], 0x07060302u);
        }
    }
}

// Second half of stage_tile: the products with the factor's table, the diagonal, and the results back into the
// tile (or to gout).  The table operands of the next row tile are read before the results of the current one
// are written, so that their latency is covered by the diagonal's arithmetic.
template <int F, int PITCH, bool STRIDED, int TW, bool GOUT = false, bool TREG = false, bool SWZ = false>
__device__ __forceinline__ void stage_finish(uint32_t *tile, const u32x4 *tab, const StageOps<F> &ops, int col, int lane, int live_ks,
                                             int want_jt, int alpha, int beta, float inv_mod, float2 *gout = nullptr, int gstride = 0,
                                             const float2 *twp = nullptr)
{
    constexpr int JT = F / 16, KS = (F + 31) / 32, TKS = table_ks(F);
    constexpr bool HALF = half_table(F);
    const int kg = lane >> 4;
    // Re = Fr Br - Fi Bi: the second product takes the negated imaginary parts of the data (nb), one chain
    u32x4 nb[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) nb[ks] = ops.bi[ks] ^ 0x80008000u;
    u32x4 nbr1 = {0, 0, 0, 0};   // HALF: the negated real parts of the second k-step, for the odd row tiles
    if constexpr (HALF) nbr1 = ops.br[1] ^ 0x80008000u;
    // TW == 1: the factors of the rows of the current tile (HALF: of the even and the odd tile of the current pair)
    float2 tw[HALF ? 2 : 1][4], step;
    if constexpr (TW == 1) {
#pragma unroll
        for (int b = 0; b < (HALF ? 2 : 1); ++b)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float rev = (float)(row_of<F>(b, 4 * kg + r) * alpha + beta) * inv_mod;   // exact: the phase stays below the modulus <= 2^24
                tw[b][r] = make_float2(__builtin_amdgcn_cosf(rev), __builtin_amdgcn_sinf(rev));
            }
        const float rev = (float)((HALF ? 32 : 16) * alpha) * inv_mod;
        step = make_float2(__builtin_amdgcn_cosf(rev), __builtin_amdgcn_sinf(rev));
    }
    const int want = HALF ? (want_jt + 1) & ~1 : want_jt;   // (an even and an odd tile make one block of 32 rows)
    uint32_t even[4] = {0u, 0u, 0u, 0u};                    // HALF, stage Y: the packed results of the even tile of the pair
    u32x4 ar[TKS], ai[TKS];                                 // the table operands of the current row tile
    auto table_of = [&](int jt) {
#pragma unroll
        for (int tk = 0; tk < TKS; ++tk) {
            if (tk < live_ks) {
                if constexpr (TREG) {   // this lane's operands, kept in registers by the caller: [jt][tk][re, im]
                    ar[tk] = tab[(jt * TKS + tk) * 2];
                    ai[tk] = tab[(jt * TKS + tk) * 2 + 1];
                } else {
                    ar[tk] = tab[(jt * TKS + tk) * 128 + lane];
                    ai[tk] = tab[(jt * TKS + tk) * 128 + 64 + lane];
                }
            }
        }
    };
    constexpr bool AHEAD = F <= 64;   // (f = 128 runs the row tiles as a loop at 128 registers: no room to read ahead)
    if (AHEAD && 0 < want) table_of(0);
    auto row_tile = [&](int jt) {
        if (jt < want) {
            f32x4 dr = {0, 0, 0, 0}, di = {0, 0, 0, 0};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                if (ks < live_ks) {
                    const int tk = HALF ? 0 : ks;
                    if constexpr (!AHEAD) {   // one k-step's operands at a time
                        ar[tk] = tab[(jt * TKS + tk) * 128 + lane];
                        ai[tk] = tab[(jt * TKS + tk) * 128 + 64 + lane];
                    }
                    const bool flip = HALF && ks == 1 && (jt & 1);   // this k-step's operands are minus the table's
                    dr = mfma(ar[tk], flip ? nbr1 : ops.br[ks], dr);
                    di = mfma(ai[tk], flip ? nbr1 : ops.br[ks], di);
                    dr = mfma(ai[tk], flip ? ops.bi[ks] : nb[ks], dr);
                    di = mfma(ar[tk], flip ? nb[ks] : ops.bi[ks], di);
                }
            }
            if (AHEAD && jt + 1 < want) table_of(jt + 1);
            uint32_t o[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float2 z = make_float2(dr[r], di[r]);
                if constexpr (TW == 1) z = cmul(z, tw[HALF ? jt & 1 : 0][r]);
                if constexpr (TW == 2) z = cmul(z, twp[4 * jt + r]);
                o[r] = pack2(z.x, z.y);
                if constexpr (GOUT)   // the spectrum leaves in natural order, 128-byte runs per 16 lanes, written once: streaming stores
                    store_stream8(&gout[(int64_t)row_of<F>(jt, 4 * kg + r) * gstride + col], make_uint2(__float_as_uint(z.x), __float_as_uint(z.y)));
            }
            if constexpr (GOUT) {
            } else if constexpr (STRIDED) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    tile[row_of<F>(jt, 4 * kg + r) * PITCH + (SWZ ? col ^ swz_bit(HALF ? 8 * kg : 16 * jt + 4 * kg) : col)] = o[r];
            } else if constexpr (HALF) {   // rows 32 J + 8 kg + 2 r + parity: the pair of tiles holds 8 neighbours
                if (jt & 1) {
                    uint32_t *dst = tile + col * PITCH + ((32 * (jt >> 1) + 8 * kg) ^ (SWZ ? swz_bit(col) : 0));
                    *reinterpret_cast<u32x4 *>(dst) = u32x4{even[0], o[0], even[1], o[1]};
                    *reinterpret_cast<u32x4 *>(dst + 4) = u32x4{even[2], o[2], even[3], o[3]};
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r) even[r] = o[r];
                }
            } else {
                *reinterpret_cast<u32x4 *>(tile + col * PITCH + ((16 * jt + 4 * kg) ^ (SWZ ? swz_bit(col) : 0))) = u32x4{o[0], o[1], o[2], o[3]};
            }
        }
        if constexpr (TW == 1) {
            if (!HALF || (jt & 1)) {
#pragma unroll
                for (int b = 0; b < (HALF ? 2 : 1); ++b)
#pragma unroll
                    for (int r = 0; r < 4; ++r) tw[b][r] = cmul(tw[b][r], step);
            }
        }
    };
    if constexpr (TW == 2 || F <= 64) {   // (TW == 2: the factors sit in registers, every index must be a constant)
#pragma unroll
        for (int jt = 0; jt < JT; ++jt) row_tile(jt);
    } else {
#pragma unroll 1
        for (int jt = 0; jt < JT; ++jt) row_tile(jt);
    }
}


// One stage on one tile of 16 columns.  STRIDED: element (c, col) at tile[c * PITCH + col] (stage X);
// otherwise at tile[col * PITCH + c] (stage Y).  live_ks: k-steps holding non-zero inputs; want_jt: 16-row
// blocks of the output that are needed.
// TW: 0 none; 1: multiply output row j by omega_(mod)^(alpha j + beta), computed here with a recurrence over
// the row tiles (alpha = col, beta = 0, mod = f1 f2 for the diagonal between the two factors); 2: the same
// factors handed in by the caller, twp[4 jt + r] for row row_of(jt, 4 (lane / 16) + r) (see twiddles_of).
// GOUT (only with !STRIDED): the results do not go back into the tile but, unrounded, to gout[j * gstride + col]
// as complex fp32 (the natural order of a two-factor transform: frequency j f1 + col).
template <int F, int PITCH, bool STRIDED, int TW, bool GOUT = false>
__device__ __forceinline__ void stage_tile(uint32_t *tile, const u32x4 *tab, int col, int lane, int live_ks, int want_jt,
                                           int alpha, int beta, float inv_mod, float2 *gout = nullptr, int gstride = 0,
                                           const float2 *twp = nullptr)
{
    StageOps<F> ops;
    stage_load<F, PITCH, STRIDED>(tile, col, lane, live_ks, ops);
    stage_finish<F, PITCH, STRIDED, TW, GOUT>(tile, tab, ops, col, lane, live_ks, want_jt, alpha, beta, inv_mod, gout, gstride, twp);
}

// The diagonal of stage_tile for a fixed column, kept by the caller across calls: twp[4 jt + r] =
// omega_(mod)^(alpha row_of(jt, 4 (lane / 16) + r)).
template <int F>
__device__ __forceinline__ void twiddles_of(float2 *twp, int lane, int alpha, float inv_mod)
{
    const int kg = lane >> 4;
#pragma unroll
    for (int jt = 0; jt < F / 16; ++jt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float rev = (float)(row_of<F>(jt, 4 * kg + r) * alpha) * inv_mod;
            twp[4 * jt + r] = make_float2(__builtin_amdgcn_cosf(rev), __builtin_amdgcn_sinf(rev));
        }
}

__device__ __forceinline__ int64_t pair_first_row(const Fft2Args &p, int64_t rc)
{
    return rc + (rc / p.pair_stride) * p.pair_stride;
}

// 8 bf16 values of a 16-byte piece as floats
__device__ __forceinline__ void unpack8(const u32x4 &w, float (&v)[8])
{
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        v[2 * t] = lo_f32(w[t]);
        v[2 * t + 1] = hi_f32(w[t]);
    }
}

// VEC: real rows are read and written 16 bytes (8 elements) at a time, which needs n_valid % 8 == 0; all
// global loads of a chunk are issued together, those of the next chunk (and the output gates of this one)
// before the stages of the current one, so that they are in flight while the matrix cores work.
// TWO (Hermitian separation, three factors): a workgroup takes a chunk o and its mirror chunk O - o in one turn,
// in two tiles: each loaded word and each separated product serves both.
template <int F1, int F2, bool INVERSE, int LOAD, int STORE, bool VEC, bool TWO>
__global__ __launch_bounds__(F1 >= 128 || F2 >= 128 ? 512 : 256) void fft2_lds_kernel(const Fft2Args p)
{
    constexpr int THREADS = F1 >= 128 || F2 >= 128 ? 512 : 256, WAVES = THREADS / 64;
    constexpr int PITCH = pitch_of(F2), CH = F1 * F2;
    constexpr bool REAL_IN = LOAD == LD_REAL || LOAD == LD_REAL_PAIR;
    constexpr bool REAL_OUT = STORE == ST_REAL_SCALE_GATE || STORE == ST_REAL_PAIR;
    constexpr bool MULK = LOAD == LD_C16_CONJ_MULK, HERM = LOAD == LD_C16_HERM_MULK;
    constexpr bool FUSED = REAL_IN && REAL_OUT;   // whole convolution of a two-factor row: forward, times kf, inverse
    constexpr bool NAT_IN = LOAD == LD_C32_CONJ;        // complex fp32 rows in natural order (monarch_ifft's input)
    constexpr bool NAT_OUT = STORE == ST_C32_NATURAL;   // complex fp32 rows in natural order (monarch_fft's output)
    constexpr int NIT4 = (CH + 4 * THREADS - 1) / (4 * THREADS);   // steps of 4 complex elements per thread
    constexpr int NIT2 = (CH + 2 * THREADS - 1) / (2 * THREADS);   // steps of 2 complex elements per thread
    // Natural order: frequency m = j2 F1 + j1 sits at tile position (j1, j2).  Step idx of a thread moves the two
    // neighbours m = 2 idx', 2 idx' + 1 (16 bytes); within a wave 16 (8 if F1 = 16) lanes run along j1 and the
    // rest along j2, which spreads the tile words over the LDS banks.
    constexpr int NAT_A = F1 / 2 < 16 ? F1 / 2 : 16, NAT_G = 64 / NAT_A;
    auto nat_pos = [](int idx, int &j1, int &j2) {
        const int a = idx % NAT_A, g = (idx / NAT_A) % NAT_G, blk = idx / 64;
        constexpr int BJ1 = (F1 / 2) / NAT_A;
        j1 = 2 * ((blk % BJ1) * NAT_A + a);
        j2 = (blk / BJ1) * NAT_G + g;
    };
    constexpr int NIT8 = (CH + 8 * THREADS - 1) / (8 * THREADS);   // steps of 8 real elements per thread
    extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
    uint32_t *tile = lds;                                                   // [F1][PITCH] packed bf16 pairs
    uint32_t *tile2 = lds + F1 * PITCH;                                     // TWO: the mirror chunk
    u32x4 *tab1 = reinterpret_cast<u32x4 *>(lds + (TWO ? 2 : 1) * F1 * PITCH);   // F_f1 operands
    u32x4 *tab2 = F1 == F2 ? tab1 : tab1 + table_words(F1) / 4;             // F_f2 operands
    __shared__ float2 roots[F1 > F2 ? F1 : F2];
    build_table<F1, THREADS>(tab1, roots);
    if constexpr (F1 != F2) build_table<F2, THREADS>(tab2, roots);

    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t nchunks = p.rows * p.O;
    const float inv_mod = 1.0f / (float)CH;
    // rows of the tile that hold input (forward, zero-padded real rows) or wanted output (inverse, truncated)
    const int real_rows_of_tile = (p.n_valid + F2 - 1) / F2;
    const int live_x = REAL_IN ? (real_rows_of_tile + 31) / 32 : (F1 + 31) / 32;   // k-steps of stage X with input
    const int want_x = REAL_OUT ? (real_rows_of_tile + 15) / 16 : F1 / 16;         // row tiles of stage X wanted
    const int lim = REAL_IN ? (live_x * 32 * F2 < CH ? live_x * 32 * F2 : CH) : CH;   // tile elements stage X reads
    auto tix = [](int e) { return (e / F2) * PITCH + (e % F2); };

    // staged inputs of one chunk
    u32x4 za[REAL_IN ? NIT8 : NAT_IN ? NIT2 : NIT4], zb[REAL_IN ? NIT8 : NAT_IN ? 1 : NIT4], zc[REAL_IN ? NIT8 : HERM ? NIT4 : 1],
        zd[REAL_IN ? NIT8 : HERM ? NIT4 : 1];
    auto request = [&](int64_t q) {
        const int64_t rc = q / p.O;
        if constexpr (NAT_IN) {
            const float *src = (const float *)p.in + 2 * rc * (int64_t)p.N;
#pragma unroll
            for (int it = 0; it < NIT2; ++it) {
                const int idx = tid + it * THREADS;
                if (2 * idx < CH) {
                    int j1, j2;
                    nat_pos(idx, j1, j2);
                    za[it] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src + 2 * (j2 * F1 + j1)));
                }
            }
        } else if constexpr (REAL_IN) {
            if constexpr (VEC) {
                const int64_t ra = LOAD == LD_REAL_PAIR ? pair_first_row(p, rc) : rc;
                const bool hasb = LOAD == LD_REAL_PAIR && ra + p.pair_stride < p.real_rows;
                const bf16_t *ua = (const bf16_t *)p.in + ra * p.n_valid, *ub = hasb ? ua + (int64_t)p.pair_stride * p.n_valid : ua;
                const bf16_t *ga = p.gate ? (const bf16_t *)p.gate + ra * p.n_valid : ua;
                const bf16_t *gb = p.gate && hasb ? ga + (int64_t)p.pair_stride * p.n_valid : ga;
#pragma unroll
                for (int it = 0; it < NIT8; ++it) {
                    const int e = 8 * (tid + it * THREADS);
                    const int ee = e < p.n_valid ? e : 0;   // past the row: any valid address, the value is dropped
                    if (it * 8 * THREADS < lim) {
                        // (ordinary loads: streaming ones made the forward transform 6 % slower, 27.7 -> 29.5 us at 6144 x 2048)
                        za[it] = *reinterpret_cast<const u32x4 *>(ua + ee);
                        zc[it] = *reinterpret_cast<const u32x4 *>(ga + ee);
                        if (LOAD == LD_REAL_PAIR) {
                            zb[it] = *reinterpret_cast<const u32x4 *>(ub + ee);
                            zd[it] = *reinterpret_cast<const u32x4 *>(gb + ee);
                        }
                    }
                }
            }
        } else {
            const int64_t at0 = rc * p.N + (q - rc * p.O) * CH;
            const uint32_t *src = (const uint32_t *)p.in + at0;
            const uint32_t *ksrc = MULK ? (const uint32_t *)p.kf + (rc % p.H) * (int64_t)p.N + (q - rc * p.O) * CH
                                   : HERM ? (const uint32_t *)p.kf + at0 : src;
#pragma unroll
            for (int it = 0; it < NIT4; ++it) {
                const int e = 4 * (tid + it * THREADS);
                if (e < CH) {
                    za[it] = *reinterpret_cast<const u32x4 *>(src + e);
                    if (MULK || HERM) zb[it] = *reinterpret_cast<const u32x4 *>(ksrc + e);
                }
            }
            if constexpr (HERM) {
                // Frequency of chunk o, position (j1, j2) is m = j2 f0 f1 + j1 f0 + o; its mirror N - m sits in
                // chunk (f0 - o) mod f0.  For o > 0 the mirror of position e is position CH - 1 - e: one 16-byte
                // piece read backwards.  For o = 0: j1' = (f1 - j1) mod f1, j2' = f2 - 1 - j2 (j1 > 0) or (f2 - j2) mod f2.
                const int o = (int)(q - rc * p.O), om = o ? p.O - o : 0;
                const uint32_t *zm = (const uint32_t *)p.in + rc * p.N + (int64_t)om * CH;
                const uint32_t *km = (const uint32_t *)p.kf + rc * p.N + (int64_t)om * CH;
#pragma unroll
                for (int it = 0; it < NIT4; ++it) {
                    const int e = 4 * (tid + it * THREADS);
                    if (e < CH) {
                        if (o) {
                            const u32x4 a = *reinterpret_cast<const u32x4 *>(zm + CH - 4 - e);
                            const u32x4 b = *reinterpret_cast<const u32x4 *>(km + CH - 4 - e);
                            zc[it] = u32x4{a[3], a[2], a[1], a[0]};
                            zd[it] = u32x4{b[3], b[2], b[1], b[0]};
                        } else {
                            const int j1 = e / F2, j1m = (F1 - j1) % F1;
#pragma unroll
                            for (int t = 0; t < 4; ++t) {
                                const int j2 = e % F2 + t, j2m = j1 ? F2 - 1 - j2 : (F2 - j2) % F2;
                                zc[it][t] = zm[j1m * F2 + j2m];
                                zd[it][t] = km[j1m * F2 + j2m];
                            }
                        }
                    }
                }
            }
        }
    };
    auto deposit = [&](int64_t q, bool paired) {   // staged inputs -> tile (natural order of the chunk)
        if constexpr (NAT_IN) {   // conjugated: the inverse is conj(F conj(.)) / N
#pragma unroll
            for (int it = 0; it < NIT2; ++it) {
                const int idx = tid + it * THREADS;
                if (2 * idx < CH) {
                    int j1, j2;
                    nat_pos(idx, j1, j2);
                    const u32x4 w = za[it];
                    tile[j1 * PITCH + j2] = pack2(__uint_as_float(w[0]), -__uint_as_float(w[1]));
                    tile[(j1 + 1) * PITCH + j2] = pack2(__uint_as_float(w[2]), -__uint_as_float(w[3]));
                }
            }
        } else if constexpr (REAL_IN) {
            const int64_t rc = q / p.O;
            const int64_t ra = LOAD == LD_REAL_PAIR ? pair_first_row(p, rc) : rc;
            const bool hasb = LOAD == LD_REAL_PAIR && ra + p.pair_stride < p.real_rows;
            if constexpr (VEC) {
#pragma unroll
                for (int it = 0; it < NIT8; ++it) {
                    const int e = 8 * (tid + it * THREADS);
                    if (e < lim) {
                        float a[8], b[8], g[8];
                        const bool ok = e < p.n_valid;
                        unpack8(za[it], a);
                        if (p.gate) {
                            unpack8(zc[it], g);
#pragma unroll
                            for (int t = 0; t < 8; ++t) a[t] *= g[t];
                        }
#pragma unroll
                        for (int t = 0; t < 8; ++t) b[t] = 0.0f;
                        if (LOAD == LD_REAL_PAIR && hasb) {
                            unpack8(zb[it], b);
                            if (p.gate) {
                                unpack8(zd[it], g);
#pragma unroll
                                for (int t = 0; t < 8; ++t) b[t] *= g[t];
                            }
                        }
                        u32x4 w0, w1;
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            w0[t] = ok ? pack2(a[t], b[t]) : 0u;
                            w1[t] = ok ? pack2(a[4 + t], b[4 + t]) : 0u;
                        }
                        *reinterpret_cast<u32x4 *>(tile + tix(e)) = w0;
                        *reinterpret_cast<u32x4 *>(tile + tix(e + 4)) = w1;
                    }
                }
            } else {   // any row length: element by element
                const bf16_t *ua = (const bf16_t *)p.in + ra * p.n_valid, *ub = ua + (int64_t)p.pair_stride * p.n_valid;
                const bf16_t *ga = p.gate ? (const bf16_t *)p.gate + ra * p.n_valid : nullptr;
                const bf16_t *gb = ga ? ga + (int64_t)p.pair_stride * p.n_valid : nullptr;
                for (int e = 4 * tid; e < lim; e += 4 * THREADS) {
                    u32x4 w;
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const bool ok = e + t < p.n_valid;
                        float re = ok ? (float)ua[e + t] : 0.0f, im = ok && hasb ? (float)ub[e + t] : 0.0f;
                        if (ga) {
                            re *= ok ? (float)ga[e + t] : 0.0f;
                            im *= ok && hasb ? (float)gb[e + t] : 0.0f;
                        }
                        w[t] = pack2(re, im);
                    }
                    *reinterpret_cast<u32x4 *>(tile + tix(e)) = w;
                }
            }
        } else {
#pragma unroll
            for (int it = 0; it < NIT4; ++it) {
                const int e = 4 * (tid + it * THREADS);
                if (e < CH) {
                    u32x4 w = za[it], w2 = za[it];
                    if constexpr (HERM) {
                        // z = a + i b, kz = ka + i kb (a, b, ka, kb real): A = (Z + conj Z') / 2, B = (Z - conj Z') / 2i,
                        // the same for the kernels; wanted: conj(A Ka + i B Kb), and for the mirror frequency
                        // conj(conj(A Ka) + i conj(B Kb)) = A Ka - i B Kb
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            const float2 z0 = make_float2(lo_f32(w[t]), hi_f32(w[t]));
                            const float2 z1 = make_float2(lo_f32(zc[it][t]), -hi_f32(zc[it][t]));
                            const float2 k0 = make_float2(lo_f32(zb[it][t]), hi_f32(zb[it][t]));
                            const float2 k1 = make_float2(lo_f32(zd[it][t]), -hi_f32(zd[it][t]));
                            const float2 A = make_float2(0.5f * (z0.x + z1.x), 0.5f * (z0.y + z1.y));
                            const float2 Bv = make_float2(0.5f * (z0.y - z1.y), -0.5f * (z0.x - z1.x));
                            const float2 Ka = make_float2(0.5f * (k0.x + k1.x), 0.5f * (k0.y + k1.y));
                            const float2 Kb = make_float2(0.5f * (k0.y - k1.y), -0.5f * (k0.x - k1.x));
                            const float2 pa = cmul(A, Ka), pb = cmul(Bv, Kb);
                            w[t] = pack2(pa.x - pb.y, -(pa.y + pb.x));
                            w2[3 - t] = pack2(pa.x + pb.y, pa.y - pb.x);
                        }
                        if (TWO && paired) *reinterpret_cast<u32x4 *>(tile2 + tix(CH - 4 - e)) = w2;   // mirror of e + t is CH - 1 - e - t
                    }
                    if constexpr (MULK) {
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            const float2 m = cmul(make_float2(lo_f32(w[t]), hi_f32(w[t])),
                                                  make_float2(lo_f32(zb[it][t]), hi_f32(zb[it][t])));
                            w[t] = pack2(m.x, -m.y);
                        }
                    }
                    *reinterpret_cast<u32x4 *>(tile + tix(e)) = w;
                }
            }
        }
    };

    // The i-th chunk of this workgroup, or -1 past the end.  Normally chunk blockIdx + i grid.  With the
    // Hermitian separation a chunk also reads its mirror chunk, so a workgroup takes the two of a mirror
    // pair back to back (the second finds the data in L2): slots 2 b, 2 b + 1, then 2 (b + grid), ... and
    // slot t of a row is chunk 0, O/2, 1, O-1, 2, O-2, ...
    // TWO: a row has O/2 + 1 turns: chunk 0 and chunk O/2 alone (they are their own mirrors), chunk t with O - t.
    const int turns_per_row = TWO ? p.O / 2 + 1 : p.O;
    const int64_t nturns = TWO ? p.rows * turns_per_row : nchunks;
    auto chunk_at = [&](int64_t i) -> int64_t {
        if constexpr (TWO) {
            const int64_t turn = blockIdx.x + i * gridDim.x;
            if (turn >= nturns) return -1;
            const int64_t row = turn / turns_per_row;
            return row * p.O + (turn - row * turns_per_row);
        } else if constexpr (!HERM) {
            const int64_t q = blockIdx.x + i * gridDim.x;
            return q < nchunks ? q : -1;
        } else {
            const int64_t slot = 2 * ((int64_t)blockIdx.x + (i >> 1) * gridDim.x) + (i & 1);
            if (slot >= nchunks) return -1;
            const int64_t row = slot / p.O;
            const int t = (int)(slot - row * p.O), k2 = t >> 1;
            const int o = t < 2 ? (t ? p.O / 2 : 0) : ((t & 1) ? p.O - k2 : k2);
            return row * p.O + (p.O > 1 ? o : 0);
        }
    };
    int64_t q = chunk_at(0);
    if (q >= 0) request(q);
    for (int64_t i = 0; q >= 0; ++i) {
        const int64_t rc = q / p.O;
        const int o_here = (int)(q - rc * p.O);
        const bool paired = TWO && o_here != 0 && 2 * o_here != p.O;   // this turn also carries chunk O - o
        const int ntile = paired ? 2 : 1;
        const int64_t qnext = chunk_at(i + 1);
        deposit(q, paired);
        __syncthreads();
        if (qnext >= 0) request(qnext);

        // output gates of this chunk, requested before the stages
        const int64_t ra = STORE == ST_REAL_PAIR ? pair_first_row(p, rc) : rc;
        const bool hasb = STORE == ST_REAL_PAIR && ra + p.pair_stride < p.real_rows;
        const void *out_gate = FUSED ? p.gate_out : p.gate;
        u32x4 oga[REAL_OUT && VEC ? NIT8 : 1], ogb[REAL_OUT && VEC ? NIT8 : 1], kfr[FUSED ? NIT4 : 1];
        if constexpr (FUSED) {   // this chunk's kernel spectrum, multiplied in between the two transforms
            const uint32_t *ksrc = (const uint32_t *)p.kf + (rc % p.H) * (int64_t)p.N;
#pragma unroll
            for (int it = 0; it < NIT4; ++it) {
                const int e = 4 * (tid + it * THREADS);
                if (e < CH) kfr[it] = *reinterpret_cast<const u32x4 *>(ksrc + e);
            }
        }
        if constexpr (REAL_OUT && VEC) {
            if (out_gate) {
                const bf16_t *ga = (const bf16_t *)out_gate + ra * p.n_valid, *gb = hasb ? ga + (int64_t)p.pair_stride * p.n_valid : ga;
#pragma unroll
                for (int it = 0; it < NIT8; ++it) {
                    const int e = 8 * (tid + it * THREADS);
                    if (e < p.n_valid) {
                        oga[it] = *reinterpret_cast<const u32x4 *>(ga + e);
                        if (STORE == ST_REAL_PAIR) ogb[it] = *reinterpret_cast<const u32x4 *>(gb + e);
                    }
                }
            }
        }

        // ---- the two stages
        if constexpr (!INVERSE) {
            for (int t = wave; t < F2 / 16; t += WAVES)
                stage_tile<F1, PITCH, true, 1>(tile, tab1, 16 * t + l16, lane, live_x, F1 / 16, 16 * t + l16, 0, inv_mod);
            __syncthreads();
            if constexpr (NAT_OUT) {
                float2 *gout = (float2 *)p.out + rc * (int64_t)p.N;
                for (int t = wave; t < F1 / 16; t += WAVES)
                    stage_tile<F2, PITCH, false, 0, true>(tile, tab2, 16 * t + l16, lane, (F2 + 31) / 32, F2 / 16, 0, 0, inv_mod,
                                                              gout, F1);
            } else {
                for (int t = wave; t < F1 / 16; t += WAVES)
                    stage_tile<F2, PITCH, false, 0>(tile, tab2, 16 * t + l16, lane, (F2 + 31) / 32, F2 / 16, 0, 0, inv_mod);
            }
        }
        if constexpr (FUSED) {
            __syncthreads();
#pragma unroll
            for (int it = 0; it < NIT4; ++it) {   // tile <- conj(tile o kf)
                const int e = 4 * (tid + it * THREADS);
                if (e < CH) {
                    u32x4 w = *reinterpret_cast<const u32x4 *>(tile + tix(e));
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const float2 m = cmul(make_float2(lo_f32(w[t]), hi_f32(w[t])),
                                              make_float2(lo_f32(kfr[it][t]), hi_f32(kfr[it][t])));
                        w[t] = pack2(m.x, -m.y);
                    }
                    *reinterpret_cast<u32x4 *>(tile + tix(e)) = w;
                }
            }
            __syncthreads();
        }
        if constexpr (INVERSE || FUSED) {
            // (tile index ti = 1 is the mirror chunk O - o of a paired turn)
            for (int t = wave; t < ntile * (F1 / 16); t += WAVES) {
                const int ti = t / (F1 / 16), tt = t - ti * (F1 / 16);
                stage_tile<F2, PITCH, false, 1>(ti ? tile2 : tile, tab2, 16 * tt + l16, lane, (F2 + 31) / 32, F2 / 16,
                                                   16 * tt + l16, 0, inv_mod);
            }
            __syncthreads();
            if (p.tw_outer) {   // three factors: the diagonal omega_N^(o (f2 c1 + c2)) that precedes the first factor's inverse
                for (int t = wave; t < ntile * (F2 / 16); t += WAVES) {
                    const int ti = t / (F2 / 16), tt = t - ti * (F2 / 16);
                    const int o = ti ? p.O - o_here : o_here;
                    stage_tile<F1, PITCH, true, 1>(ti ? tile2 : tile, tab1, 16 * tt + l16, lane, (F1 + 31) / 32, want_x, o * F2,
                                                      o * (16 * tt + l16), 1.0f / (float)p.N);
                }
            } else {
                for (int t = wave; t < F2 / 16; t += WAVES)
                    stage_tile<F1, PITCH, true, 0>(tile, tab1, 16 * t + l16, lane, (F1 + 31) / 32, want_x, 0, 0, inv_mod);
            }
        }
        __syncthreads();

        // ---- tile -> global
        if constexpr (NAT_OUT) {
            // (written by the second stage)
        } else if constexpr (!REAL_OUT) {
            uint32_t *dst = (uint32_t *)p.out + rc * p.N + (q - rc * p.O) * CH;
#pragma unroll
            for (int it = 0; it < NIT4; ++it) {
                const int e = 4 * (tid + it * THREADS);
                if (e < CH) {
                    u32x4 w = *reinterpret_cast<const u32x4 *>(tile + tix(e));
                    if constexpr (STORE == ST_CPLX_CONJ_SCALE) {   // the inverse's result: conj(tile) / N, as bf16 pairs
#pragma unroll
                        for (int t = 0; t < 4; ++t) w[t] = pack2(lo_f32(w[t]) * p.scale, -hi_f32(w[t]) * p.scale);
                    }
                    *reinterpret_cast<u32x4 *>(dst + e) = w;
                }
            }
            if (TWO && paired) {
                uint32_t *dst2 = (uint32_t *)p.out + rc * p.N + (int64_t)(p.O - o_here) * CH;
#pragma unroll
                for (int it = 0; it < NIT4; ++it) {
                    const int e = 4 * (tid + it * THREADS);
                    if (e < CH) *reinterpret_cast<u32x4 *>(dst2 + e) = *reinterpret_cast<const u32x4 *>(tile2 + tix(e));
                }
            }
        } else {
            // F^-1 = conj(F conj(.)) / N: first member = Re / N, second = -Im / N, times the output gate
            bf16_t *ya = (bf16_t *)p.out + ra * p.n_valid, *yb = ya + (int64_t)p.pair_stride * p.n_valid;
            if constexpr (VEC) {
#pragma unroll
                for (int it = 0; it < NIT8; ++it) {
                    const int e = 8 * (tid + it * THREADS);
                    if (e < p.n_valid) {
                        const bool gated = out_gate != nullptr;
                        const u32x4 w0 = *reinterpret_cast<const u32x4 *>(tile + tix(e));
                        const u32x4 w1 = *reinterpret_cast<const u32x4 *>(tile + tix(e + 4));
                        float va[8], vb[8], g[8];
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            va[t] = lo_f32(w0[t]) * p.scale;
                            vb[t] = -hi_f32(w0[t]) * p.scale;
                            va[4 + t] = lo_f32(w1[t]) * p.scale;
                            vb[4 + t] = -hi_f32(w1[t]) * p.scale;
                        }
                        if (gated) {
                            unpack8(oga[it], g);
#pragma unroll
                            for (int t = 0; t < 8; ++t) va[t] *= g[t];
                        }
                        __builtin_nontemporal_store(u32x4{pack2(va[0], va[1]), pack2(va[2], va[3]), pack2(va[4], va[5]), pack2(va[6], va[7])},
                                                    reinterpret_cast<u32x4 *>(ya + e));
                        if (STORE == ST_REAL_PAIR && hasb) {
                            if (gated) {
                                unpack8(ogb[it], g);
#pragma unroll
                                for (int t = 0; t < 8; ++t) vb[t] *= g[t];
                            }
                            __builtin_nontemporal_store(u32x4{pack2(vb[0], vb[1]), pack2(vb[2], vb[3]), pack2(vb[4], vb[5]), pack2(vb[6], vb[7])},
                                                        reinterpret_cast<u32x4 *>(yb + e));
                        }
                    }
                }
            } else {
                const bf16_t *ga = out_gate ? (const bf16_t *)out_gate + ra * p.n_valid : nullptr;
                const bf16_t *gb = ga ? ga + (int64_t)p.pair_stride * p.n_valid : nullptr;
                for (int e = 4 * tid; e < p.n_valid; e += 4 * THREADS) {
                    const u32x4 w = *reinterpret_cast<const u32x4 *>(tile + tix(e));
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        if (e + t < p.n_valid) {
                            float va = lo_f32(w[t]) * p.scale, vb = -hi_f32(w[t]) * p.scale;
                            if (ga) va *= (float)ga[e + t];
                            ya[e + t] = (bf16_t)va;
                            if (hasb) {
                                if (gb) vb *= (float)gb[e + t];
                                yb[e + t] = (bf16_t)vb;
                            }
                        }
                    }
                }
            }
        }
        __syncthreads();
        q = qnext;
    }
}

// Runs the tasks wave, wave + WAVES, ... < TOTAL of one stage.  (Reading the next task's operands before the current
// task's products was tried: no gain, 16 registers.)
template <int F, int TOTAL, int WAVES, class Load, class Finish>
__device__ __forceinline__ void staged_tasks(int wave, Load &&load, Finish &&finish)
{
    constexpr int NT = (TOTAL + WAVES - 1) / WAVES;
#pragma unroll
    for (int i = 0; i < NT; ++i) {
        const int t = wave + i * WAVES;
        if (t < TOTAL) {
            StageOps<F> ops;
            load(t, ops);
            finish(t, ops);
        }
    }
}

// The four sums of products of the Hermitian separation of two channel-paired spectra, from packed bf16 words
// (re | im << 16): z, k at a frequency, zm, km at its mirror; sk, skm: k and km with their halves swapped.
//   q1 = z k + conj(zm km),   q2 = z conj(km) + conj(zm) k
// as two-term dot products with fp32 accumulation, the signs as operand modifiers.  One block of assembly: a dot
// product's result may be read by another kind of vector instruction only three wait states later, which the
// compiler cannot know about for instructions it does not see; the block ends with them.
__device__ __forceinline__ void separation_sums(uint32_t z, uint32_t zm, uint32_t k, uint32_t km, uint32_t sk, uint32_t skm,
                                                float &q1re, float &q1im, float &q2re, float &q2im)
{
    asm("v_dot2_f32_bf16 %0, %4, %6, 0 neg_hi:[0,1,0]\n\t"
        "v_dot2_f32_bf16 %1, %4, %8, 0\n\t"
        "v_dot2_f32_bf16 %2, %4, %7, 0\n\t"
        "v_dot2_f32_bf16 %3, %4, %9, 0 neg_lo:[0,1,0]\n\t"
        "v_dot2_f32_bf16 %0, %5, %7, %0 neg_hi:[0,1,0]\n\t"
        "v_dot2_f32_bf16 %1, %5, %9, %1 neg_lo:[0,1,0] neg_hi:[0,1,0]\n\t"
        "v_dot2_f32_bf16 %2, %5, %6, %2\n\t"
        "v_dot2_f32_bf16 %3, %5, %8, %3 neg_hi:[0,1,0]\n\t"
        "s_nop 2"
        : "=&v"(q1re), "=&v"(q1im), "=&v"(q2re), "=&v"(q2im)
        : "v"(z), "v"(zm), "v"(k), "v"(km), "v"(sk), "v"(skm));
}

// Middle of a three-factor convolution whose complex rows pair two channels (one sequence per channel), in one
// kernel: the chunk factors of the forward transform of the row and of its kernel row, the separation of the two
// channels' spectra by Hermitian symmetry, their products, and the chunk factors of the inverse with the diagonal
// that precedes the first factor's inverse; the result is 4 times the product spectrum's inverse (the halves of the
// separation are left to the scale of the last pass).  in / kf: the rows of g_in o u and of k after the strided pass on
// the first factor (packed bf16 pairs, chunk o of row r at (r N + o CH) words); out: the same layout, ready for
// the strided inverse pass.
// The spectrum at frequency m needs the one at N - m, which sits in chunk (O - o) mod O: a turn of a workgroup
// takes chunk o and chunk O - o of a row together, four tiles in LDS (0: u chunk o, 1: u mirror chunk, 2 and 3
// the same of k).  Chunks 0 and O / 2 mirror onto themselves and take a turn each with two tiles.  Nothing of the
// spectra ever reaches HBM.
template <int F1, int F2, int THREADS>
__global__ __launch_bounds__(THREADS, 512 / THREADS) void conv3_middle_kernel(const Fft2Args p)
{
    constexpr int WAVES = THREADS / 64, PITCH = pitch_of(F2), CH = F1 * F2, TILE = F1 * PITCH;
    constexpr int NIT4 = (CH + 4 * THREADS - 1) / (4 * THREADS);   // steps of 4 complex elements per thread
    constexpr int XT = F2 / 16, YT = F1 / 16;                     // column tiles of stage X, row tiles of stage Y
    extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
    u32x4 *tab1 = reinterpret_cast<u32x4 *>(lds + 4 * TILE);
    u32x4 *tab2 = F1 == F2 ? tab1 : tab1 + table_words(F1) / 4;
    __shared__ float2 roots[F1 > F2 ? F1 : F2];
    build_table<F1, THREADS>(tab1, roots);
    if constexpr (F1 != F2) build_table<F2, THREADS>(tab2, roots);

    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const float inv_mod = 1.0f / (float)CH;
    constexpr bool SWZ = F1 >= 32 && F2 >= 32;   // (see stage_load)
    auto at_of = [](int row, int col) { return row * PITCH + (SWZ ? col ^ swz_bit(row) : col); };
    auto tix = [&](int e) { return at_of(e / F2, e % F2); };
    // this lane's operands of the two factor matrices stay in registers for the whole kernel
    constexpr int T1 = (F1 / 16) * table_ks(F1) * 2, T2 = (F2 / 16) * table_ks(F2) * 2;
    u32x4 treg1[T1], treg2[F1 == F2 ? 1 : T2];
#pragma unroll
    for (int q = 0; q < T1; ++q) treg1[q] = tab1[q * 64 + lane];
    if constexpr (F1 != F2) {
#pragma unroll
        for (int q = 0; q < T2; ++q) treg2[q] = tab2[q * 64 + lane];
    }
    const u32x4 *tr1 = treg1, *tr2 = F1 == F2 ? treg1 : treg2;
    // a turn is a chunk o in 1 .. O/2 - 1 with its mirror O - o, or (turn 0) the two chunks 0 and O/2 that mirror onto
    // themselves: every turn carries four tiles and the same work
    const int turns_per_row = p.O / 2;
    const int64_t nturns = p.rows * turns_per_row;
    // A wave meets the same column in every task of a stage when the tasks of a tile divide the waves: then the
    // diagonal between the two factors (forward after stage X, inverse after stage Y) is computed once.
    constexpr bool HOIST = WAVES % XT == 0 && WAVES % YT == 0 && F1 <= 64 && F2 <= 64;
    float2 twx[HOIST ? F1 / 4 : 1], twy[HOIST ? F2 / 4 : 1];
    if constexpr (HOIST) {
        twiddles_of<F1>(twx, lane, 16 * (wave % XT) + l16, inv_mod);
        twiddles_of<F2>(twy, lane, 16 * (wave % YT) + l16, inv_mod);
    }

    u32x4 z[4][NIT4];
    auto request = [&](int64_t turn) {
        const int64_t row = turn / turns_per_row;
        const int o = (int)(turn - row * turns_per_row), om = o ? p.O - o : p.O / 2;
        const uint32_t *src[4] = {(const uint32_t *)p.in + row * p.N + (int64_t)o * CH, (const uint32_t *)p.in + row * p.N + (int64_t)om * CH,
                                  (const uint32_t *)p.kf + row * p.N + (int64_t)o * CH, (const uint32_t *)p.kf + row * p.N + (int64_t)om * CH};
#pragma unroll
        for (int it = 0; it < NIT4; ++it) {
            const int e = 4 * (tid + it * THREADS);
            const int ee = e < CH ? e : 0;
#pragma unroll
            for (int t = 0; t < 4; ++t) z[t][it] = *reinterpret_cast<const u32x4 *>(src[t] + ee);
        }
    };

    int64_t turn = blockIdx.x;
    if (turn < nturns) request(turn);
    for (; turn < nturns; turn += gridDim.x) {
        const int64_t row = turn / turns_per_row;
        const int o = (int)(turn - row * turns_per_row), om = o ? p.O - o : p.O / 2;
#pragma unroll
        for (int it = 0; it < NIT4; ++it) {
            const int e = 4 * (tid + it * THREADS);
            if (e < CH) {
#pragma unroll
                for (int t = 0; t < 4; ++t) *reinterpret_cast<u32x4 *>(lds + t * TILE + tix(e)) = z[t][it];
            }
        }
        __syncthreads();
        if (turn + gridDim.x < nturns) request(turn + gridDim.x);

        // ---- forward chunk factors of the row (tiles 0, 1) and of its kernel row (tiles 2, 3)
        constexpr int KX = (F1 + 31) / 32, KY = (F2 + 31) / 32;
        staged_tasks<F1, 4 * XT, WAVES>(
            wave, [&](int t, StageOps<F1> &ops) { stage_load<F1, PITCH, true, SWZ>(lds + (t / XT) * TILE, 16 * (t % XT) + l16, lane, KX, ops); },
            [&](int t, const StageOps<F1> &ops) {
                const int col = 16 * (t % XT) + l16;
                if constexpr (HOIST)
                    stage_finish<F1, PITCH, true, 2, false, true, SWZ>(lds + (t / XT) * TILE, tr1, ops, col, lane, KX, F1 / 16, 0, 0, inv_mod, nullptr, 0, twx);
                else
                    stage_finish<F1, PITCH, true, 1, false, true, SWZ>(lds + (t / XT) * TILE, tr1, ops, col, lane, KX, F1 / 16, col, 0, inv_mod);
            });
        __syncthreads();
        staged_tasks<F2, 4 * YT, WAVES>(
            wave, [&](int t, StageOps<F2> &ops) { stage_load<F2, PITCH, false, SWZ>(lds + (t / YT) * TILE, 16 * (t % YT) + l16, lane, KY, ops); },
            [&](int t, const StageOps<F2> &ops) {
                stage_finish<F2, PITCH, false, 0, false, true, SWZ>(lds + (t / YT) * TILE, tr2, ops, 16 * (t % YT) + l16, lane, KY, F2 / 16, 0, 0, inv_mod);
            });
        __syncthreads();

        // ---- separation and products.  z = a + i b and kz = ka + i kb carry two real channels each:
        // A = (Z + conj Z') / 2, B = (Z - conj Z') / 2i with Z' the value at the mirror frequency, the same for the
        // kernels; the inverse runs as conj o F o conj, so the tile takes conj(A Ka + i B Kb) and the mirror
        // position conj(conj(A Ka) + i conj(B Kb)).  The tiles hold 4 times that: the halves are not applied here.
        // With the words kept packed, the four products Z K, Z conj K', conj Z' K, conj(Z' K') are two-term dot
        // products (exact products, fp32 sums): Q1 = Z K + conj(Z' K'), Q2 = Z conj K' + conj Z' K,
        // 4 A Ka = Q1 + Q2, 4 B Kb = Q2 - Q1.
        auto separate = [](uint32_t zu, uint32_t zum, uint32_t zk, uint32_t zkm, uint32_t &here, uint32_t &there) {
            const uint32_t sk = __builtin_amdgcn_alignbit(zk, zk, 16), skm = __builtin_amdgcn_alignbit(zkm, zkm, 16);   // (im, re)
            float q1re, q1im, q2re, q2im;
            separation_sums(zu, zum, zk, zkm, sk, skm, q1re, q1im, q2re, q2im);
            const float a = q1re + q2re, b = q1im - q2im, c = q1im + q2im, d = q2re - q1re;
            here = pack2(a + b, -c - d);
            there = pack2(a - b, c - d);
        };
        uint32_t *res0 = lds;            // the product tile of chunk o
        uint32_t *res1 = lds + TILE;     // the product tile of chunk O - o (turn 0: of chunk O / 2)
        // The mirror of position e of chunk o is position CH - 1 - e of chunk O - o: 16-byte pieces read backwards.
        // Chunk O / 2 mirrors onto itself that way: the lower half of its positions does both ends.
        {
            uint32_t *zu = o ? lds : lds + TILE, *zk = o ? lds + 2 * TILE : lds + 3 * TILE;
            uint32_t *um = lds + TILE, *km = lds + 3 * TILE;
            const int lim = o ? CH : CH / 2;
#pragma unroll
            for (int it = 0; it < NIT4; ++it) {
                const int e = 4 * (tid + it * THREADS);
                if (e < lim) {
                    const u32x4 a = *reinterpret_cast<const u32x4 *>(zu + tix(e)), b = *reinterpret_cast<const u32x4 *>(um + tix(CH - 4 - e));
                    const u32x4 c = *reinterpret_cast<const u32x4 *>(zk + tix(e)), d = *reinterpret_cast<const u32x4 *>(km + tix(CH - 4 - e));
                    u32x4 w, w2;
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        uint32_t here, there;
                        separate(a[t], b[3 - t], c[t], d[3 - t], here, there);
                        w[t] = here;
                        w2[3 - t] = there;
                    }
                    *reinterpret_cast<u32x4 *>(zu + tix(e)) = w;
                    *reinterpret_cast<u32x4 *>(um + tix(CH - 4 - e)) = w2;
                }
            }
        }
        if (o == 0) {
            // chunk 0 (tiles 0 and 2): the mirror of (j1, j2) is ((f1 - j1) mod f1, f2 - 1 - j2) for j1 > 0 and
            // (0, (f2 - j2) mod f2) for j1 = 0, in the same tile.  One end of every such pair, taken from the rows
            // 0 .. f1 / 2, does both ends in place; a position that is its own mirror is written once.
            for (int e = tid; e < (F1 / 2 + 1) * F2; e += THREADS) {
                const int j1 = e / F2, j2 = e - j1 * F2;
                const bool mine = j1 == 0 ? j2 <= F2 / 2 : (j1 < F1 / 2 || j2 < F2 / 2);
                if (mine) {
                    const int at = at_of(j1, j2);
                    const int m = at_of((F1 - j1) % F1, j1 ? F2 - 1 - j2 : (F2 - j2) % F2);
                    uint32_t w, w2;
                    separate(lds[at], lds[m], lds[2 * TILE + at], lds[2 * TILE + m], w, w2);
                    lds[at] = w;
                    if (m != at) lds[m] = w2;
                }
            }
        }
        __syncthreads();

        // ---- inverse chunk factors, then the diagonal omega_N^(o (f2 c1 + c2)) that precedes the first factor's inverse
        staged_tasks<F2, 2 * YT, WAVES>(
            wave, [&](int t, StageOps<F2> &ops) { stage_load<F2, PITCH, false, SWZ>(t / YT ? res1 : res0, 16 * (t % YT) + l16, lane, KY, ops); },
            [&](int t, const StageOps<F2> &ops) {
                const int col = 16 * (t % YT) + l16;
                if constexpr (HOIST)
                    stage_finish<F2, PITCH, false, 2, false, true, SWZ>(t / YT ? res1 : res0, tr2, ops, col, lane, KY, F2 / 16, 0, 0, inv_mod, nullptr, 0, twy);
                else
                    stage_finish<F2, PITCH, false, 1, false, true, SWZ>(t / YT ? res1 : res0, tr2, ops, col, lane, KY, F2 / 16, col, 0, inv_mod);
            });
        __syncthreads();
        staged_tasks<F1, 2 * XT, WAVES>(
            wave, [&](int t, StageOps<F1> &ops) { stage_load<F1, PITCH, true, SWZ>(t / XT ? res1 : res0, 16 * (t % XT) + l16, lane, KX, ops); },
            [&](int t, const StageOps<F1> &ops) {
                const int col = 16 * (t % XT) + l16, oo = t / XT ? om : o;
                stage_finish<F1, PITCH, true, 1, false, true, SWZ>(t / XT ? res1 : res0, tr1, ops, col, lane, KX, F1 / 16, oo * F2, oo * col, 1.0f / (float)p.N);
            });
        __syncthreads();

        uint32_t *dst = (uint32_t *)p.out + row * p.N + (int64_t)o * CH;
        uint32_t *dst2 = (uint32_t *)p.out + row * p.N + (int64_t)om * CH;
#pragma unroll
        for (int it = 0; it < NIT4; ++it) {
            const int e = 4 * (tid + it * THREADS);
            if (e < CH) {
                // (streaming stores, and streaming loads in the last pass that reads these rows: 261 -> 253 us at config 5a;
                //  streaming between the first pass and this kernel gained nothing)
                __builtin_nontemporal_store(*reinterpret_cast<const u32x4 *>(res0 + tix(e)), reinterpret_cast<u32x4 *>(dst + e));
                __builtin_nontemporal_store(*reinterpret_cast<const u32x4 *>(res1 + tix(e)), reinterpret_cast<u32x4 *>(dst2 + e));
            }
        }
        __syncthreads();
    }
}

static size_t middle_lds_bytes(int f1, int f2)
{
    return ((size_t)4 * f1 * pitch_of(f2) + table_words(f1) + (f1 == f2 ? 0 : table_words(f2))) * 4;
}

template <int F1, int F2>
static int launch_middle(const Fft2Args &p, hipStream_t s)
{
    constexpr int THREADS = 256;   // two workgroups per compute unit when four tiles and the tables fit in half of LDS
    const size_t lds = middle_lds_bytes(F1, F2);
    int dev = 0, ncu = 0;
    MONARCH_HIP_CHECK(hipGetDevice(&dev));
    MONARCH_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
    const int per_cu = (int)((160 * 1024) / (lds + 1024));
    const int64_t nturns = p.rows * (p.O / 2);
    int64_t grid = (int64_t)ncu * (per_cu < 1 ? 1 : per_cu > 2 ? 2 : per_cu);
    if (grid > nturns) grid = nturns;
    auto kern = conv3_middle_kernel<F1, F2, THREADS>;
    if (lds > 48 * 1024)
        MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(THREADS), lds, s, p);
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

static size_t lds_bytes(int f1, int f2, int tiles = 1)
{
    return ((size_t)tiles * f1 * pitch_of(f2) + table_words(f1) + (f1 == f2 ? 0 : table_words(f2))) * 4;
}

template <int F1, int F2, bool INVERSE, int LOAD, int STORE, bool VEC, bool TWO = false>
static int launch_vec(const Fft2Args &p, hipStream_t s)
{
    constexpr int THREADS = F1 >= 128 || F2 >= 128 ? 512 : 256;
    const size_t lds = lds_bytes(F1, F2, TWO ? 2 : 1);
    int dev = 0, ncu = 0;
    MONARCH_HIP_CHECK(hipGetDevice(&dev));
    MONARCH_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
    const int per_cu = (int)((160 * 1024) / (lds + 1024));
    const int64_t nchunks = TWO ? p.rows * (p.O / 2 + 1) : p.rows * p.O;   // turns of a workgroup
    int64_t grid = (int64_t)ncu * (per_cu < 1 ? 1 : per_cu > 4 ? 4 : per_cu);
    if (grid > nchunks) grid = nchunks;
    if (!TWO && LOAD == LD_C16_HERM_MULK && grid > (nchunks + 1) / 2) grid = (nchunks + 1) / 2;   // two chunks per turn
    auto kern = fft2_lds_kernel<F1, F2, INVERSE, LOAD, STORE, VEC, TWO>;
    if (lds > 48 * 1024)
        MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(THREADS), lds, s, p);
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

template <int F1, int F2, bool INVERSE, int LOAD, int STORE>
static int launch_one(const Fft2Args &p, hipStream_t s)
{
    constexpr bool real_rows = LOAD == LD_REAL || LOAD == LD_REAL_PAIR || STORE == ST_REAL_SCALE_GATE || STORE == ST_REAL_PAIR;
    if (!real_rows || p.n_valid % 8 == 0) return launch_vec<F1, F2, INVERSE, LOAD, STORE, true>(p, s);
    return launch_vec<F1, F2, INVERSE, LOAD, STORE, false>(p, s);
}

template <int F1, int F2>
static int launch_modes(const Fft2Args &p, hipStream_t s)
{
    if (p.O == 1 && !p.inverse && p.load == LD_REAL && p.store == ST_C32_NATURAL)   // monarch_fft, real rows
        return launch_one<F1, F2, false, LD_REAL, ST_C32_NATURAL>(p, s);
    if (p.O == 1 && p.inverse && p.load == LD_C32_CONJ && p.store == ST_REAL_SCALE_GATE)   // monarch_ifft, real rows
        return launch_one<F1, F2, true, LD_C32_CONJ, ST_REAL_SCALE_GATE>(p, s);
    if (p.O == 1 && !p.inverse && p.load == LD_C16 && p.store == ST_C32_NATURAL)   // monarch_fft, complex bf16 rows
        return launch_one<F1, F2, false, LD_C16, ST_C32_NATURAL>(p, s);
    if (p.O == 1 && p.inverse && p.load == LD_C32_CONJ && p.store == ST_CPLX_CONJ_SCALE)   // monarch_ifft, complex bf16 rows
        return launch_one<F1, F2, true, LD_C32_CONJ, ST_CPLX_CONJ_SCALE>(p, s);
    if (!p.inverse && p.store != ST_C16) {   // whole convolution in one kernel
        if (p.n_valid % 8) return fail(MONARCH_EINVAL, "internal: the fused chunk convolution needs rows of a multiple of 8 elements");
        if (p.load == LD_REAL_PAIR && p.store == ST_REAL_PAIR) return launch_vec<F1, F2, false, LD_REAL_PAIR, ST_REAL_PAIR, true>(p, s);
        if (p.load == LD_REAL && p.store == ST_REAL_SCALE_GATE) return launch_vec<F1, F2, false, LD_REAL, ST_REAL_SCALE_GATE, true>(p, s);
        return fail(MONARCH_EINVAL, "internal: fused chunk convolution modes %d/%d not built", p.load, p.store);
    }
    if (!p.inverse) {
        switch (p.load) {
        case LD_REAL: return launch_one<F1, F2, false, LD_REAL, ST_C16>(p, s);
        case LD_REAL_PAIR: return launch_one<F1, F2, false, LD_REAL_PAIR, ST_C16>(p, s);
        case LD_C16: return launch_one<F1, F2, false, LD_C16, ST_C16>(p, s);
        default: break;
        }
    } else if (p.load == LD_C16_CONJ_MULK) {
        switch (p.store) {
        case ST_REAL_SCALE_GATE: return launch_one<F1, F2, true, LD_C16_CONJ_MULK, ST_REAL_SCALE_GATE>(p, s);
        case ST_REAL_PAIR: return launch_one<F1, F2, true, LD_C16_CONJ_MULK, ST_REAL_PAIR>(p, s);
        case ST_C16: return launch_one<F1, F2, true, LD_C16_CONJ_MULK, ST_C16>(p, s);
        default: break;
        }
    } else if (p.load == LD_C16_HERM_MULK) {
        if (p.store == ST_C16) {
            // three factors and room for two tiles: mirror chunks together
            if (p.O >= 2 && p.O % 2 == 0 && lds_bytes(F1, F2, 2) + 1024 <= 80 * 1024)
                return launch_vec<F1, F2, true, LD_C16_HERM_MULK, ST_C16, true, true>(p, s);
            return launch_one<F1, F2, true, LD_C16_HERM_MULK, ST_C16>(p, s);
        }
        if (p.store == ST_REAL_PAIR) return launch_one<F1, F2, true, LD_C16_HERM_MULK, ST_REAL_PAIR>(p, s);
    }
    return fail(MONARCH_EINVAL, "internal: chunk kernel modes %d/%d not built", p.load, p.store);
}

}  // namespace f2l

// the chunk shapes that are instantiated below
static bool chunk_built(int f1, int f2)
{
    static const int shapes[][2] = {{128, 128}, {64, 64}, {64, 32}, {32, 64}, {32, 32}, {16, 16}, {128, 64}, {64, 128}};
    for (const auto &sh : shapes)
        if (sh[0] == f1 && sh[1] == f2) return true;
    return false;
}

bool fft2_lds_supported(int f1, int f2, monarch_dtype dt)
{
    return dt == MONARCH_BF16 && chunk_built(f1, f2) && f2l::lds_bytes(f1, f2) + 1024 <= 160 * 1024;
}

// chunk shapes of the fused middle of a three-factor convolution: four tiles and the tables fit in LDS
static bool middle_built(int f1, int f2)
{
    static const int shapes[][2] = {{64, 64}, {64, 32}, {32, 64}, {32, 32}, {16, 16}};
    for (const auto &sh : shapes)
        if (sh[0] == f1 && sh[1] == f2) return true;
    return false;
}

bool conv3_middle_supported(int O, int f1, int f2, monarch_dtype dt)
{
    return dt == MONARCH_BF16 && O >= 2 && O % 2 == 0 && middle_built(f1, f2) && f2l::middle_lds_bytes(f1, f2) + 1024 <= 160 * 1024;
}

int launch_conv3_middle(const Fft2Args &p, hipStream_t s)
{
    if (p.rows == 0) return MONARCH_OK;
    if ((int64_t)p.O * p.f1 * p.f2 != p.N || p.O % 2) return fail(MONARCH_EINVAL, "internal: chunk geometry of the fused middle");
#define MONARCH_MID(A, B) \
    if (p.f1 == A && p.f2 == B) return f2l::launch_middle<A, B>(p, s)
    MONARCH_MID(64, 64);
    MONARCH_MID(64, 32);
    MONARCH_MID(32, 64);
    MONARCH_MID(32, 32);
    MONARCH_MID(16, 16);
#undef MONARCH_MID
    return fail(MONARCH_EINVAL, "internal: fused middle %d x %d not built", p.f1, p.f2);
}

int launch_fft2_lds(const Fft2Args &p, hipStream_t s)
{
    if (p.rows == 0) return MONARCH_OK;
    if ((int64_t)p.O * p.f1 * p.f2 != p.N) return fail(MONARCH_EINVAL, "internal: chunk geometry does not multiply to N");
#define MONARCH_F2L(A, B) \
    if (p.f1 == A && p.f2 == B) return f2l::launch_modes<A, B>(p, s)
    MONARCH_F2L(128, 128);
    MONARCH_F2L(64, 64);
    MONARCH_F2L(64, 32);
    MONARCH_F2L(32, 64);
    MONARCH_F2L(32, 32);
    MONARCH_F2L(16, 16);
    MONARCH_F2L(128, 64);
    MONARCH_F2L(64, 128);
#undef MONARCH_F2L
    return fail(MONARCH_EINVAL, "internal: chunk %d x %d not built", p.f1, p.f2);
}

}  // namespace monarch
