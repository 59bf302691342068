// Fused gated causal Monarch-FFT convolution, nfft = 16384 = 128 x 128, bf16 I/O, fp32 accumulate.
//
// One workgroup of 8 waves per compute unit walks over channels.  For a channel it first turns k[h] into its
// spectrum k_f, which stays in LDS in the lanes' own accumulator order (64 KB), then takes the channel's batch rows in PAIRS
// z = x0 + i x1 (the kernel is real, so conv(z) = conv(x0) + i conv(x1)) through
//   pad -> X -> twiddle -> Y -> (.) k_f -> Y' -> twiddle -> X' -> truncate -> gate
// on one 128 x 128 tile of packed (re | im) bf16 words in LDS.  Row r of the tile is digit c1 (later j1) of the
// position c1*128 + c2, column c is digit c2 (later j2): the Monarch factors are R = I (x) F_128 down the
// columns (stage X), the diagonal w_16384^(j1 c2), and L = F_128 blocks along the rows (stage Y); the spectrum
// sits at [j1][j2] = frequency j2*128 + j1 and the inverse, written conj o F o conj with its factors in the
// opposite order, consumes it in place.  The permutations P of M = P L P R P are the choice of which tile
// axis a stage contracts; nothing is ever moved for them.
//
// How the 128 x 128 DFT matrix fits in 32 registers per lane.  A stage computes out[j][col] = sum_c F[j][c] in[c][col]
// as 16x16x32 MFMAs: A = 16 rows of F, B = 32 contraction values of 16 columns.  Because
// F[j][32 ks + c'] = i^(j ks) F[j][c'], a row tile whose 16 rows all have the same j mod 4 = q needs only the
// first 32 columns of F: the factor i^(q ks) of contraction block ks is a compile-time choice of which of four
// accumulator chains (+Re, -Re, +Im, -Im) each of the four real products of the complex product feeds.  The 8
// row tiles (q, T) hold rows j = 64 T + 32 (r>>1) + 8 kg + 4 (r&1) + q (kg = lane / 16, r = accumulator
// register), chosen so that the packed accumulators of the 8 tiles are, without any data movement, the B
// operands of a following stage that contracts the index just produced (block ks = 2T + (r>>1), slot
// 8 kg + 4 (r&1) + q): stage Y' starts from stage Y's registers.  And the tiles T = 1 need no registers of their
// own: F[j + 64][c] = (-1)^c F[j][c] is a sign flip of the odd slots.  No operand table lives in LDS, every wave
// owns whole columns (X, X') or whole rows (Y, Y') of the tile, and a stage works in place.
//
// Appendix DFT corollary (Monarch form of F_N), Sec. 3.2 Eq. 2 with gating, Thm 3 (padding).
#include "const_roots.h"
#include "kernels.h"

namespace monarch {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

namespace c16k {

constexpr int F = 128, NFFT = 16384, NMAX = 8192;
constexpr int PITCH = 132;            // words per tile row (16-byte aligned rows, 4 banks off per row)
constexpr int THREADS = 512;     // 8 waves: wave w owns columns (rows) 16 w .. 16 w + 15 of the tile
constexpr int TILE_WORDS = F * PITCH;

// Output row of accumulator register r of lane group kg in row tile (T, q).
constexpr int jrow(int T, int q, int kg, int r) { return 64 * T + 32 * (r >> 1) + 8 * kg + 4 * (r & 1) + q; }

// Per-lane constant A operands of the tiles T = 0: [lane][q][re, im][word h]: F_128[j][8 kg + 2h], [8 kg + 2h + 1]
// with j the tile's row for A-operand row lane % 16 (= accumulator row 4 kg' + r).  The tiles T = 1 hold the rows
// j + 64, and F[j + 64][c] = (-1)^c F[j][c]: the same words with the sign of every odd slot (the high halves) flipped.
struct OperandTable { uint32_t v[64][4][2][4]; };
constexpr OperandTable make_operands()
{
    OperandTable t{};
    for (int lane = 0; lane < 64; ++lane)
        for (int tile = 0; tile < 4; ++tile)
            for (int h = 0; h < 4; ++h) {
                const int rho = lane & 15, kg = lane >> 4;
                const int j = jrow(0, tile, rho >> 2, rho & 3), c0 = 8 * kg + 2 * h;
                const croots::CosSin w0 = croots::unit_root(j * c0, F), w1 = croots::unit_root(j * (c0 + 1), F);
                t.v[lane][tile][0][h] = croots::bf16_bits(w0.c) | (croots::bf16_bits(w1.c) << 16);
                t.v[lane][tile][1][h] = croots::bf16_bits(w0.s) | (croots::bf16_bits(w1.s) << 16);
            }
    return t;
}
__device__ const OperandTable g_operands = make_operands();

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

// Column of the tile word (row, col): the 16-column groups of a row are swapped when bits 3 and 4 of the row differ.
// The four lane groups of a strided access read rows 8 apart: 8 rows are 32 banks, so with the swap they fall on
// four different sets of 16 banks, whether the LDS has 32 banks (two lane groups per pass) or 64; runs of 16
// columns stay contiguous for the 16-byte accesses along a row.
__device__ __forceinline__ int swz_bit(int row) { return (((row >> 3) ^ (row >> 4)) & 1) << 4; }
__device__ __forceinline__ int swz(int row, int col) { return col ^ swz_bit(row); }

struct Ops { u32x4 re[4], im[4]; };     // the whole F_128 as this lane's A operands: 32 registers (rows j < 64)
template <int T> __device__ __forceinline__ u32x4 half_rows(const u32x4 &a)   // rows j + 64 T of the same tile
{
    if (T == 0) return a;
    uint32_t odd = 0x80000000u;
    asm volatile("" : "+v"(odd));   // opaque, so that the flipped copies are made where they are used and not kept
    return u32x4{a[0] ^ odd, a[1] ^ odd, a[2] ^ odd, a[3] ^ odd};
}
struct Bops { u32x4 re[4], im[4]; };    // B operands of one stage: four contraction blocks of 32

// Splits 8 packed (re | im) words of one contraction block into the re and im operands.
__device__ __forceinline__ void split_block(const uint32_t (&w)[8], u32x4 &re, u32x4 &im)
{
#pragma unroll
    for (int h = 0; h < 4; ++h) {
        re[h] = __builtin_amdgcn_perm(w[2 * h + 1], w[2 * h], 0x05040100u);
        im[h] = __builtin_amdgcn_perm(w[2 * h + 1], w[2 * h], 0x07060302u);
    }
}

// One row tile (T, Q): out[j] = sum over blocks ks < NKS of i^(Q ks) F0[j][:] B[ks], as four accumulator chains.
template <int Q, int NKS, bool HAS_IM>
__device__ __forceinline__ void row_tile(const u32x4 &ar, const u32x4 &ai, const Bops &b, f32x4 &re, f32x4 &im)
{
    f32x4 rp = {0, 0, 0, 0}, rm = {0, 0, 0, 0}, ip = {0, 0, 0, 0}, in = {0, 0, 0, 0};
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
        switch ((Q * ks) & 3) {
        case 0:
            rp = mfma(ar, b.re[ks], rp);
            ip = mfma(ai, b.re[ks], ip);
            if (HAS_IM) {
                rm = mfma(ai, b.im[ks], rm);
                ip = mfma(ar, b.im[ks], ip);
            }
            break;
        case 1:   // times i: Re -= Q, Im += P
            ip = mfma(ar, b.re[ks], ip);
            rm = mfma(ai, b.re[ks], rm);
            if (HAS_IM) {
                in = mfma(ai, b.im[ks], in);
                rm = mfma(ar, b.im[ks], rm);
            }
            break;
        case 2:   // times -1
            rm = mfma(ar, b.re[ks], rm);
            in = mfma(ai, b.re[ks], in);
            if (HAS_IM) {
                rp = mfma(ai, b.im[ks], rp);
                in = mfma(ar, b.im[ks], in);
            }
            break;
        default:  // times -i: Re += Q, Im -= P
            in = mfma(ar, b.re[ks], in);
            rp = mfma(ai, b.re[ks], rp);
            if (HAS_IM) {
                ip = mfma(ai, b.im[ks], ip);
                rp = mfma(ar, b.im[ks], rp);
            }
            break;
        }
    }
    re = rp - rm;
    im = ip - in;
}

// The diagonal w_16384^(x j) for this lane's fixed index x (its column in stage X, its row in stage Y') and the
// accumulator rows j of the tiles visited in the order T = 0: q = 0..3, T = 1: q = 0..3: a recurrence in fp32.
struct Twiddle {
    float2 cur[4], step_q, step_t;
    __device__ __forceinline__ void init(int x, int kg)
    {
        const float inv = 1.0f / (float)NFFT;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float rev = (float)(x * (8 * kg + 32 * (r >> 1) + 4 * (r & 1))) * inv;   // x j < 2^14: exact
            cur[r] = make_float2(__builtin_amdgcn_cosf(rev), __builtin_amdgcn_sinf(rev));
        }
        const float r1 = (float)x * inv, r60 = (float)(60 * x) * inv;
        step_q = make_float2(__builtin_amdgcn_cosf(r1), __builtin_amdgcn_sinf(r1));
        step_t = make_float2(__builtin_amdgcn_cosf(r60), __builtin_amdgcn_sinf(r60));
    }
    __device__ __forceinline__ void next_q()
    {
#pragma unroll
        for (int r = 0; r < 4; ++r) cur[r] = cmul(cur[r], step_q);
    }
    __device__ __forceinline__ void next_t()   // after four next_q: from j + 4 to j + 64
    {
#pragma unroll
        for (int r = 0; r < 4; ++r) cur[r] = cmul(cur[r], step_t);
    }
};

// Rows of one job as loaded: two 16-byte pieces per thread of each of the (up to) four rows.
struct RowRegs { u32x4 a[2], b[2], ga[2], gb[2]; };

// (rows of u, k and the gates are read once per launch, y written once: streaming accesses)
__device__ __forceinline__ u32x4 load_here(const bf16_t *p) { return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p)); }

__device__ __forceinline__ void unpack8(const u32x4 &w, float (&v)[8])
{
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        v[2 * t] = lo_f32(w[t]);
        v[2 * t + 1] = hi_f32(w[t]);
    }
}

template <bool GIN, bool GOUT>
__global__ __launch_bounds__(THREADS, 2) void conv16k_bf16_kernel(
    const bf16_t *__restrict__ u, const bf16_t *__restrict__ k, const bf16_t *__restrict__ g_in,
    const bf16_t *__restrict__ g_out, bf16_t *__restrict__ y, int B, int H, int n, int klen)
{
    extern __shared__ __attribute__((aligned(16))) uint32_t tile[];   // [128][PITCH] packed (re | im << 16)
    const int tid = threadIdx.x, lane = tid & 63, l16 = lane & 15, kg = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int P = (B + 1) >> 1;                 // row pairs per channel
    const int jobs_per_channel = 1 + P;         // the kernel's spectrum, then the pairs

    Ops A;
    {
        const u32x4 *src = reinterpret_cast<const u32x4 *>(g_operands.v[lane]);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            A.re[t] = src[2 * t];
            A.im[t] = src[2 * t + 1];
        }
    }
    // k_f / NFFT of this lane's accumulator positions in stage Y: [tile][lane] pieces of four packed (re | im) words
    u32x4 *kf = reinterpret_cast<u32x4 *>(tile + TILE_WORDS) + (size_t)wave * 8 * 64 + lane;

    // stage X / X': this wave's 16 columns; this lane's words sit at xbase + row' * PITCH, row' = row - 8 kg
    const int xcol = 16 * wave + l16;
    const int xbase = 8 * kg * PITCH + (xcol ^ swz_bit(8 * kg));
    // stage Y / Y': this wave's 16 rows
    const int yrow = 16 * wave + l16;
    const int yswz = swz_bit(yrow);
    const uint32_t *yline = tile + yrow * PITCH;

    // job g of this workgroup: channel blockIdx.x + (g / jobs_per_channel) * gridDim.x, step g % jobs_per_channel
    auto job_channel = [&](int g) { return (int)blockIdx.x + (g / jobs_per_channel) * (int)gridDim.x; };
    RowRegs in;
    u32x4 oga[2], ogb[2];
    // All loads of a job, issued together.  One straight line of code for both kinds of job (a kernel job reads
    // its row of k as the first row and one dummy piece for the others; a job past the end reads valid rows that
    // nobody uses): the same registers are loaded by the same instructions every time, so nothing has to be
    // copied, and therefore waited for, where the requests are made.
    auto request = [&](int g) {
        int h = job_channel(g);
        const int s = g % jobs_per_channel;
        if (h >= H) h = (int)blockIdx.x;
        const bool isk = s == 0;
        const int b0 = isk ? 0 : 2 * (s - 1), b1 = b0 + 1 < B ? b0 + 1 : b0;
        const int len = isk ? klen : n;
        const size_t ra = ((size_t)b0 * H + h) * n, rb = ((size_t)b1 * H + h) * n;
        const bf16_t *pa = isk ? k + (size_t)h * klen : u + ra;
        const bf16_t *pb = isk ? pa : u + rb;
        const bf16_t *pga = isk ? pa : g_in + ra, *pgb = isk ? pa : g_in + rb;
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int e = 8 * (tid + it * THREADS), ee = e < len ? e : 0, eo = isk ? 0 : ee;
            in.a[it] = load_here(pa + ee);
            in.b[it] = load_here(pb + eo);
            if (GIN) {
                in.ga[it] = load_here(pga + eo);
                in.gb[it] = load_here(pgb + eo);
            }
        }
    };

    // B operands of a column stage: rows 32 ks + 8 kg + e of this lane's column
    auto read_columns = [&](Bops &b, int nks) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if (ks < nks) {
                uint32_t w[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) w[e] = tile[xbase + (32 * ks + e) * PITCH];
                split_block(w, b.re[ks], b.im[ks]);
            }
        }
    };

    // Rows of job g (as requested) -> tile rows c1 < 64, zero past the end of the row.  Every thread writes the same
    // tile words that it reads in the last pass of a pair job, so no barrier is needed between that pass and this.
    auto deposit = [&](int g) {
        const int s = g % jobs_per_channel;
        const bool isk = s == 0;
        const bool two = !isk && 2 * (s - 1) + 1 < B;
        const int len = isk ? klen : n;
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int e = 8 * (tid + it * THREADS), row = e >> 7, col = e & 127;
            float a[8], bb[8], gt[8];
            unpack8(in.a[it], a);
            if (GIN && !isk) {
                unpack8(in.ga[it], gt);
#pragma unroll
                for (int t = 0; t < 8; ++t) a[t] *= gt[t];
            }
#pragma unroll
            for (int t = 0; t < 8; ++t) bb[t] = 0.0f;
            if (two) {
                unpack8(in.b[it], bb);
                if (GIN) {
                    unpack8(in.gb[it], gt);
#pragma unroll
                    for (int t = 0; t < 8; ++t) bb[t] *= gt[t];
                }
            }
            const bool ok = e < len;
            u32x4 w0, w1;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                w0[t] = ok ? pack2(a[t], bb[t]) : 0u;
                w1[t] = ok ? pack2(a[4 + t], bb[4 + t]) : 0u;
            }
            uint32_t *dst = tile + row * PITCH + swz(row, col);
            *reinterpret_cast<u32x4 *>(dst) = w0;
            *reinterpret_cast<u32x4 *>(dst + 4) = w1;
        }
    };

    request(0);
    deposit(0);
    __syncthreads();
    for (int g = 0;; ++g) {
        const int h = job_channel(g), s = g % jobs_per_channel;
        if (h >= H) break;
        const bool is_kernel = s == 0;
        const int b0 = 2 * (s - 1);
        const bool hasb = !is_kernel && b0 + 1 < B;
        const bool more = job_channel(g + 1) < H;   // another job follows
        request(g + 1);   // the next job's rows travel while this one is transformed

        // ---- stage X: contract c1 down this wave's columns (rows >= 64 are padding: two blocks), twiddle
        {
            Bops b;
            read_columns(b, 2);
            Twiddle tw;
            tw.init(xcol, kg);
            auto emit = [&](int T, int q, const f32x4 &re, const f32x4 &im) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float2 z = cmul(make_float2(re[r], im[r]), tw.cur[r]);
                    tile[xbase + (64 * T + 32 * (r >> 1) + 4 * (r & 1) + q) * PITCH] = pack2(z.x, z.y);
                }
            };
#define MONARCH_C16K_X_TILE(T, Q)                                                       \
    {                                                                                   \
        f32x4 re, im;                                                                   \
        if (is_kernel) row_tile<Q, 2, false>(half_rows<T>(A.re[Q]), half_rows<T>(A.im[Q]), b, re, im); \
        else row_tile<Q, 2, true>(half_rows<T>(A.re[Q]), half_rows<T>(A.im[Q]), b, re, im);         \
        emit(T, Q, re, im);                                                             \
    }
            MONARCH_C16K_X_TILE(0, 0) tw.next_q();
            MONARCH_C16K_X_TILE(0, 1) tw.next_q();
            MONARCH_C16K_X_TILE(0, 2) tw.next_q();
            MONARCH_C16K_X_TILE(0, 3) tw.next_q(); tw.next_t();
            MONARCH_C16K_X_TILE(1, 0) tw.next_q();
            MONARCH_C16K_X_TILE(1, 1) tw.next_q();
            MONARCH_C16K_X_TILE(1, 2) tw.next_q();
            MONARCH_C16K_X_TILE(1, 3)
#undef MONARCH_C16K_X_TILE
        }
        __syncthreads();

        // ---- stage Y: contract c2 along this wave's rows
        Bops by;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const u32x4 v0 = *reinterpret_cast<const u32x4 *>(yline + ((32 * ks + 8 * kg) ^ yswz));
            const u32x4 v1 = *reinterpret_cast<const u32x4 *>(yline + ((32 * ks + 8 * kg) ^ yswz) + 4);
            const uint32_t w[8] = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
            split_block(w, by.re[ks], by.im[ks]);
        }
        if (is_kernel) {
            // the spectrum of k, scaled by 1 / nfft, stays in LDS for the pairs of this channel (each lane its own pieces)
            const float inv = 1.0f / (float)NFFT;
#define MONARCH_C16K_K_TILE(T, Q)                                                          \
    {                                                                                      \
        f32x4 re, im;                                                                      \
        row_tile<Q, 4, true>(half_rows<T>(A.re[Q]), half_rows<T>(A.im[Q]), by, re, im);   \
        kf[(4 * T + Q) * 64] = u32x4{pack2(re[0] * inv, im[0] * inv), pack2(re[1] * inv, im[1] * inv),     \
                                     pack2(re[2] * inv, im[2] * inv), pack2(re[3] * inv, im[3] * inv)};     \
    }
            MONARCH_C16K_K_TILE(0, 0) MONARCH_C16K_K_TILE(0, 1) MONARCH_C16K_K_TILE(0, 2) MONARCH_C16K_K_TILE(0, 3)
            MONARCH_C16K_K_TILE(1, 0) MONARCH_C16K_K_TILE(1, 1) MONARCH_C16K_K_TILE(1, 2) MONARCH_C16K_K_TILE(1, 3)
#undef MONARCH_C16K_K_TILE
            __syncthreads();   // every wave has read its rows: the next job's rows may overwrite the tile
            deposit(g + 1);    // (a pair job always follows a kernel job)
            __syncthreads();
            continue;
        }

        // ---- times k_f, conjugated (the inverse is conj o F o conj), straight into the B operands of stage Y':
        //      block 2T + (r>>1), word 2 (r&1) + (q>>1), half q&1
        Bops bz;
#define MONARCH_C16K_Y_PAIR(T, QP)                                                                              \
    {                                                                                                            \
        f32x4 re0, im0, re1, im1;                                                                                \
        row_tile<2 * QP, 4, true>(half_rows<T>(A.re[2 * QP]), half_rows<T>(A.im[2 * QP]), by, re0, im0);         \
        row_tile<2 * QP + 1, 4, true>(half_rows<T>(A.re[2 * QP + 1]), half_rows<T>(A.im[2 * QP + 1]), by, re1, im1); \
        const u32x4 kq0 = kf[(4 * T + 2 * QP) * 64], kq1 = kf[(4 * T + 2 * QP + 1) * 64];                         \
        _Pragma("unroll") for (int r = 0; r < 4; ++r) {                                                         \
            const uint32_t k0 = kq0[r], k1 = kq1[r];                                                             \
            const float2 p0 = cmul(make_float2(re0[r], im0[r]), make_float2(lo_f32(k0), hi_f32(k0)));            \
            const float2 p1 = cmul(make_float2(re1[r], im1[r]), make_float2(lo_f32(k1), hi_f32(k1)));            \
            bz.re[2 * T + (r >> 1)][2 * (r & 1) + QP] = pack2(p0.x, p1.x);                                       \
            bz.im[2 * T + (r >> 1)][2 * (r & 1) + QP] = pack2(-p0.y, -p1.y);                                     \
        }                                                                                                        \
    }
        MONARCH_C16K_Y_PAIR(0, 0) MONARCH_C16K_Y_PAIR(0, 1) MONARCH_C16K_Y_PAIR(1, 0) MONARCH_C16K_Y_PAIR(1, 1)
#undef MONARCH_C16K_Y_PAIR

        // ---- stage Y': contract j2 along the same rows, twiddle, back into the tile (positions c2)
        {
            Twiddle tw;
            tw.init(yrow, kg);
            uint32_t *line = tile + yrow * PITCH;
#define MONARCH_C16K_YI_HALF(T)                                                                                 \
    {                                                                                                            \
        uint32_t o[4][4];                                                                                        \
        _Pragma("unroll") for (int q = 0; q < 4; ++q) {                                                         \
            f32x4 re, im;                                                                                        \
            switch (q) {                                                                                         \
            case 0: row_tile<0, 4, true>(half_rows<T>(A.re[0]), half_rows<T>(A.im[0]), bz, re, im); break;       \
            case 1: row_tile<1, 4, true>(half_rows<T>(A.re[1]), half_rows<T>(A.im[1]), bz, re, im); break;       \
            case 2: row_tile<2, 4, true>(half_rows<T>(A.re[2]), half_rows<T>(A.im[2]), bz, re, im); break;       \
            default: row_tile<3, 4, true>(half_rows<T>(A.re[3]), half_rows<T>(A.im[3]), bz, re, im); break;      \
            }                                                                                                    \
            _Pragma("unroll") for (int r = 0; r < 4; ++r) {                                                     \
                const float2 z = cmul(make_float2(re[r], im[r]), tw.cur[r]);                                     \
                o[q][r] = pack2(z.x, z.y);                                                                       \
            }                                                                                                    \
            tw.next_q();                                                                                         \
        }                                                                                                        \
        _Pragma("unroll") for (int rh = 0; rh < 2; ++rh) {                                                      \
            uint32_t *dst = line + ((64 * T + 32 * rh + 8 * kg) ^ yswz);                                         \
            *reinterpret_cast<u32x4 *>(dst) = u32x4{o[0][2 * rh], o[1][2 * rh], o[2][2 * rh], o[3][2 * rh]};     \
            *reinterpret_cast<u32x4 *>(dst + 4) = u32x4{o[0][2 * rh + 1], o[1][2 * rh + 1], o[2][2 * rh + 1], o[3][2 * rh + 1]}; \
        }                                                                                                        \
    }
            MONARCH_C16K_YI_HALF(0)
            tw.next_t();
            MONARCH_C16K_YI_HALF(1)
#undef MONARCH_C16K_YI_HALF
        }
        __syncthreads();

        // this pair's output gates travel while the last stage runs
        const size_t ra = ((size_t)b0 * H + h) * n, rb = ra + (size_t)H * n, rb_or_ra = hasb ? rb : ra;
        if (GOUT) {
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int e = 8 * (tid + it * THREADS), ee = e < n ? e : 0;
                oga[it] = load_here(g_out + ra + ee);
                ogb[it] = load_here(g_out + rb_or_ra + ee);
            }
        }

        // ---- stage X': contract j1 down this wave's columns; only rows c1 < 64 are kept (truncation to n)
        {
            Bops b;
            read_columns(b, 4);
#define MONARCH_C16K_XI_TILE(Q)                                                                 \
    {                                                                                            \
        f32x4 re, im;                                                                            \
        row_tile<Q, 4, true>(A.re[Q], A.im[Q], b, re, im);                                       \
        _Pragma("unroll") for (int r = 0; r < 4; ++r)                                           \
            tile[xbase + (32 * (r >> 1) + 4 * (r & 1) + Q) * PITCH] = pack2(re[r], im[r]);       \
    }
            MONARCH_C16K_XI_TILE(0) MONARCH_C16K_XI_TILE(1) MONARCH_C16K_XI_TILE(2) MONARCH_C16K_XI_TILE(3)
#undef MONARCH_C16K_XI_TILE
        }
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);   // nothing of the store pass (it waits for the gates) moves up into the stage

        // ---- tile -> rows: F^-1 = conj(F conj(.)) / N (the 1/N sits in k_f): first row = Re, second = -Im.
        //      All arithmetic comes first, unconditionally, and only the stores at the end are guarded, so that the
        //      loads of the gates stay where they were issued (a load whose uses all sit under a condition is moved
        //      down into it, past the stage it was meant to overlap).
        u32x4 ya[2], yb[2];
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int e = 8 * (tid + it * THREADS), row = e >> 7, col = e & 127;
            const uint32_t *src = tile + row * PITCH + swz(row, col);
            const u32x4 w0 = *reinterpret_cast<const u32x4 *>(src), w1 = *reinterpret_cast<const u32x4 *>(src + 4);
            float va[8], vb[8], gt[8];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                va[t] = lo_f32(w0[t]);
                vb[t] = -hi_f32(w0[t]);
                va[4 + t] = lo_f32(w1[t]);
                vb[4 + t] = -hi_f32(w1[t]);
            }
            if (GOUT) {
                unpack8(oga[it], gt);
#pragma unroll
                for (int t = 0; t < 8; ++t) va[t] *= gt[t];
                unpack8(ogb[it], gt);
#pragma unroll
                for (int t = 0; t < 8; ++t) vb[t] *= gt[t];
            }
            ya[it] = u32x4{pack2(va[0], va[1]), pack2(va[2], va[3]), pack2(va[4], va[5]), pack2(va[6], va[7])};
            yb[it] = u32x4{pack2(vb[0], vb[1]), pack2(vb[2], vb[3]), pack2(vb[4], vb[5]), pack2(vb[6], vb[7])};
        }
        asm volatile("" : "+v"(ya[0]), "+v"(ya[1]), "+v"(yb[0]), "+v"(yb[1]));   // computed here, not inside the tests
        // the next job's rows go into the tile words this thread has just read; the stores come last, so that
        // nothing waits for them
        if (more) deposit(g + 1);
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int e = 8 * (tid + it * THREADS);
            if (e < n) {
                __builtin_nontemporal_store(ya[it], reinterpret_cast<u32x4 *>(y + ra + e));
                if (hasb) __builtin_nontemporal_store(yb[it], reinterpret_cast<u32x4 *>(y + rb + e));
            }
        }
        __syncthreads();   // the next job's rows are in the tile
    }
}

}  // namespace c16k

bool conv_mfma_16k_supported(int n, int klen, const int *factors, int nf, monarch_dtype dt)
{
    return dt == MONARCH_BF16 && nf == 2 && factors[0] == 128 && factors[1] == 128 && n <= c16k::NMAX &&
           klen <= c16k::NMAX && n % 8 == 0 && klen % 8 == 0;
}

int launch_conv_mfma_16k(const void *u, const void *k, const void *g_in, const void *g_out, void *y,
                         int B, int H, int n, int klen, hipStream_t s)
{
    int dev = 0, ncu = 0;
    MONARCH_HIP_CHECK(hipGetDevice(&dev));
    MONARCH_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
    const int grid = H < ncu ? H : ncu;   // one workgroup per compute unit, channels h = block, block + grid, ...
    const size_t lds = (size_t)c16k::TILE_WORDS * sizeof(uint32_t) + (size_t)8 * 8 * 64 * 16;   // the tile and k_f
#define MONARCH_LAUNCH_C16K(GINV, GOUTV)                                                                          \
    do {                                                                                                          \
        auto kern = c16k::conv16k_bf16_kernel<GINV, GOUTV>;                                                       \
        MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)); \
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(c16k::THREADS), lds, s, (const bf16_t *)u,            \
                           (const bf16_t *)k, (const bf16_t *)g_in, (const bf16_t *)g_out, (bf16_t *)y, B, H, n, klen); \
    } while (0)
    switch ((g_in ? 2 : 0) | (g_out ? 1 : 0)) {
    case 3: MONARCH_LAUNCH_C16K(true, true); break;
    case 2: MONARCH_LAUNCH_C16K(true, false); break;
    case 1: MONARCH_LAUNCH_C16K(false, true); break;
    default: MONARCH_LAUNCH_C16K(false, false); break;
    }
#undef MONARCH_LAUNCH_C16K
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

}  // namespace monarch
