// Fused gated causal Monarch-FFT convolution, nfft = 2048 = 64 x 32, bf16 or fp16 I/O, fp32 accumulate.
//
// A workgroup (4 waves) takes a work item (channel h, chunk of batch pairs): it first turns k[h]
// into its spectrum k_f (one quarter per wave, kept in LDS), then every wave takes PAIRS of batch
// rows of that channel and runs the whole chain
//   pad -> Monarch DFT -> (.) k_f -> inverse Monarch DFT -> truncate -> gate
// in registers:
//
//   * two real rows ride as one complex row z = x0 + i x1 (the kernel is real, so the
//     convolution of z is conv(x0) + i conv(x1)): half the transforms;
//   * the row is the N1 x N2 = 64 x 32 matrix x[c*32 + a]; the Monarch factors are
//     R = I (x) F_64 (contract c), twiddle w_2048^(i a), L = F_32 blocks (contract a);
//     the zero-padded half (c >= 32) is never multiplied and only outputs c < 32 are formed;
//   * every factor is a 16-bit MFMA (16x16x32, bf16 or fp16) with the constant DFT matrix as one operand and
//     the previous stage's accumulators, re-rounded to 16 bits, as the other.  Two stacked
//     accumulator tiles (32 rows in registers, 16 columns on lanes) are a valid B operand
//     (contract the rows, keep the columns on lanes) and equally a valid A operand (contract the
//     rows, the lane index becomes the new row index), so no stage needs a transpose: the
//     permutations P of M = P L P R P never exist as data movement, not even in LDS;
//   * the spectrum is walked in four chunks of 16 columns, which keeps the live fp32 tiles small
//     enough for three waves per SIMD: all workgroups of the benchmark shape are resident at
//     once and hide each other's MFMA, LDS and HBM latencies;
//   * twiddles, the spectrum product and the gates are fp32 on the accumulators.
//
// Appendix DFT corollary (Monarch form of F_N), Sec. 3.2 Eq. 2 with gating, Thm 3 (padding).
#include "const_roots.h"
#include "half16.h"
#include "kernels.h"

namespace monarch {

using h16::f32x4;
using h16::hi32;
using h16::lo32;
using h16::mfma;
using h16::op8;
using h16::pack16;

namespace c2048 {

constexpr int N1 = 64, N2 = 32, NFFT = 2048, NHALF = 1024;
constexpr int TW_LD = 34;        // padded row length (complex) of the twiddle table
#ifndef MONARCH_C2048_WAVES
#define MONARCH_C2048_WAVES 3
#endif
constexpr int WAVES_PER_SIMD = MONARCH_C2048_WAVES;   // the register budget (512 / 3) the kernel is written for

constexpr int ST_LD = 36;        // padded row length (words) of a staging tile: lane groups 4 rows
                                 // apart fall on different LDS banks

struct Smem {
    float2 tw[N1][TW_LD];        // w_2048^(i*a), i < 64, a < 32
    float4 kf_re[4][2][64];      // k_f / NFFT in accumulator layout [chunk][row tile][lane]
    float4 kf_im[4][2][64];
    uint32_t stage[4][32 * ST_LD];   // per wave: (re bf16 | im bf16 << 16) at [c*ST_LD + a]
};

// ---- constant tables, evaluated by the compiler --------------------------------------------
using croots::CosSin;
using croots::bf16_bits;
using croots::unit_root;
constexpr int cslot(int kg, int j) { return 16 * (j >> 2) + 4 * kg + (j & 3); }

// fp16 bits of a value of magnitude <= 1 (a cosine or sine): round to nearest even; the tables hold no value
// between 0 and the smallest normal number (the smallest non-zero one is sin(2 pi / 2048)).
constexpr uint32_t f16_bits(double v)
{
    if (v == 0.0) return 0u;
    const uint32_t sign = v < 0 ? 0x8000u : 0u;
    double a = v < 0 ? -v : v;
    int e = 0;
    while (a < 1.0) { a *= 2.0; --e; }
    while (a >= 2.0) { a *= 0.5; ++e; }
    // a in [1, 2): 10 fraction bits
    double f = (a - 1.0) * 1024.0;
    uint32_t m = (uint32_t)f;
    const double rest = f - (double)m;
    if (rest > 0.5 || (rest == 0.5 && (m & 1u))) ++m;
    uint32_t ebits = (uint32_t)(e + 15);
    if (m == 1024u) { m = 0u; ++ebits; }
    return sign | (ebits << 10) | m;
}
template <typename E> constexpr uint32_t half_bits(double v);
template <> constexpr uint32_t half_bits<bf16_t>(double v) { return bf16_bits(v); }
template <> constexpr uint32_t half_bits<f16_t>(double v) { return f16_bits(v); }

struct TwiddleTable { float v[N1][N2][2]; };   // unpadded in memory (16 KB); the copy in LDS has rows of TW_LD
constexpr TwiddleTable make_twiddles()
{
    TwiddleTable t{};
    for (int i = 0; i < N1; ++i)
        for (int a = 0; a < N2; ++a) {
            const CosSin w = unit_root(i * a, NFFT);
            t.v[i][a][0] = (float)w.c;
            t.v[i][a][1] = (float)w.s;
        }
    return t;
}
// Per-lane constant MFMA operands, 8 x 16 bytes per lane:
//   [2t], [2t+1]: real / imaginary part of F64[slot][16t + lane%16]  (= F64[16t + lane%16][slot])
//   [4+2t], [5+2t]: real / imaginary part of F32[16t + lane%16][slot]
struct OperandTable { uint32_t v[64][8][4]; };
template <typename E>
constexpr OperandTable make_operands()
{
    OperandTable t{};
    for (int lane = 0; lane < 64; ++lane)
        for (int tile = 0; tile < 2; ++tile)
            for (int jj = 0; jj < 4; ++jj) {
                const int row = 16 * tile + (lane & 15), s0 = cslot(lane >> 4, 2 * jj);
                const CosSin f0 = unit_root(s0 * row, 64), f1 = unit_root((s0 + 1) * row, 64);
                const CosSin g0 = unit_root(s0 * row, 32), g1 = unit_root((s0 + 1) * row, 32);
                t.v[lane][2 * tile][jj] = half_bits<E>(f0.c) | (half_bits<E>(f1.c) << 16);
                t.v[lane][2 * tile + 1][jj] = half_bits<E>(f0.s) | (half_bits<E>(f1.s) << 16);
                t.v[lane][4 + 2 * tile][jj] = half_bits<E>(g0.c) | (half_bits<E>(g1.c) << 16);
                t.v[lane][5 + 2 * tile][jj] = half_bits<E>(g0.s) | (half_bits<E>(g1.s) << 16);
            }
    return t;
}
__device__ const TwiddleTable g_twiddles = make_twiddles();
__device__ const OperandTable g_operands_bf16 = make_operands<bf16_t>();
__device__ const OperandTable g_operands_f16 = make_operands<f16_t>();
template <typename E> __device__ __forceinline__ const OperandTable &operands();
template <> __device__ __forceinline__ const OperandTable &operands<bf16_t>() { return g_operands_bf16; }
template <> __device__ __forceinline__ const OperandTable &operands<f16_t>() { return g_operands_f16; }

union Pack8 {
    op8 v;
    uint32_t d[4];
};

struct COp { op8 r, i, ni; };    // constant complex operand: real part, imaginary part and its negative

// (The element type E, bf16_t or f16_t, only shows in the helpers of half16.h, the constant tables and the
// two-term dot product of the gating.)

// Contraction index carried by operand slot j of lane group kg when the operand is made from two
// stacked 16x16 accumulator tiles: tile j/4, register j%4 holds row 16*(j/4) + 4*kg + j%4.
__device__ __forceinline__ int slot_index(int kg, int j) { return 16 * (j >> 2) + 4 * kg + (j & 3); }

// Sign flips on packed 16-bit operands (bit 15 of each half is the sign in both types).
__device__ __forceinline__ op8 flip(op8 v, uint32_t mask) { return v ^ mask; }
__device__ __forceinline__ op8 neg_all(op8 v) { return flip(v, 0x80008000u); }

// Two stacked accumulator tiles -> one 16-bit operand (slot 4*t + r <- tile t, register r).
template <typename E> __device__ __forceinline__ op8 pack_tiles(const f32x4 &t0, const f32x4 &t1)
{
    return op8{pack16<E>(t0[0], t0[1]), pack16<E>(t0[2], t0[3]), pack16<E>(t1[0], t1[1]), pack16<E>(t1[2], t1[3])};
}

// Rows of u, the gates and y are touched once per launch: their loads and stores carry the non-temporal hint, so
// that they do not displace the constant tables and k in L2 and the output leaves no dirty lines behind for the end of
// the kernel (measured on config 2, same box: 18.4 us with ordinary accesses, 16.7 us with streaming stores, 15.8 us
// with streaming loads too, 15.2 us when k, which four waves read, keeps ordinary loads).
// 8 consecutive bf16 of a row (chunk ch), zero past the end of the row.  FULL: the row has all
// 128 chunks, so the load is unconditional (no exec-mask branch per load).
template <bool FULL, bool STREAM, typename E>
__device__ __forceinline__ uint4 load_chunk(const E *row, int ch, int len)
{
    if (FULL || ch * 8 < len) {
        return STREAM ? load_stream16(row + ch * 8) : *reinterpret_cast<const uint4 *>(row + ch * 8);
    }
    return make_uint4(0u, 0u, 0u, 0u);
}

// Raw rows as loaded: chunks lane and lane+64 of two rows (the second may be absent).
struct RowLoad { uint4 a[2], b[2]; };

// Both pointers must be valid rows (no null checks: the loads stay free of branches).
template <bool FULL, bool STREAM, typename E>
__device__ __forceinline__ void load_rows(RowLoad &ld, int lane, const E *r0, const E *r1, int len)
{
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const int ch = lane + 64 * half;
        ld.a[half] = load_chunk<FULL, STREAM, E>(r0, ch, len);
        ld.b[half] = load_chunk<FULL, STREAM, E>(r1, ch, len);
    }
}

// One row only (the kernel k, read by all four waves: ordinary loads); the second row of the pair is zero.
template <bool FULL, typename E>
__device__ __forceinline__ void load_row(RowLoad &ld, int lane, const E *r0, int len)
{
    const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        ld.a[half] = load_chunk<FULL, false, E>(r0, lane + 64 * half, len);
        ld.b[half] = zero;
    }
}

// (lo | hi << 16) interleave of two packed rows: element e of each into word e.
__device__ __forceinline__ void interleave_store(uint32_t *dst, const uint32_t (&r)[4], const uint32_t (&m)[4])
{
    uint4 o0, o1;
    o0.x = __builtin_amdgcn_perm(m[0], r[0], 0x05040100u); o0.y = __builtin_amdgcn_perm(m[0], r[0], 0x07060302u);
    o0.z = __builtin_amdgcn_perm(m[1], r[1], 0x05040100u); o0.w = __builtin_amdgcn_perm(m[1], r[1], 0x07060302u);
    o1.x = __builtin_amdgcn_perm(m[2], r[2], 0x05040100u); o1.y = __builtin_amdgcn_perm(m[2], r[2], 0x07060302u);
    o1.z = __builtin_amdgcn_perm(m[3], r[3], 0x05040100u); o1.w = __builtin_amdgcn_perm(m[3], r[3], 0x07060302u);
    reinterpret_cast<uint4 *>(dst)[0] = o0;
    reinterpret_cast<uint4 *>(dst)[1] = o1;
}

// d[i] = x_i.lo * g_i.lo + x_i.hi * g_i.hi of packed 16-bit pairs, in fp32 (exact when one of the products is
// zero), for i = 0..3 with x = (x0, x1, x0, x1).  One block of assembly that ends with the three wait states a
// dot product's result needs before another kind of vector instruction may read it: the compiler inserts them
// only for instructions it can see.
template <typename E> __device__ __forceinline__ void dot2x4(uint32_t x0, uint32_t x1, uint32_t g0, uint32_t g1, uint32_t g2, uint32_t g3, float (&d)[4]);
template <> __device__ __forceinline__ void dot2x4<bf16_t>(uint32_t x0, uint32_t x1, uint32_t g0, uint32_t g1, uint32_t g2, uint32_t g3, float (&d)[4])
{
    asm("v_dot2_f32_bf16 %0, %4, %6, 0\n\tv_dot2_f32_bf16 %1, %5, %7, 0\n\tv_dot2_f32_bf16 %2, %4, %8, 0\n\tv_dot2_f32_bf16 %3, %5, %9, 0\n\ts_nop 2"
        : "=&v"(d[0]), "=&v"(d[1]), "=&v"(d[2]), "=&v"(d[3])
        : "v"(x0), "v"(x1), "v"(g0), "v"(g1), "v"(g2), "v"(g3));
}
template <> __device__ __forceinline__ void dot2x4<f16_t>(uint32_t x0, uint32_t x1, uint32_t g0, uint32_t g1, uint32_t g2, uint32_t g3, float (&d)[4])
{
    asm("v_dot2_f32_f16 %0, %4, %6, 0\n\tv_dot2_f32_f16 %1, %5, %7, 0\n\tv_dot2_f32_f16 %2, %4, %8, 0\n\tv_dot2_f32_f16 %3, %5, %9, 0\n\ts_nop 2"
        : "=&v"(d[0]), "=&v"(d[1]), "=&v"(d[2]), "=&v"(d[3])
        : "v"(x0), "v"(x1), "v"(g0), "v"(g1), "v"(g2), "v"(g3));
}

// Writes two rows into the wave's staging tile as (row a | row b << 16) words at [c*ST_LD + a'],
// multiplied elementwise by the gate rows when `gated`.  Gated: each product of two 16-bit values is one
// two-term dot product against the gate word with its other half masked away (exact in fp32), and the
// rounding of the products of the two rows to 16 bits is the instruction that interleaves them.
template <typename E>
__device__ __forceinline__ void stage_rows(uint32_t *stage, int lane, const RowLoad &x, const RowLoad &gt, bool gated)
{
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const int ch = lane + 64 * half;
        const uint32_t r[4] = {x.a[half].x, x.a[half].y, x.a[half].z, x.a[half].w};
        const uint32_t m[4] = {x.b[half].x, x.b[half].y, x.b[half].z, x.b[half].w};
        uint32_t *dst = stage + (ch >> 2) * ST_LD + (ch & 3) * 8;
        if (gated) {
            const uint32_t ga[4] = {gt.a[half].x, gt.a[half].y, gt.a[half].z, gt.a[half].w};
            const uint32_t gb[4] = {gt.b[half].x, gt.b[half].y, gt.b[half].z, gt.b[half].w};
            uint32_t o[8];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float d[4];
                dot2x4<E>(r[q], m[q], ga[q] & 0xffffu, gb[q] & 0xffffu, ga[q] & 0xffff0000u, gb[q] & 0xffff0000u, d);
                o[2 * q] = pack16<E>(d[0], d[1]);
                o[2 * q + 1] = pack16<E>(d[2], d[3]);
            }
            reinterpret_cast<uint4 *>(dst)[0] = make_uint4(o[0], o[1], o[2], o[3]);
            reinterpret_cast<uint4 *>(dst)[1] = make_uint4(o[4], o[5], o[6], o[7]);
        } else {
            interleave_store(dst, r, m);
        }
    }
}

// A operands of the first factor: for row tile m, lane (a = 16m + lane%16, kg) holds x[c][a]
// for the 8 contraction indices c = slot_index(kg, j).
__device__ __forceinline__ void read_stage_operands(const uint32_t *stage, int l16, int kg, op8 (&xr)[2], op8 (&xi)[2])
{
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        Pack8 pr, pi;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const int c0 = slot_index(kg, 2 * jj);
            const uint32_t d0 = stage[c0 * ST_LD + 16 * m + l16];
            const uint32_t d1 = stage[(c0 + 1) * ST_LD + 16 * m + l16];
            pr.d[jj] = __builtin_amdgcn_perm(d1, d0, 0x05040100u);
            pi.d[jj] = __builtin_amdgcn_perm(d1, d0, 0x07060302u);
        }
        xr[m] = pr.v;
        xi[m] = pi.v;
    }
}

// Forward transform of spectrum columns i = 16*CH + lane%16:
//   Z1[a,i] = sum_c x[c,a] F64[c,i];  Z1 *= w_2048^(i a);  Z2[k,i] = sum_a F32[k,a] Z1[a,i].
// F holds F64[c][16*(CH%2) + lane%16]; columns 32..63 differ from it by (-1)^c, which the caller
// has applied to the data operands (odd slots negated) for CH >= 2.
// Result: rows k = 16m + 4kg + r in registers (z2[m][r]), column i on the lane.
template <typename E, int CH, bool HAS_IM>
__device__ __forceinline__ void forward_chunk(const Smem &sm, int l16, int kg, const op8 (&xr)[2],
                                              const op8 (&xi)[2], const COp &F, const COp (&G)[2],
                                              f32x4 (&z2r)[2], f32x4 (&z2i)[2])
{
    f32x4 zr[2], zi[2];
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        zr[m] = mfma<E>(xr[m], F.r, (f32x4){0, 0, 0, 0});
        zi[m] = mfma<E>(xr[m], F.i, (f32x4){0, 0, 0, 0});
        if (HAS_IM) {
            zr[m] = mfma<E>(xi[m], F.ni, zr[m]);
            zi[m] = mfma<E>(xi[m], F.r, zi[m]);
        }
    }
    // twiddle: rows a = 16m + 4kg + r in registers, column i on the lane
    const float2 *trow = sm.tw[16 * CH + l16] + 4 * kg;
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        const float4 t01 = *reinterpret_cast<const float4 *>(trow + 16 * m);
        const float4 t23 = *reinterpret_cast<const float4 *>(trow + 16 * m + 2);
        const float tr[4] = {t01.x, t01.z, t23.x, t23.z}, ti[4] = {t01.y, t01.w, t23.y, t23.w};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float a = zr[m][r], b = zi[m][r];
            zr[m][r] = a * tr[r] - b * ti[r];
            zi[m][r] = a * ti[r] + b * tr[r];
        }
    }
    const op8 br = pack_tiles<E>(zr[0], zr[1]), bi = pack_tiles<E>(zi[0], zi[1]);
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        z2r[m] = mfma<E>(G[m].r, br, (f32x4){0, 0, 0, 0});
        z2i[m] = mfma<E>(G[m].i, br, (f32x4){0, 0, 0, 0});
        z2r[m] = mfma<E>(G[m].ni, bi, z2r[m]);
        z2i[m] = mfma<E>(G[m].r, bi, z2i[m]);
    }
}

// Spectrum product, third factor and conjugate twiddle for columns i = 16*CH + ...; writes this
// chunk's 16 contraction rows into the last factor's B operands (half of each operand).
template <typename E, int CH>
__device__ __forceinline__ void inverse_chunk(const Smem &sm, int lane, int l16, int kg, f32x4 (&zr)[2],
                                              f32x4 (&zi)[2], const COp (&G)[2], Pack8 (&wr_op)[2], Pack8 (&wi_op)[2])
{
    // Y = Z2 (.) k_f   (rows k in registers, column i on the lane)
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        const float4 kr = sm.kf_re[CH][m][lane], ki = sm.kf_im[CH][m][lane];
        const float kre[4] = {kr.x, kr.y, kr.z, kr.w}, kim[4] = {ki.x, ki.y, ki.z, ki.w};
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float a = zr[m][r], b = zi[m][r];
            zr[m][r] = a * kre[r] - b * kim[r];
            zi[m][r] = a * kim[r] + b * kre[r];
        }
    }
    // third factor: W[i,a] = sum_k Y[i,k] conj(F32)[k,a]; Y's lane index i becomes the row index
    const op8 ar = pack_tiles<E>(zr[0], zr[1]), ai = pack_tiles<E>(zi[0], zi[1]);
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
        f32x4 wr = mfma<E>(ar, G[nt].r, (f32x4){0, 0, 0, 0});
        f32x4 wi = mfma<E>(ai, G[nt].r, (f32x4){0, 0, 0, 0});
        wr = mfma<E>(ai, G[nt].i, wr);
        wi = mfma<E>(ar, G[nt].ni, wi);
        // conjugate twiddle: rows i = 16*CH + 4kg + r in registers, column a = 16nt + lane%16
        const float2 *tcol = &sm.tw[16 * CH + 4 * kg][16 * nt + l16];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float2 w = tcol[r * TW_LD];
            const float a = wr[r], b = wi[r];
            wr[r] = a * w.x + b * w.y;
            wi[r] = b * w.x - a * w.y;
        }
        // contraction rows 32*(CH/2) + 16*(CH%2) + 4kg + r  ->  slots 4*(CH%2) + r of kstep CH/2
        wr_op[nt].d[2 * (CH & 1)] = pack16<E>(wr[0], wr[1]);
        wr_op[nt].d[2 * (CH & 1) + 1] = pack16<E>(wr[2], wr[3]);
        wi_op[nt].d[2 * (CH & 1)] = pack16<E>(wi[0], wi[1]);
        wi_op[nt].d[2 * (CH & 1) + 1] = pack16<E>(wi[2], wi[3]);
    }
}

// FULL: n == klen == 1024, every row load is unconditional.  GIN / GOUT: the gates are present.
// Keeping the loads free of branches lets the compiler wait for exactly the load it needs
// (k first, then u and g_in, g_out last) instead of draining all of them at once.
// HEADS (the gated-convolution layer with heads of dh features): the batch index of the
// convolution is ((b dh + i) dh + j) and the channel the head; u is read from row (b, head dh + j) and g_in from row
// (b, head dh + i) of tensors of d = H dh channels, so the outer products X2[i] o V[j] of a head are formed on the loads
// and never stored.  y keeps the plain (batch, channel) rows.
template <typename E, bool FULL, bool GIN, bool GOUT, bool HEADS = false>
__global__ __launch_bounds__(256, WAVES_PER_SIMD) void conv2048_kernel(
    const E *__restrict__ u, const E *__restrict__ k, const E *__restrict__ g_in,
    const E *__restrict__ g_out, E *__restrict__ y, int B, int H, int n, int klen, int dh = 1)
{
    __shared__ Smem sm;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, l16 = lane & 15, kg = lane >> 4;
    uint32_t *stage = sm.stage[wave];
    // work item = (channel h, group of 4 pairs); wave w of the group takes pair 4*group + w
    const int h = blockIdx.x % H;
    const int p = 4 * (blockIdx.x / H) + wave;
    const bool active = 2 * p < B, two = 2 * p + 1 < B;
    // rows of this wave's pair; a missing row is replaced by a valid one so that the loads need no
    // branch (its data is ignored: the imaginary part is forced to zero, the store is skipped)
    const int b0 = active ? 2 * p : 0, b1 = two ? 2 * p + 1 : b0;
    const size_t row0 = ((size_t)b0 * H + h) * n, row1 = ((size_t)b1 * H + h) * n;
    size_t urow0 = row0, urow1 = row1, grow0 = row0, grow1 = row1;
    if constexpr (HEADS) {
        const int d = H * dh, dd = dh * dh;
        urow0 = ((size_t)(b0 / dd) * d + h * dh + b0 % dh) * n;
        urow1 = ((size_t)(b1 / dd) * d + h * dh + b1 % dh) * n;
        grow0 = ((size_t)(b0 / dd) * d + h * dh + (b0 / dh) % dh) * n;
        grow1 = ((size_t)(b1 / dd) * d + h * dh + (b1 / dh) % dh) * n;
    }

    // Constant tables first (they come from L2 and gate everything else), then the rows.
    static_assert(sizeof(TwiddleTable) == 4 * 256 * sizeof(uint4), "twiddle copy assumes 1024 pieces of two entries");
    const uint4 *tw_src = reinterpret_cast<const uint4 *>(&g_twiddles);
    const uint4 tw0 = tw_src[tid], tw1 = tw_src[tid + 256], tw2 = tw_src[tid + 512], tw3 = tw_src[tid + 768];
    // The per-lane operand table (8 KB, the same for the four waves) is fetched once per workgroup: two pieces per
    // thread, through the area of LDS that k_f fills later (each lane fetching its own 128 bytes, 32 KB per workgroup,
    // cost 3.5 %: the constants share the compute unit's vector memory path with the rows).
    const uint4 *ops_src = reinterpret_cast<const uint4 *>(&operands<E>());
    const uint4 op0 = ops_src[tid], op1 = ops_src[tid + 256];
    // k is staged once for the four waves: thread t brings elements 4 t .. 4 t + 3 (ordinary loads: 8 bytes per lane)
    RowLoad ldx, ldg, ldo;
    uint2 kraw = make_uint2(0u, 0u);
    if (FULL || 4 * tid < klen) kraw = *reinterpret_cast<const uint2 *>(k + (size_t)h * klen + 4 * tid);
    load_rows<FULL, !HEADS, E>(ldx, lane, u + urow0, u + urow1, n);   // (with heads a row is read dh times: ordinary loads)

    if (GIN) load_rows<FULL, !HEADS, E>(ldg, lane, g_in + grow0, g_in + grow1, n);
    {
        // piece p = entries (i, a), (i, a + 1) with i = p / 16, a = 2 (p % 16): rows of TW_LD entries in LDS (16-byte aligned:
        // TW_LD and a are even)
        static_assert(TW_LD % 2 == 0 && N2 == 32, "twiddle pieces");
        const uint4 twv[4] = {tw0, tw1, tw2, tw3};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int p = tid + 256 * q;
            *reinterpret_cast<uint4 *>(&sm.tw[p >> 4][2 * (p & 15)]) = twv[q];
        }
    }
    {   // k into the first wave's staging tile, imaginary halves zero (same word layout as stage_rows)
        const int ch = tid >> 1;
        uint32_t *dst = sm.stage[0] + (ch >> 2) * ST_LD + (ch & 3) * 8 + 4 * (tid & 1);
        *reinterpret_cast<uint4 *>(dst) = make_uint4(kraw.x & 0xffffu, kraw.x >> 16, kraw.y & 0xffffu, kraw.y >> 16);
    }
    uint4 *ops_lds = reinterpret_cast<uint4 *>(&sm.kf_re[0][0][0]);   // piece j of lane l at [j][l]
    ops_lds[(tid & 7) * 64 + (tid >> 3)] = op0;
    ops_lds[(tid & 7) * 64 + 32 + (tid >> 3)] = op1;
    __syncthreads();   // twiddle and operand tables and k complete
    COp F[2], G[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        F[t].r = __builtin_bit_cast(op8, ops_lds[(2 * t) * 64 + lane]);
        F[t].i = __builtin_bit_cast(op8, ops_lds[(2 * t + 1) * 64 + lane]);
        G[t].r = __builtin_bit_cast(op8, ops_lds[(4 + 2 * t) * 64 + lane]);
        G[t].i = __builtin_bit_cast(op8, ops_lds[(5 + 2 * t) * 64 + lane]);
        F[t].ni = neg_all(F[t].i);
        G[t].ni = neg_all(G[t].i);
    }
    __syncthreads();   // every wave holds its operands: the area is free for k_f
    const uint32_t lane_sign = (l16 & 1) ? 0x80008000u : 0u;   // (-1)^(row of this lane) on every slot

    // spectrum of the kernel: wave w transforms spectrum columns 16w .. 16w+15
    {
        op8 xr[2], xi[2];
        read_stage_operands(sm.stage[0], l16, kg, xr, xi);   // (the first wave's tile is rewritten only after the next barrier)
        if (wave >= 2) {   // spectrum columns 32..63: (-1)^c on the data (odd slots)
            xr[0] = flip(xr[0], 0x80000000u);
            xr[1] = flip(xr[1], 0x80000000u);
        }
        f32x4 zr[2], zi[2];
        switch (wave) {
        case 0: forward_chunk<E, 0, false>(sm, l16, kg, xr, xi, F[0], G, zr, zi); break;
        case 1: forward_chunk<E, 1, false>(sm, l16, kg, xr, xi, F[1], G, zr, zi); break;
        case 2: forward_chunk<E, 2, false>(sm, l16, kg, xr, xi, F[0], G, zr, zi); break;
        default: forward_chunk<E, 3, false>(sm, l16, kg, xr, xi, F[1], G, zr, zi); break;
        }
        const float inv = 1.0f / (float)NFFT;
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            sm.kf_re[wave][m][lane] = make_float4(zr[m][0] * inv, zr[m][1] * inv, zr[m][2] * inv, zr[m][3] * inv);
            sm.kf_im[wave][m][lane] = make_float4(zi[m][0] * inv, zi[m][1] * inv, zi[m][2] * inv, zi[m][3] * inv);
        }
    }
    __syncthreads();   // k_f complete
    if (!active) return;
    if (!two) {   // single row: its partner's data was only a placeholder
        const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
        ldx.b[0] = ldx.b[1] = zero;
    }

    {
        {
            __builtin_amdgcn_wave_barrier();
            stage_rows<E>(stage, lane, ldx, ldg, GIN);
            __builtin_amdgcn_wave_barrier();
            op8 xr[2], xi[2];
            read_stage_operands(stage, l16, kg, xr, xi);
            __builtin_amdgcn_wave_barrier();
            // (the tile is free again)

            // B operands of the last factor: [kstep = contraction rows 32ks..32ks+31][column tile nt]
            Pack8 wr_op[2][2], wi_op[2][2];
            __builtin_amdgcn_sched_barrier(0);
            {
                f32x4 zr[2], zi[2];
                forward_chunk<E, 0, true>(sm, l16, kg, xr, xi, F[0], G, zr, zi);
                inverse_chunk<E, 0>(sm, lane, l16, kg, zr, zi, G, wr_op[0], wi_op[0]);
            }
            __builtin_amdgcn_sched_barrier(0);
            {
                f32x4 zr[2], zi[2];
                forward_chunk<E, 1, true>(sm, l16, kg, xr, xi, F[1], G, zr, zi);
                inverse_chunk<E, 1>(sm, lane, l16, kg, zr, zi, G, wr_op[0], wi_op[0]);
            }
            // The output gates are asked for here, half-way through the transforms: needed last, they queue behind the rows
            // that other workgroups of the compute unit still wait for (asked for before the transforms: +2 %).
            if (GOUT) load_rows<FULL, true, E>(ldo, lane, g_out + row0, g_out + row1, n);
            // spectrum columns 32..63 see F64[c][32 + i'] = (-1)^c F64[c][i']: negate the odd slots of the data
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                xr[m] = flip(xr[m], 0x80000000u);
                xi[m] = flip(xi[m], 0x80000000u);
            }
            __builtin_amdgcn_sched_barrier(0);
            {
                f32x4 zr[2], zi[2];
                forward_chunk<E, 2, true>(sm, l16, kg, xr, xi, F[0], G, zr, zi);
                inverse_chunk<E, 2>(sm, lane, l16, kg, zr, zi, G, wr_op[1], wi_op[1]);
            }
            __builtin_amdgcn_sched_barrier(0);
            {
                f32x4 zr[2], zi[2];
                forward_chunk<E, 3, true>(sm, l16, kg, xr, xi, F[1], G, zr, zi);
                inverse_chunk<E, 3>(sm, lane, l16, kg, zr, zi, G, wr_op[1], wi_op[1]);
            }
            __builtin_amdgcn_sched_barrier(0);
            // last factor: y[c,a] = sum_i conj(F64)[c,i] W[i,a], c < 32 only (truncation to n).
            // Contraction rows i >= 32 use F64[c][32+i'] = (-1)^c F64[c][i'], c being this lane's row.
            f32x4 yr[2][2], yi[2][2];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                const op8 hr = flip(F[mt].r, lane_sign), hi = flip(F[mt].i, lane_sign), nhi = flip(F[mt].ni, lane_sign);
#pragma unroll
                for (int nt = 0; nt < 2; ++nt) {
                    f32x4 ar = mfma<E>(F[mt].r, wr_op[0][nt].v, (f32x4){0, 0, 0, 0});
                    f32x4 ai = mfma<E>(F[mt].r, wi_op[0][nt].v, (f32x4){0, 0, 0, 0});
                    ar = mfma<E>(F[mt].i, wi_op[0][nt].v, ar);
                    ai = mfma<E>(F[mt].ni, wr_op[0][nt].v, ai);
                    ar = mfma<E>(hr, wr_op[1][nt].v, ar);
                    ai = mfma<E>(hr, wi_op[1][nt].v, ai);
                    ar = mfma<E>(hi, wi_op[1][nt].v, ar);
                    ai = mfma<E>(nhi, wr_op[1][nt].v, ai);
                    yr[mt][nt] = ar;
                    yi[mt][nt] = ai;
                }
            }
            // rows c = 16mt + 4kg + r, column a = 16nt + l16: gate in fp32, round once, park in the
            // staging tile (all gate words are read before the first result is written)
            __builtin_amdgcn_sched_barrier(0);
            // The output gates are parked in the staging tile (same word layout) only now: waiting for them before the
            // transforms put their arrival on the path of the workgroups that receive their rows last.
            if (GOUT) stage_rows<E>(stage, lane, ldo, ldo, false);
            __builtin_amdgcn_wave_barrier();
            uint32_t gw[2][2][4];
            if (GOUT) {
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                        for (int r = 0; r < 4; ++r) gw[mt][nt][r] = stage[(16 * mt + 4 * kg + r) * ST_LD + 16 * nt + l16];
            }
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int nt = 0; nt < 2; ++nt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        float v0 = yr[mt][nt][r], v1 = yi[mt][nt][r];
                        if (GOUT) {
                            v0 *= lo32<E>(gw[mt][nt][r]);
                            v1 *= hi32<E>(gw[mt][nt][r]);
                        }
                        stage[(16 * mt + 4 * kg + r) * ST_LD + 16 * nt + l16] = pack16<E>(v0, v1);
                    }
            __builtin_amdgcn_wave_barrier();
            // coalesced stores: lane takes chunks lane and lane+64 of both rows
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int ch = lane + 64 * half;
                if (!FULL && ch * 8 >= n) continue;
                const uint4 *src = reinterpret_cast<const uint4 *>(stage + (ch >> 2) * ST_LD + (ch & 3) * 8);
                const uint4 s0 = src[0], s1 = src[1];
                const uint32_t d[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
                uint32_t re[4], im[4];
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    re[jj] = __builtin_amdgcn_perm(d[2 * jj + 1], d[2 * jj], 0x05040100u);
                    im[jj] = __builtin_amdgcn_perm(d[2 * jj + 1], d[2 * jj], 0x07060302u);
                }
                store_stream16(y + row0 + ch * 8, make_uint4(re[0], re[1], re[2], re[3]));
                if (two) store_stream16(y + row1 + ch * 8, make_uint4(im[0], im[1], im[2], im[3]));
            }
        }
    }
}

}  // namespace c2048

bool conv_mfma_2048_supported(int n, int klen, const int *factors, int nf, monarch_dtype dt)
{
    return (dt == MONARCH_BF16 || dt == MONARCH_F16) && nf == 2 && factors[0] == 64 && factors[1] == 32 && n <= 1024 &&
           klen <= 1024 && n % 8 == 0 && klen % 8 == 0;
}

template <typename E>
static int launch_typed(const void *u, const void *k, const void *g_in, const void *g_out, void *y,
                        int B, int H, int n, int klen, hipStream_t s)
{
    // One workgroup per (channel, group of 4 batch pairs); with B <= 8 that is one per channel.
    const int64_t groups = ((B + 1) / 2 + 3) / 4;
    const int64_t grid = (int64_t)H * groups;
    if (grid > 0x7fffffffLL) return fail(MONARCH_ESHAPE, "B*H too large for one launch");
    const bool full = n == c2048::NHALF && klen == c2048::NHALF;
#define MONARCH_LAUNCH_C2048(FULLV, GINV, GOUTV)                                                                  \
    hipLaunchKernelGGL((c2048::conv2048_kernel<E, FULLV, GINV, GOUTV>), dim3((unsigned)grid), dim3(256), 0, s,    \
                       (const E *)u, (const E *)k, (const E *)g_in, (const E *)g_out, (E *)y, B, H, n, klen)
    switch ((full ? 4 : 0) | (g_in ? 2 : 0) | (g_out ? 1 : 0)) {
    case 7: MONARCH_LAUNCH_C2048(true, true, true); break;
    case 6: MONARCH_LAUNCH_C2048(true, true, false); break;
    case 5: MONARCH_LAUNCH_C2048(true, false, true); break;
    case 4: MONARCH_LAUNCH_C2048(true, false, false); break;
    case 3: MONARCH_LAUNCH_C2048(false, true, true); break;
    case 2: MONARCH_LAUNCH_C2048(false, true, false); break;
    case 1: MONARCH_LAUNCH_C2048(false, false, true); break;
    default: MONARCH_LAUNCH_C2048(false, false, false); break;
    }
#undef MONARCH_LAUNCH_C2048
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

// The long convolutions of the gated-convolution layer with heads: v, x2: (B, d, n) with d = heads dh; k: (heads, klen);
// yv: (B dh^2, heads, n), row ((b dh + i) dh + j, head) = conv(k[head], x2[b, head dh + i] o v[b, head dh + j]).
template <typename E>
static int launch_heads_typed(const void *v, const void *k, const void *x2, void *yv, int B, int heads, int dh, int n, int klen,
                              hipStream_t s)
{
    const int64_t cb = (int64_t)B * dh * dh, groups = ((cb + 1) / 2 + 3) / 4, grid = heads * groups;
    if (grid > 0x7fffffffLL) return fail(MONARCH_ESHAPE, "B*d*head_dim too large for one launch");
    if (n == c2048::NHALF && klen == c2048::NHALF)
        hipLaunchKernelGGL((c2048::conv2048_kernel<E, true, true, false, true>), dim3((unsigned)grid), dim3(256), 0, s, (const E *)v,
                           (const E *)k, (const E *)x2, (const E *)nullptr, (E *)yv, (int)cb, heads, n, klen, dh);
    else
        hipLaunchKernelGGL((c2048::conv2048_kernel<E, false, true, false, true>), dim3((unsigned)grid), dim3(256), 0, s, (const E *)v,
                           (const E *)k, (const E *)x2, (const E *)nullptr, (E *)yv, (int)cb, heads, n, klen, dh);
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

int launch_conv_mfma_2048_heads(const void *v, const void *k, const void *x2, void *yv, int B, int heads, int dh, int n, int klen,
                                monarch_dtype dt, hipStream_t s)
{
    if (dt == MONARCH_F16) return launch_heads_typed<f16_t>(v, k, x2, yv, B, heads, dh, n, klen, s);
    return launch_heads_typed<bf16_t>(v, k, x2, yv, B, heads, dh, n, klen, s);
}

int launch_conv_mfma_2048(const void *u, const void *k, const void *g_in, const void *g_out, void *y,
                          int B, int H, int n, int klen, monarch_dtype dt, hipStream_t s)
{
    if (dt == MONARCH_F16) return launch_typed<f16_t>(u, k, g_in, g_out, y, B, H, n, klen, s);
    return launch_typed<bf16_t>(u, k, g_in, g_out, y, B, H, n, klen, s);
}

}  // namespace monarch
