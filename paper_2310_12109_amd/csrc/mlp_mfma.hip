// Fused block-diagonal MLP (order 1: the M2-BERT dimension mixer), bf16 I/O, fp32 accumulate:
//   y[t, blk] = W2_blk * act(W1_blk * x[t, blk] + b1_blk) + b2_blk        (Sec. 3.2, Eq. 3)
//
// One workgroup (4 waves, one per SIMD, up to 512 registers each) takes 64 tokens of one block.
// Everything is computed transposed so that tokens sit on the MFMA column (lane) index:
//   H^T[hidden, token] = W1[hidden, din] * X^T[din, token]      A = W1 rows, B = x rows
//   Y^T[out,    token] = W2[out, hidden] * H^T[hidden, token]   A = W2 rows, B = the accumulators of H^T
// Both weight operands and the x operand are plain 16-byte global loads (8 consecutive inputs of one
// row), and the activated hidden tile re-enters the second GEMM straight from the accumulators (two
// stacked 16x16 tiles = one K=32 operand), so the hidden vector never exists in LDS or HBM.
// The waves split the hidden units (chunks of 32, wave w takes chunks w, w+4, ...): every weight is
// fetched once per workgroup; the four partial Y tiles are summed through LDS in two rounds of plain
// 16-byte stores and loads (waves 2,3 -> 0,1, then 1 -> 0; LDS float atomics are an order of magnitude
// slower), then written with coalesced 16-byte stores.
#include <type_traits>
#include "half16.h"
#include "kernels.h"
#include "lds_dma.h"

namespace monarch {

using h16::f32x4;
using h16::op8;

namespace mlp1 {

using h16::hi32;
using h16::lo32;
using h16::mfma;
using h16::pack16;

constexpr int TOK = 64;   // tokens per workgroup (4 column tiles of 16)

union Pack8 {
    op8 v;
    uint32_t d[4];
    uint4 q;
};

// GELU(z) = z * Phi(z) for two pre-activations at once, returned as a packed bf16 pair (the operand of the second
// GEMM).  Phi is evaluated on packed fp16 pairs, two values per instruction: t = z / 4,
// Phi - 1/2 = t * q(t^2 - 0.4) with q of degree 4 fitted on |z| <= 3.25 (c = 3.25 / 4) under the constraint
// c q(c^2 - 0.4) = 1/2 (the shift by 0.4 keeps the Horner steps well conditioned in fp16); beyond the fitted range the
// polynomial keeps growing, and the last fused multiply-add clamps Phi to [0, 1] with its output modifier (checked
// over every fp16 t: no NaN, infinities end at 0 or 1).  The last product z * Phi takes z in fp32.  11 instructions
// per pair.
// Accuracy: |Phi_approx - Phi| <= 1e-3 for every z (fit 5.8e-4, fp16 evaluation the rest), an ABSOLUTE bound: the
// result is within 1e-3 |z| of z Phi(z), which is below the bf16 rounding of results of ordinary size but is not a
// relative bound in the far negative tail (GELU(-3) = -0.004 may be off by 0.003; below z = -3.3 the result is 0).
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
__device__ __forceinline__ f16x2 splat16(float v) { return (f16x2){(_Float16)v, (_Float16)v}; }
template <typename E> __device__ __forceinline__ uint32_t gelu_pack(float z0, float z1)
{
    const f16x2 h = __builtin_bit_cast(f16x2, __builtin_amdgcn_cvt_pkrtz(z0, z1));
    const f16x2 t = h * splat16(0.25f);
    const f16x2 u = t * t - splat16(0.4f);
    f16x2 q = splat16(4.0132f);
    q = q * u + splat16(-2.2824f);
    q = q * u + splat16(1.2712f);
    q = q * u + splat16(-0.8877f);
    q = q * u + splat16(0.7821f);
    f16x2 w;   // t q + 1/2, clamped to [0, 1] by the instruction's output modifier
    const f16x2 half = splat16(0.5f);
    asm("v_pk_fma_f16 %0, %1, %2, %3 clamp" : "=v"(w) : "v"(t), "v"(q), "v"(half));
    float g0, g1;   // Phi (fp16, low / high half) times z (fp32)
    asm("v_fma_mix_f32 %0, %1, %2, 0 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(g0) : "v"(w), "v"(z0));
    asm("v_fma_mix_f32 %0, %1, %2, 0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(g1) : "v"(w), "v"(z1));
    return pack16<E>(g0, g1);
}

// The same for pre-activations that arrive divided by four (W1 and b1 scaled by 1/4, exact in binary floating point):
// returns GELU / 4 (the caller scales W2 by 4), without gelu_pack's division by four: 10 instructions per pair.
template <typename E> __device__ __forceinline__ uint32_t gelu_pack_quarter(float t0, float t1)
{
    const f16x2 t = __builtin_bit_cast(f16x2, __builtin_amdgcn_cvt_pkrtz(t0, t1));
    const f16x2 u = t * t - splat16(0.4f);
    f16x2 q = splat16(4.0132f);
    q = q * u + splat16(-2.2824f);
    q = q * u + splat16(1.2712f);
    q = q * u + splat16(-0.8877f);
    q = q * u + splat16(0.7821f);
    f16x2 w;
    const f16x2 half = splat16(0.5f);
    asm("v_pk_fma_f16 %0, %1, %2, %3 clamp" : "=v"(w) : "v"(t), "v"(q), "v"(half));
    float g0, g1;   // Phi (fp16, low / high half) times the scaled pre-activation (fp32)
    asm("v_fma_mix_f32 %0, %1, %2, 0 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(g0) : "v"(w), "v"(t0));
    asm("v_fma_mix_f32 %0, %1, %2, 0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(g1) : "v"(w), "v"(t1));
    return pack16<E>(g0, g1);
}

// eight packed elements times a power of two (exact but for results below the smallest normal number)
template <typename E> __device__ __forceinline__ uint4 scale8(uint4 v, float f)
{
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = pack16<E>(lo32<E>(w[i]) * f, hi32<E>(w[i]) * f);
    return make_uint4(w[0], w[1], w[2], w[3]);
}

// Activation of two neighbouring accumulator values, packed for the second GEMM.
template <typename E, int ACT>
__device__ __forceinline__ uint32_t act_pack(float z0, float z1)
{
    if (ACT == 2) return gelu_pack<E>(z0, z1);
    if (ACT == 1) return pack16<E>(fmaxf(z0, 0.0f), fmaxf(z1, 0.0f));
    return pack16<E>(z0, z1);
}

// KS = din / 32 (K steps of the first GEMM); din / 16 row tiles of the second GEMM.
template <typename E, int KS, int ACT>
__global__ __launch_bounds__(256, 1) void mlp_order1_kernel(
    const E *__restrict__ x, E *__restrict__ y, int64_t tokens, int d, int d_hidden, int nb,
    const E *__restrict__ W1, const E *__restrict__ b1, const E *__restrict__ W2,
    const E *__restrict__ b2, int b1_interleaved)
{
    constexpr int DIN = 32 * KS, MT = 2 * KS, LD = DIN + 1;   // LD: padded row of the output tile
    constexpr int PART = MT * 4 * 64;                            // f32x4 pieces of one wave's partial tile
    extern __shared__ f32x4 lds_raw[];
    f32x4 *part = lds_raw;                                       // [2][PART] partial tiles, [piece][lane]
    float *ytile = reinterpret_cast<float *>(lds_raw + 2 * PART);   // [TOK][LD] summed tile
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, l16 = lane & 15, kg = lane >> 4;
    const int blk = blockIdx.y;
    const int64_t t0 = (int64_t)blockIdx.x * TOK;
    const int dh = d_hidden / nb;   // hidden units of this block

    // B operands of the first GEMM: lane (token 16nt + l16, kg) holds x[token][blk*DIN + 32ks + 8kg .. +7]
    Pack8 xop[4][KS];
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
        int64_t t = t0 + 16 * nt + l16;
        if (t >= tokens) t = tokens - 1;   // clamp: the column is computed but never stored
        const E *row = x + t * d + blk * DIN + 8 * kg;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) xop[nt][ks].q = *reinterpret_cast<const uint4 *>(row + 32 * ks);
    }
    f32x4 acc[MT][4];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = (f32x4){0, 0, 0, 0};

    const E *W1b = W1 + (size_t)blk * dh * DIN;   // [dh][DIN]
    const E *W2b = W2 + (size_t)blk * DIN * dh;   // [DIN][dh]
    // Row r of accumulator tile mt in lane group kg is accumulator row 16mt + 4kg + r.  The hidden unit
    // given to first-GEMM row (mt, l16) is chosen so that the 8 operand slots of a lane group are 8
    // consecutive hidden units (one 16-byte load of W2): unit(mt, row) = 8*(row/4) + 4*mt + row%4.
    const int unit_of_lane[2] = {8 * (l16 >> 2) + (l16 & 3), 8 * (l16 >> 2) + 4 + (l16 & 3)};

    for (int j = wave; j < dh / 32; j += 4) {
        const int h0 = 32 * j;   // first hidden unit of the chunk
        // Everything the chunk needs is requested up front: biases of the 8 hidden units this lane
        // group's accumulator rows carry (h0 + 8kg .. +7), both W1 row tiles, all W2 row tiles.
        // (b1_interleaved: hidden unit h of block blk sits at b1[h nb + blk], the layout an order-2
        // Monarch leaves its outputs in; otherwise at b1[blk dh + h])
        uint4 braw = make_uint4(0u, 0u, 0u, 0u);
        if (b1) {
            if (!b1_interleaved) braw = *reinterpret_cast<const uint4 *>(b1 + (size_t)blk * dh + h0 + 8 * kg);
            else {
                const uint16_t *bsrc = reinterpret_cast<const uint16_t *>(b1) + (size_t)(h0 + 8 * kg) * nb + blk;
                uint32_t w[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) w[e] = bsrc[(size_t)e * nb];
                braw = make_uint4(w[0] | (w[1] << 16), w[2] | (w[3] << 16), w[4] | (w[5] << 16), w[6] | (w[7] << 16));
            }
        }
        Pack8 w1[2][KS], w2[MT];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            const E *wrow = W1b + (size_t)(h0 + unit_of_lane[mt]) * DIN + 8 * kg;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) w1[mt][ks].q = *reinterpret_cast<const uint4 *>(wrow + 32 * ks);
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            w2[mt].q = *reinterpret_cast<const uint4 *>(W2b + (size_t)(16 * mt + l16) * dh + h0 + 8 * kg);

        // first GEMM: H^T chunk (32 hidden x 64 tokens).  Tile mt, register r of lane group kg is hidden
        // unit h0 + 8kg + 4mt + r, the same for every token: the accumulators start from the bias.
        f32x4 bias[2];
        {
            const uint32_t bw[4] = {braw.x, braw.y, braw.z, braw.w};
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const uint32_t w = bw[2 * mt + (r >> 1)];
                    bias[mt][r] = ((r & 1) ? hi32<E>(w) : lo32<E>(w));
                }
        }
        f32x4 hacc[2][4];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
                f32x4 a = bias[mt];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) a = mfma<E>(w1[mt][ks].v, xop[nt][ks].v, a);
                hacc[mt][nt] = a;
            }
        // activation on the accumulators; two stacked tiles become one K=32 operand (slot 4mt + r)
        Pack8 hop[4];
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
                hop[nt].d[2 * mt] = act_pack<E, ACT>(hacc[mt][nt][0], hacc[mt][nt][1]);
                hop[nt].d[2 * mt + 1] = act_pack<E, ACT>(hacc[mt][nt][2], hacc[mt][nt][3]);
            }
        // second GEMM: Y^T += W2[:, chunk] * H^T chunk; A operand = 8 consecutive hidden units of one output row
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = mfma<E>(w2[mt].v, hop[nt].v, acc[mt][nt]);
    }

    // Sum the four waves' partial tiles.  Piece (mt, nt) of a wave sits at part[slot][(mt*4+nt)*64 + lane].
    auto spill = [&](int slot) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) part[slot * PART + (mt * 4 + nt) * 64 + lane] = acc[mt][nt];
    };
    auto absorb = [&](int slot) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) acc[mt][nt] += part[slot * PART + (mt * 4 + nt) * 64 + lane];
    };
    if (wave >= 2) spill(wave - 2);
    __syncthreads();
    if (wave < 2) absorb(wave);
    __syncthreads();
    if (wave == 1) spill(0);
    __syncthreads();
    if (wave == 0) {
        absorb(0);
        // row = out feature 16mt + 4kg + r, column = token 16nt + l16  ->  ytile[token][feature]
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                for (int r = 0; r < 4; ++r) ytile[(16 * nt + l16) * LD + 16 * mt + 4 * kg + r] = acc[mt][nt][r];
    }
    __syncthreads();

    // bias, rounding, coalesced stores: 8 consecutive features per thread
    constexpr int PIECES = DIN / 8;   // 16-byte pieces per token
    for (int idx = tid; idx < TOK * PIECES; idx += 256) {
        const int t = idx / PIECES, o0 = (idx - t * PIECES) * 8;
        if (t0 + t >= tokens) continue;
        uint4 b2raw = make_uint4(0u, 0u, 0u, 0u);
        if (b2) b2raw = *reinterpret_cast<const uint4 *>(b2 + (size_t)blk * DIN + o0);
        const uint32_t b2w[4] = {b2raw.x, b2raw.y, b2raw.z, b2raw.w};
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t w = b2w[e >> 1];
            v[e] = ytile[t * LD + o0 + e] + ((e & 1) ? hi32<E>(w) : lo32<E>(w));
        }
        uint4 o;
        o.x = pack16<E>(v[0], v[1]);
        o.y = pack16<E>(v[2], v[3]);
        o.z = pack16<E>(v[4], v[5]);
        o.w = pack16<E>(v[6], v[7]);
        *reinterpret_cast<uint4 *>(y + (t0 + t) * d + blk * DIN + o0) = o;
    }
}


// ---- variant for small blocks and many tokens -------------------------------------------------
// When both weight matrices of a block fit in LDS (64 KB) they are staged there once, already in
// MFMA operand order, by a persistent workgroup that then walks over tiles of 256 tokens of that
// block: wave w owns tokens 64 w .. 64 w + 63 of the tile and the whole hidden vector, so nothing is
// summed across waves and every weight byte leaves L2 once per workgroup instead of once per 64 tokens.
// The next tile's x rows are requested before the current tile is computed.
// Token rows move in the cheap lane order: a wave-wide 16-byte access costs the vector memory pipe about 20 cycles
// when the four lanes of a quad stay inside one 128-byte line and about 69 when they touch four lines, which is
// what the MFMA operand order (lane = token + 16 group) does.  So lane 4 t + p loads and stores piece p of token t
// (a quad = 64 contiguous bytes of one row), and a per-wave LDS area of 16 token rows turns that order into the
// operand order and back (wave-private: no barrier).  The rows of W2 are dealt to the row tiles so that tiles 2 m
// and 2 m + 1 give a lane 8 neighbouring features: tile 2 m + h, row 4 g + r is feature 32 m + 8 g + 4 h + r.
// With GELU the staged W1 and b1 carry a factor 1/4 and W2 a factor 4 (see gelu_pack_quarter).
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
template <typename E, int KS, int ACT, bool STREAM>
__global__ __launch_bounds__(256, 2) void mlp_order1_resident_kernel(
    const E *__restrict__ x, E *__restrict__ y, int64_t tokens, int d, int d_hidden, int nb,
    const E *__restrict__ W1, const E *__restrict__ b1, const E *__restrict__ W2,
    const E *__restrict__ b2, int b1_interleaved, int wgs_per_block)
{
    constexpr int DIN = 32 * KS, MT = 2 * KS, OPS = 4 * KS;   // operand pieces (64 lanes x 16 B) per hidden chunk
    extern __shared__ uint4 lds_ops[];                          // [chunk][OPS][lane], then the bias [dh] as bf16
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, l16 = lane & 15, kg = lane >> 4;
    const int blk = blockIdx.x % nb, slot = blockIdx.x / nb;
    const int dh = d_hidden / nb, nch = dh / 32;
    const E *W1b = W1 + (size_t)blk * dh * DIN;   // [dh][DIN]
    const E *W2b = W2 + (size_t)blk * DIN * dh;   // [DIN][dh]
    uint16_t *bias_lds = reinterpret_cast<uint16_t *>(lds_ops + (size_t)nch * OPS * 64);
    constexpr int WST = 16 * (4 * KS + 1);   // a wave's exchange area: 16 token rows of 4 KS pieces, one piece of padding
    u32x4 *wst = reinterpret_cast<u32x4 *>(lds_ops + (size_t)nch * OPS * 64 + (dh * 2 + 15) / 16 + wave * WST);
    const int qt = lane >> 2, qp = lane & 3;   // quad order: token qt of a column tile, piece 4 i + qp of its row

    // stage the block's weights: piece (chunk j, op o, lane) is exactly the 16-byte operand that lane
    // will feed to the MFMA (same row / slot assignment as mlp_order1_kernel)
    for (int idx = tid; idx < nch * OPS * 64; idx += 256) {
        const int ln = idx & 63, q = idx >> 6, j = q / OPS, o = q - j * OPS;
        const int r16 = ln & 15, g = ln >> 4;
        const E *src;
        if (o < 2 * KS) {
            const int mt = o / KS, ks = o - mt * KS;
            const int unit = 8 * (r16 >> 2) + 4 * mt + (r16 & 3);
            src = W1b + (size_t)(32 * j + unit) * DIN + 32 * ks + 8 * g;
        } else {
            const int mt = o - 2 * KS;
            src = W2b + (size_t)(32 * (mt >> 1) + 8 * (r16 >> 2) + 4 * (mt & 1) + (r16 & 3)) * dh + 32 * j + 8 * g;
        }
        uint4 piece = *reinterpret_cast<const uint4 *>(src);
        if (ACT == 2) piece = scale8<E>(piece, o < 2 * KS ? 0.25f : 4.0f);
        lds_ops[idx] = piece;
    }
    for (int h = tid; h < dh; h += 256) {
        uint16_t v = 0;
        if (b1) v = reinterpret_cast<const uint16_t *>(b1)[b1_interleaved ? (size_t)h * nb + blk : (size_t)blk * dh + h];
        if (ACT == 2) v = (uint16_t)pack16<E>(lo32<E>((uint32_t)v) * 0.25f, 0.0f);
        bias_lds[h] = v;
    }
    // output bias of the rows this lane's accumulators carry: features 16 mt + 4 kg + r
    float bias2[MT][4];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r) bias2[mt][r] = b2 ? (float)b2[(size_t)blk * DIN + 32 * (mt >> 1) + 8 * kg + 4 * (mt & 1) + r] : 0.0f;
    __syncthreads();

    const int64_t ntiles = (tokens + 255) / 256;
    // Token rows that are read once and written once per launch take streaming accesses (config 5b: 105 -> 99.6 us);
    // between the factor launches of an order-2 layer (the interleaved bias marks it) the rows come from and go to the
    // neighbouring launch and keep ordinary ones (streaming there cost 1 us): STREAM.
    u32x4 xnext[4][KS];
    auto request = [&](int64_t tile) {
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
            int64_t t = tile * 256 + 64 * wave + 16 * nt + qt;
            if (t >= tokens) t = tokens - 1;   // clamp: the column is computed but never stored
            const E *row = x + t * d + blk * DIN + 8 * qp;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) xnext[nt][ks] = STREAM ? __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(row + 32 * ks))
                                                                    : *reinterpret_cast<const u32x4 *>(row + 32 * ks);
        }
    };
    if (slot < ntiles) request(slot);
    for (int64_t tile = slot; tile < ntiles; tile += wgs_per_block) {
        u32x4 xop[4][KS];   // quad order -> operand order: lane (token l16, group kg) takes pieces 4 ks + kg of its row
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) wst[qt * (4 * KS + 1) + 4 * ks + qp] = xnext[nt][ks];
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) xop[nt][ks] = wst[l16 * (4 * KS + 1) + 4 * ks + kg];
            __builtin_amdgcn_wave_barrier();
        }
        const int64_t after = tile + wgs_per_block;
        request(after < ntiles ? after : tile);

        f32x4 acc[MT][4];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = (f32x4){0, 0, 0, 0};
        for (int j = 0; j < nch; ++j) {
            const uint4 *ops = lds_ops + (size_t)j * OPS * 64 + lane;
            Pack8 w1[2][KS], w2[MT];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) w1[mt][ks].q = ops[(mt * KS + ks) * 64];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) w2[mt].q = ops[(2 * KS + mt) * 64];
            const uint4 braw = *reinterpret_cast<const uint4 *>(bias_lds + 32 * j + 8 * kg);

            f32x4 bias[2];   // the accumulators of the first GEMM start from the bias of their rows
            {
                const uint32_t bw[4] = {braw.x, braw.y, braw.z, braw.w};
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const uint32_t w = bw[2 * mt + (r >> 1)];
                        bias[mt][r] = ((r & 1) ? hi32<E>(w) : lo32<E>(w));
                    }
            }
            f32x4 hacc[2][4];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) {
                    f32x4 a = bias[mt];
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) a = mfma<E>(w1[mt][ks].v, __builtin_bit_cast(op8, xop[nt][ks]), a);
                    hacc[mt][nt] = a;
                }
            Pack8 hop[4];
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
                    if constexpr (ACT == 2) {
                        hop[nt].d[2 * mt] = gelu_pack_quarter<E>(hacc[mt][nt][0], hacc[mt][nt][1]);
                        hop[nt].d[2 * mt + 1] = gelu_pack_quarter<E>(hacc[mt][nt][2], hacc[mt][nt][3]);
                    } else {
                        hop[nt].d[2 * mt] = act_pack<E, ACT>(hacc[mt][nt][0], hacc[mt][nt][1]);
                        hop[nt].d[2 * mt + 1] = act_pack<E, ACT>(hacc[mt][nt][2], hacc[mt][nt][3]);
                    }
                }
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = mfma<E>(w2[mt].v, hop[nt].v, acc[mt][nt]);
        }
        // the accumulators of tiles 2 m, 2 m + 1 are features 32 m + 8 kg .. + 7 of token 16 nt + l16: piece 4 m + kg of
        // its row; through the exchange area into quad order, then 16-byte stores
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
#pragma unroll
            for (int m = 0; m < KS; ++m) {
                wst[l16 * (4 * KS + 1) + 4 * m + kg] =
                    u32x4{pack16<E>(acc[2 * m][nt][0] + bias2[2 * m][0], acc[2 * m][nt][1] + bias2[2 * m][1]),
                          pack16<E>(acc[2 * m][nt][2] + bias2[2 * m][2], acc[2 * m][nt][3] + bias2[2 * m][3]),
                          pack16<E>(acc[2 * m + 1][nt][0] + bias2[2 * m + 1][0], acc[2 * m + 1][nt][1] + bias2[2 * m + 1][1]),
                          pack16<E>(acc[2 * m + 1][nt][2] + bias2[2 * m + 1][2], acc[2 * m + 1][nt][3] + bias2[2 * m + 1][3])};
            }
            __builtin_amdgcn_wave_barrier();
            const int64_t t = tile * 256 + 64 * wave + 16 * nt + qt;
            E *dst = y + t * d + blk * DIN + 8 * qp;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const u32x4 o = wst[qt * (4 * KS + 1) + 4 * ks + qp];
                if (t < tokens) {
                    if (STREAM) __builtin_nontemporal_store(o, reinterpret_cast<u32x4 *>(dst + 32 * ks));
                    else *reinterpret_cast<u32x4 *>(dst + 32 * ks) = o;
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
}


// ---- variant for large blocks ---------------------------------------------------------------------
// One workgroup takes 64 tokens of one block, wave w the tokens 16 w .. 16 w + 15 and the whole hidden
// vector (nothing is summed across waves).  The weights of one chunk of 32 hidden units (both matrices, in
// MFMA operand order, 4 KS KB) go from L2 straight into a ring of LDS slots (direct-to-LDS 16-byte loads:
// the 64 lanes of a wave fill one 1 KB operand piece) and are read from there by all four waves: a quarter
// of the L2 traffic of mlp_order1_kernel, and requests RING - 1 chunks ahead of their use without holding
// registers.  One barrier per chunk: it publishes chunk j and frees the slot chunk j - 1 was read from.
// slots of the weight ring: as many chunks of 4 KS KB as fit in 148 KB, at most 8
constexpr int ring_slots(int ks) { return 148 / (4 * ks) < 8 ? 148 / (4 * ks) : 8; }

template <typename E, int KS, int ACT, int NT>
__global__ __launch_bounds__(256, 1) void mlp_order1_stream_kernel(
    const E *__restrict__ x, E *__restrict__ y, int64_t tokens, int d, int d_hidden, int nb,
    const E *__restrict__ W1, const E *__restrict__ b1, const E *__restrict__ W2,
    const E *__restrict__ b2, int b1_interleaved)
{
    constexpr int DIN = 32 * KS, MT = 2 * KS, OPS = 4 * KS;   // operand pieces (64 lanes x 16 B) per hidden chunk
    constexpr int ring = ring_slots(KS);
    extern __shared__ __attribute__((aligned(16))) uint4 lds_ring[];   // [ring][OPS * 64], then the hidden bias [dh]
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, l16 = lane & 15, kg = lane >> 4;
    const int blk = blockIdx.y;
    const int64_t t0 = (int64_t)blockIdx.x * (64 * NT) + 16 * NT * wave;   // NT column tiles of 16 tokens per wave
    const int dh = d_hidden / nb, nch = dh / 32;
    const E *W1b = W1 + (size_t)blk * dh * DIN;   // [dh][DIN]
    const E *W2b = W2 + (size_t)blk * DIN * dh;   // [DIN][dh]
    uint16_t *bias_lds = reinterpret_cast<uint16_t *>(lds_ring + (size_t)ring * OPS * 64);

    // Wave w fetches the pieces o = w, w + 4, ... of a chunk (KS of them); piece o holds the 64 x 16 bytes that
    // feed MFMA o (rows / slots as in mlp_order1_kernel: W1 rows in hidden-unit order
    // 8 (r/4) + 4 mt + r%4, W2 rows = output features).  Past the last chunk the last one is fetched again, so
    // that every iteration issues the same number of loads and the wait below can count them.
    // The lane that FETCHES operand entry (row, lane group) is 4 row + group, not the lane that uses it
    // (row + 16 group): four neighbouring lanes then fetch one 64-byte run of a row and the vector cache looks
    // up one line for them instead of four (measured: 45 against 15 bytes per clock and compute unit).  A piece
    // therefore sits in LDS in fetch order, and lane (l16, kg) reads entry 4 l16 + kg of it (free of bank
    // conflicts, as measured).
    const int frow = lane >> 2, fkg = lane & 3;
    int src_off[KS], src_step[KS];   // element offset of this lane's pieces in chunk 0, and per chunk
#pragma unroll
    for (int u = 0; u < KS; ++u) {
        const int o = wave + 4 * u;
        if (o < 2 * KS) {
            const int mt = o / KS, ks = o - mt * KS;
            src_off[u] = (8 * (frow >> 2) + 4 * mt + (frow & 3)) * DIN + 32 * ks + 8 * fkg;
            src_step[u] = 32 * DIN;
        } else {
            src_off[u] = (int)((W2b - W1b) + (16 * (o - 2 * KS) + frow) * dh + 8 * fkg);
            src_step[u] = 32;
        }
    }
    auto request = [&](int j) {
        const int jj = j < nch ? j : nch - 1;
        uint4 *slot = lds_ring + (size_t)(j % ring) * OPS * 64;
#pragma unroll
        for (int u = 0; u < KS; ++u) dma_16(W1b + src_off[u] + jj * src_step[u], slot + (wave + 4 * u) * 64);
    };
    for (int a = 0; a < ring - 1; ++a) request(a);

    for (int h = tid; h < dh; h += 256) {
        uint16_t v = 0;
        if (b1) v = reinterpret_cast<const uint16_t *>(b1)[b1_interleaved ? (size_t)h * nb + blk : (size_t)blk * dh + h];
        bias_lds[h] = v;
    }
    Pack8 xop[NT][KS];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        int64_t t = t0 + 16 * nt + l16;
        if (t >= tokens) t = tokens - 1;   // clamp: the column is computed but never stored
        const E *row = x + t * d + blk * DIN + 8 * kg;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) xop[nt][ks].q = *reinterpret_cast<const uint4 *>(row + 32 * ks);
    }
    float bias2[MT][4];   // output bias of the rows this lane's accumulators carry
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r) bias2[mt][r] = b2 ? (float)b2[(size_t)blk * DIN + 16 * mt + 4 * kg + r] : 0.0f;
    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = (f32x4){0, 0, 0, 0};
    // (x, the biases and the first ring - 1 chunks are in flight; the loop below waits by count)
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    for (int j = 0; j < nch; ++j) {
        // the barrier that ended the previous iteration published chunk j and guaranteed that chunk j - 1 has
        // been read by every wave: its slot is the one the next request overwrites
        request(j + ring - 1);
        // bias of the 8 hidden units this lane group's accumulator rows carry: 32 j + 8 kg .. + 7
        f32x4 bias[2];
        {
            const uint4 braw = *reinterpret_cast<const uint4 *>(bias_lds + 32 * j + 8 * kg);
            const uint32_t bw[4] = {braw.x, braw.y, braw.z, braw.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) bias[e >> 2][e & 3] = ((e & 1) ? hi32<E>(bw[e >> 1]) : lo32<E>(bw[e >> 1]));
        }
        const uint4 *ops = lds_ring + (size_t)(j % ring) * OPS * 64 + 4 * l16 + kg;
        Pack8 hop[NT];
        {
            Pack8 w1[2][KS];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) w1[mt][ks].q = ops[(mt * KS + ks) * 64];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
                    f32x4 a = bias[mt];
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) a = mfma<E>(w1[mt][ks].v, xop[nt][ks].v, a);
                    hop[nt].d[2 * mt] = act_pack<E, ACT>(a[0], a[1]);
                    hop[nt].d[2 * mt + 1] = act_pack<E, ACT>(a[2], a[3]);
                }
            }
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            Pack8 w2;
            w2.q = ops[(2 * KS + mt) * 64];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = mfma<E>(w2.v, hop[nt].v, acc[mt][nt]);
        }
        // own pieces of chunk j + 1 landed (the KS (ring - 2) requests after them may still be in flight)
        wait_vm_at_most<KS * (ring - 2)>();
        __syncthreads();
    }

    // accumulator rows 4 kg .. 4 kg + 3 of tile mt are 4 consecutive features of a token: 8-byte stores
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int64_t t = t0 + 16 * nt + l16;
        if (t < tokens) {
            E *dst = y + t * d + blk * DIN + 4 * kg;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                uint2 o;
                o.x = pack16<E>(acc[mt][nt][0] + bias2[mt][0], acc[mt][nt][1] + bias2[mt][1]);
                o.y = pack16<E>(acc[mt][nt][2] + bias2[mt][2], acc[mt][nt][3] + bias2[mt][3]);
                *reinterpret_cast<uint2 *>(dst + 16 * mt) = o;
            }
        }
    }
}


// ---- variant for large blocks and few tokens --------------------------------------------------------
// Same decomposition as mlp_order1_kernel (64 tokens of one block per workgroup, the waves split the hidden
// units, partial tiles summed at the end), fed differently.  Measured on that kernel: a wave-wide 16-byte
// load whose 16 rows are 16 different cache lines per lane quad costs the vector cache about 69 cycles, a
// load whose lane quads each stay inside one line about 20; with every weight fetched in the first form the
// compute unit spent most of its time in those look-ups.  Here
//   * a wave brings the weights of its chunks into a private ring of three LDS slots with direct-to-LDS
//     loads in the cheap lane order (lane 4 row + group fetches entry (row, group)), alternating the W1
//     part and the W2 part of a chunk (2 KS KB each), ahead of their use, and reads each 1 KB operand from
//     there once for all four column tiles.  The ring is private, so the main loop has no
//     barrier: a wave waits on its own load counter only;
//   * x goes through LDS once in the same way (each wave fetches a quarter of the tile);
//   * at the end every wave owns the row tiles mt = wave (mod 4): the other waves' partial tiles go through
//     LDS in one exchange (one barrier), the owner adds them, applies the output bias and stores.
// Load accounting: direct-to-LDS loads and ordinary loads share the counter and complete in order; between
// the prologue and the epilogue the only loads are the ring's, 2 KS per part.

constexpr size_t split_lds_bytes(int ks, int dh) { return (size_t)24 * ks * 1024 + (size_t)dh * 2; }

template <typename E, int KS, int ACT>
__global__ __launch_bounds__(256, 1) void mlp_order1_split_kernel(
    const E *__restrict__ x, E *__restrict__ y, int64_t tokens, int d, int d_hidden, int nb,
    const E *__restrict__ W1, const E *__restrict__ b1, const E *__restrict__ W2,
    const E *__restrict__ b2, int b1_interleaved)
{
    constexpr int DIN = 32 * KS, MT = 2 * KS, ITEM = 2 * KS;   // ITEM: 1 KB pieces of one ring part
    extern __shared__ __attribute__((aligned(16))) uint4 lds_split[];   // [3 slots][4 waves][ITEM * 64], bias [dh]
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, l16 = lane & 15, kg = lane >> 4;
    const int frow = lane >> 2, fkg = lane & 3;   // the operand entry this lane fetches
    const int rd = 4 * l16 + kg;                  // where the entry this lane uses sits in a piece
    const int blk = blockIdx.y;
    const int64_t t0 = (int64_t)blockIdx.x * TOK;
    const int dh = d_hidden / nb, nch = dh / 32;
    const int nmine = wave < nch ? (nch - wave + 3) / 4 : 0;   // chunks wave, wave + 4, ...
    const E *W1b = W1 + (size_t)blk * dh * DIN;   // [dh][DIN]
    const E *W2b = W2 + (size_t)blk * DIN * dh;   // [DIN][dh]
    uint16_t *bias_lds = reinterpret_cast<uint16_t *>(lds_split + (size_t)12 * ITEM * 64);
    auto slot_ptr = [&](int slot) { return lds_split + ((size_t)slot * 4 + wave) * ITEM * 64; };

    // Parts of this wave, in the order they are needed: part 0 = W1 rows of its first chunk, then for
    // jj = 0, 1, ...: part 2 jj + 1 = W1 rows of chunk jj + 1, part 2 jj + 2 = W2 columns of chunk jj (chunk jj
    // of the wave is chunk wave + 4 jj of the block).  Part i lives in slot i % 3.  Past the wave's last chunk
    // the last chunk is fetched again (never read), so that every request issues ITEM loads.
    const E *w1_lane = W1b + (size_t)(8 * (frow >> 2) + (frow & 3)) * DIN + 8 * fkg;
    const E *w2_lane = W2b + (size_t)frow * dh + 8 * fkg;
    const uint32_t ring_addr = lds_address(lds_split) + (uint32_t)wave * ITEM * 1024;
    auto request = [&](int i) {
        const bool w1_part = i == 0 || (i & 1);
        int c = i == 0 ? 0 : (i & 1) ? (i + 1) >> 1 : (i - 2) >> 1;
        if (c > nmine - 1) c = nmine - 1;
        const int h0 = 32 * (wave + 4 * c);
        const uint32_t dst = ring_addr + (uint32_t)(i % 3) * 4 * ITEM * 1024;
        if (w1_part) {
            const E *src = w1_lane + (size_t)h0 * DIN;
#pragma unroll
            for (int o = 0; o < 2 * KS; o += 2)
                dma_16_pair(src + 4 * (o / KS) * DIN + 32 * (o % KS), src + 4 * ((o + 1) / KS) * DIN + 32 * ((o + 1) % KS),
                            dst + o * 1024);
        } else {
            const E *src = w2_lane + h0;
#pragma unroll
            for (int mt = 0; mt < MT; mt += 2)
                dma_16_pair(src + (size_t)16 * mt * dh, src + (size_t)16 * (mt + 1) * dh, dst + mt * 1024);
        }
    };

    // Prologue: the biases, then x (a quarter of the tile per wave) into the third slot's area and the first
    // two parts into the first two slots.
    uint4 b1piece = make_uint4(0u, 0u, 0u, 0u);   // hidden bias, 8 units per thread (the usual layout)
    const bool b1_vec = b1 && !b1_interleaved && dh <= 2048;
    if (b1_vec && tid < dh / 8) b1piece = *reinterpret_cast<const uint4 *>(b1 + (size_t)blk * dh + 8 * tid);
    uint2 b2raw[(MT + 3) / 4];                    // output bias of the row tiles this wave owns (mt = wave + 4 q)
#pragma unroll
    for (int q = 0; q < (MT + 3) / 4; ++q) {
        b2raw[q] = make_uint2(0u, 0u);
        if (b2 && wave + 4 * q < MT) b2raw[q] = *reinterpret_cast<const uint2 *>(b2 + (size_t)blk * DIN + 16 * (wave + 4 * q) + 4 * kg);
    }
    uint4 *xstage = lds_split + (size_t)2 * 4 * ITEM * 64;   // 4 KS pieces: piece (nt, ks) at (nt * KS + ks) * 64
    {
        int64_t t = t0 + 16 * wave + frow;   // wave w fetches the column tile nt = w
        if (t >= tokens) t = tokens - 1;     // clamp: the column is computed but never stored
        const E *row = x + t * d + blk * DIN + 8 * fkg;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) dma_16(row + 32 * ks, xstage + (wave * KS + ks) * 64);
    }
    if (nmine > 0) {
        request(0);
        request(1);
    }
    if (b1_vec) {
        if (tid < dh / 8) reinterpret_cast<uint4 *>(bias_lds)[tid] = b1piece;
    } else {
        for (int h = tid; h < dh; h += 256) {
            uint16_t v = 0;
            if (b1) v = reinterpret_cast<const uint16_t *>(b1)[b1_interleaved ? (size_t)h * nb + blk : (size_t)blk * dh + h];
            bias_lds[h] = v;
        }
    }
    // (x was requested before the two parts: at most those, 2 ITEM loads, may still be in flight)
    if (nmine > 0) wait_loads_at_most<2 * ITEM>();
    else wait_loads_at_most<0>();
    __syncthreads();
    Pack8 xop[4][KS];
#pragma unroll
    for (int nt = 0; nt < 4; ++nt)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) xop[nt][ks].q = xstage[(nt * KS + ks) * 64 + rd];
    wait_lds_reads();
    __syncthreads();   // everybody holds x: the third slot is free
    if (nmine > 0) request(2);

    f32x4 acc[MT][4];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = (f32x4){0, 0, 0, 0};

    // Tile mt, register r of lane group kg of the first GEMM is hidden unit h0 + 8 kg + 4 mt + r, the same for
    // every token: the accumulators start from the bias.
    auto start_from_bias = [&](f32x4 (&h)[2][4], int h0) {
        const uint4 braw = *reinterpret_cast<const uint4 *>(bias_lds + h0 + 8 * kg);
        const uint32_t bw[4] = {braw.x, braw.y, braw.z, braw.w};
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            f32x4 b;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const uint32_t w = bw[2 * mt + (r >> 1)];
                b[r] = ((r & 1) ? hi32<E>(w) : lo32<E>(w));
            }
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) h[mt][nt] = b;
        }
    };
    auto first_gemm = [&](f32x4 (&h)[2][4], const Pack8 (&w1)[2][KS]) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) h[mt][nt] = mfma<E>(w1[mt][ks].v, xop[nt][ks].v, h[mt][nt]);
    };
    auto read_piece_set = [&](Pack8 *dst, int slot) {
        const uint4 *ops = slot_ptr(slot) + rd;
#pragma unroll
        for (int o = 0; o < ITEM; ++o) dst[o].q = ops[o * 64];
    };

    // The loop is software-pipelined so that the matrix core and the vector ALU of the SIMD (which has this one
    // wave) work at the same time: while the activation of chunk jj runs on the vector ALU, the first GEMM of
    // the wave's next chunk runs on the matrix core, one MFMA issued between slices of the activation (the
    // order is pinned with scheduling barriers: left alone the compiler issues the MFMAs back to back, and a
    // wave cannot issue anything while its next MFMA waits for the pipe); then the second GEMM of chunk jj.
    // Load accounting of a step: when its W1 part is needed the two parts requested after it may be in flight,
    // and the same holds for its W2 part: 2 ITEM loads at most.
    constexpr int NM = 8 * KS;   // MFMAs of a first GEMM
    f32x4 hacc[2][4];
    auto step = [&](int jj, auto last_tag) {
        constexpr bool LAST = decltype(last_tag)::value;
        const int p = 2 * jj + 1;   // this step's parts: p (W1 of the next chunk), p + 1 (W2 of this chunk)
        if (!LAST && jj > 0) {
            wait_lds_reads();   // (the previous step's W2 operands are long in registers)
            request(p + 2);     // into the slot they came from
        }
        Pack8 w1[2][KS];
        f32x4 hnext[2][4];
        if (!LAST) {
            wait_loads_at_most<2 * ITEM>();
            read_piece_set(&w1[0][0], p % 3);
            wait_lds_reads();
            request(p + 3);
            start_from_bias(hnext, 32 * (wave + 4 * (jj + 1)));
        }
        // activation on the accumulators; two stacked tiles become one K=32 operand (slot 4mt + r)
        Pack8 hop[4];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < NM; ++u) {
            if (!LAST) {
                const int ks = u / 8, mt = (u / 4) % 2, nt = u % 4;
                hnext[mt][nt] = mfma<E>(w1[mt][ks].v, xop[nt][ks].v, hnext[mt][nt]);
            }
#pragma unroll
            for (int v = (u * 16) / NM; v < ((u + 1) * 16) / NM; ++v)   // pair v: values 2v, 2v + 1 of 8 nt + 4 mt + r
                hop[v >> 2].d[v & 3] = act_pack<E, ACT>(hacc[(v >> 1) & 1][v >> 2][2 * (v & 1)], hacc[(v >> 1) & 1][v >> 2][2 * (v & 1) + 1]);
        }
        if (!LAST) {
#pragma unroll
            for (int u = 0; u < NM; ++u) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                       // one MFMA
                __builtin_amdgcn_sched_group_barrier(0x002, (224 + NM - 1) / NM, 0);   // its share of the activation
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        // second GEMM: Y^T += W2[:, chunk] * H^T chunk (the last step requested nothing: it waits for all)
        if (LAST) wait_loads_at_most<0>();
        else wait_loads_at_most<2 * ITEM>();
        Pack8 w2[MT];
        read_piece_set(w2, (p + 1) % 3);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = mfma<E>(w2[mt].v, hop[nt].v, acc[mt][nt]);
        // operand reads run four row tiles ahead of the MFMAs that use them
        __builtin_amdgcn_sched_group_barrier(0x100, MT < 4 ? MT : 4, 1);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            __builtin_amdgcn_sched_group_barrier(0x008, 4, 1);
            if (mt + 4 < MT) __builtin_amdgcn_sched_group_barrier(0x100, 1, 1);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (!LAST) {
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) hacc[mt][nt] = hnext[mt][nt];
        }
    };
    if (nmine > 0) {
        wait_loads_at_most<2 * ITEM>();   // part 0 has landed
        Pack8 w1[2][KS];
        read_piece_set(&w1[0][0], 0);
        wait_lds_reads();
        request(3);
        start_from_bias(hacc, 32 * wave);
        first_gemm(hacc, w1);
#pragma unroll 1
        for (int jj = 0; jj < nmine - 1; ++jj) step(jj, std::false_type{});
        step(nmine - 1, std::true_type{});
    }

    // Exchange: tile mt belongs to wave mt % 4; the three other waves park their partial of it at
    // [mt][(wave - owner - 1) mod 4][nt][lane].  The ring is dead, but its last (repeated) requests may still
    // be landing: they are waited for before the area is reused.
    wait_loads_at_most<0>();
    __syncthreads();
    f32x4 *part = reinterpret_cast<f32x4 *>(lds_split);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int owner = mt & 3;
        if (wave != owner) {
            f32x4 *dst = part + ((size_t)(mt * 3 + ((wave - owner - 1) & 3)) * 4) * 64 + lane;
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) dst[nt * 64] = acc[mt][nt];
        }
    }
    __syncthreads();
    // accumulator rows 4 kg .. 4 kg + 3 of tile mt are 4 consecutive features of a token: 8-byte stores
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        if (wave != (mt & 3)) continue;
        const uint2 braw = b2raw[mt >> 2];
        const float bias2[4] = {lo32<E>(braw.x), hi32<E>(braw.x),
                                lo32<E>(braw.y), hi32<E>(braw.y)};
        const f32x4 *src = part + (size_t)mt * 3 * 4 * 64 + lane;
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
            f32x4 v = acc[mt][nt];
#pragma unroll
            for (int q = 0; q < 3; ++q) v += src[(q * 4 + nt) * 64];
            const int64_t t = t0 + 16 * nt + l16;
            if (t < tokens) {
                uint2 o;
                o.x = pack16<E>(v[0] + bias2[0], v[1] + bias2[1]);
                o.y = pack16<E>(v[2] + bias2[2], v[3] + bias2[3]);
                *reinterpret_cast<uint2 *>(y + t * d + blk * DIN + 16 * mt + 4 * kg) = o;
            }
        }
    }
}

}  // namespace mlp1

bool mlp_mfma_order1_supported(int d, int d_hidden, int nb, monarch_dtype dt)
{
    if ((dt != MONARCH_BF16 && dt != MONARCH_F16) || d % nb || d_hidden % nb) return false;
    const int din = d / nb, dh = d_hidden / nb;
    return din % 32 == 0 && din >= 32 && din <= 192 && dh % 32 == 0 && d % 8 == 0;
}

namespace {

template <typename E>
int launch_typed(const void *x, void *y, int64_t tokens, int d, int d_hidden, int nb, const void *W1,
                 const void *b1, const void *W2, const void *b2, int act, int b1_interleaved, hipStream_t s)
{
    const int din = d / nb;
    // small blocks, many tokens: weights resident in LDS, persistent workgroups
    const int dh_blk = d_hidden / nb;
    // the weights in operand order, the hidden bias, and the four waves' exchange areas (16 rows of din / 8 + 1 pieces)
    const size_t res_lds = (size_t)dh_blk * din * 4 + (((size_t)dh_blk * 2 + 15) & ~(size_t)15) + (size_t)4 * 16 * (din / 8 + 1) * 16;
    if (din <= 64 && res_lds <= 79 * 1024 && tokens >= 2048) {
        int dev = 0, ncu = 0;
        MONARCH_HIP_CHECK(hipGetDevice(&dev));
        MONARCH_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
        const int64_t ntiles = (tokens + 255) / 256;
        int64_t per_block = (2 * (int64_t)ncu + nb - 1) / nb;   // two workgroups per compute unit
        if (per_block < 1) per_block = 1;
        if (per_block > ntiles) per_block = ntiles;
        const dim3 rgrid((unsigned)(per_block * nb));
#define MONARCH_LAUNCH_RES(KSV, ACTV)                                                                           \
    do {                                                                                                        \
        auto kern = b1_interleaved ? mlp1::mlp_order1_resident_kernel<E, KSV, ACTV, false>                      \
                                   : mlp1::mlp_order1_resident_kernel<E, KSV, ACTV, true>;                      \
        if (res_lds > 48 * 1024)                                                                                \
            MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, \
                                                  (int)res_lds));                                               \
        hipLaunchKernelGGL(kern, rgrid, dim3(256), res_lds, s, (const E *)x, (E *)y, tokens, d,       \
                           d_hidden, nb, (const E *)W1, (const E *)b1, (const E *)W2,            \
                           (const E *)b2, b1_interleaved, (int)per_block);                                 \
    } while (0)
#define MONARCH_LAUNCH_RES_ACT(KSV)                     \
    do {                                                \
        if (act == 2) MONARCH_LAUNCH_RES(KSV, 2);       \
        else if (act == 1) MONARCH_LAUNCH_RES(KSV, 1);  \
        else MONARCH_LAUNCH_RES(KSV, 0);                \
    } while (0)
        switch (din / 32) {
        case 1: MONARCH_LAUNCH_RES_ACT(1); break;
        default: MONARCH_LAUNCH_RES_ACT(2); break;
        }
#undef MONARCH_LAUNCH_RES_ACT
#undef MONARCH_LAUNCH_RES
        MONARCH_HIP_CHECK(hipGetLastError());
        return MONARCH_OK;
    }
    const int64_t tiles = (tokens + mlp1::TOK - 1) / mlp1::TOK;
    if (tiles > 0x7fffffffLL || nb > 65535) return fail(MONARCH_ESHAPE, "too many tokens or blocks for one launch");
    const dim3 grid((unsigned)tiles, (unsigned)nb);
    int dev = 0, ncu = 0;
    MONARCH_HIP_CHECK(hipGetDevice(&dev));
    MONARCH_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
    if (tokens * nb >= (int64_t)256 * ncu) {
        // Enough tokens for wider tiles: weights streamed through an LDS ring, 64 NT tokens per workgroup (less
        // weight traffic out of L2 per token, which is what bounds the 64-token kernel below): the largest NT
        // that still gives every compute unit a workgroup.
        const int ntv = tokens * nb >= (int64_t)512 * ncu ? 4 : 2;
        const int64_t wtiles = (tokens + 64 * ntv - 1) / (64 * ntv);
        const dim3 sgrid((unsigned)wtiles, (unsigned)nb);
        const size_t str_lds = (size_t)mlp1::ring_slots(din / 32) * (din / 8) * 1024 + (size_t)dh_blk * 2;
#define MONARCH_LAUNCH_STR(KSV, ACTV, NTV)                                                                       \
    do {                                                                                                         \
        auto kern = mlp1::mlp_order1_stream_kernel<E, KSV, ACTV, NTV>;                                              \
        MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,    \
                                              (int)str_lds));                                                    \
        hipLaunchKernelGGL(kern, sgrid, dim3(256), str_lds, s, (const E *)x, (E *)y, tokens, d,        \
                           d_hidden, nb, (const E *)W1, (const E *)b1, (const E *)W2,             \
                           (const E *)b2, b1_interleaved);                                                  \
    } while (0)
#define MONARCH_LAUNCH_STR_NT(KSV, ACTV)                      \
    do {                                                      \
        if (ntv == 4) MONARCH_LAUNCH_STR(KSV, ACTV, 4);       \
        else MONARCH_LAUNCH_STR(KSV, ACTV, 2);                \
    } while (0)
#define MONARCH_LAUNCH_STR_ACT(KSV)                        \
    do {                                                   \
        if (act == 2) MONARCH_LAUNCH_STR_NT(KSV, 2);       \
        else if (act == 1) MONARCH_LAUNCH_STR_NT(KSV, 1);  \
        else MONARCH_LAUNCH_STR_NT(KSV, 0);                \
    } while (0)
        switch (din / 32) {
        case 1: MONARCH_LAUNCH_STR_ACT(1); break;
        case 2: MONARCH_LAUNCH_STR_ACT(2); break;
        case 3: MONARCH_LAUNCH_STR_ACT(3); break;
        case 4: MONARCH_LAUNCH_STR_ACT(4); break;
        case 5: MONARCH_LAUNCH_STR_ACT(5); break;
        default: MONARCH_LAUNCH_STR_ACT(6); break;
        }
#undef MONARCH_LAUNCH_STR_ACT
#undef MONARCH_LAUNCH_STR_NT
#undef MONARCH_LAUNCH_STR
        MONARCH_HIP_CHECK(hipGetLastError());
        return MONARCH_OK;
    }
    const size_t split_lds = mlp1::split_lds_bytes(din / 32, dh_blk);
    if (split_lds <= 160 * 1024) {
#define MONARCH_LAUNCH_SPL(KSV, ACTV)                                                                            \
    do {                                                                                                         \
        auto kern = mlp1::mlp_order1_split_kernel<E, KSV, ACTV>;                                                    \
        if (split_lds > 48 * 1024)                                                                               \
            MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, \
                                                  (int)split_lds));                                              \
        hipLaunchKernelGGL(kern, grid, dim3(256), split_lds, s, (const E *)x, (E *)y, tokens, d,       \
                           d_hidden, nb, (const E *)W1, (const E *)b1, (const E *)W2,             \
                           (const E *)b2, b1_interleaved);                                                  \
    } while (0)
#define MONARCH_LAUNCH_SPL_ACT(KSV)                     \
    do {                                                \
        if (act == 2) MONARCH_LAUNCH_SPL(KSV, 2);       \
        else if (act == 1) MONARCH_LAUNCH_SPL(KSV, 1);  \
        else MONARCH_LAUNCH_SPL(KSV, 0);                \
    } while (0)
        switch (din / 32) {
        case 1: MONARCH_LAUNCH_SPL_ACT(1); break;
        case 2: MONARCH_LAUNCH_SPL_ACT(2); break;
        case 3: MONARCH_LAUNCH_SPL_ACT(3); break;
        case 4: MONARCH_LAUNCH_SPL_ACT(4); break;
        case 5: MONARCH_LAUNCH_SPL_ACT(5); break;
        default: MONARCH_LAUNCH_SPL_ACT(6); break;
        }
#undef MONARCH_LAUNCH_SPL_ACT
#undef MONARCH_LAUNCH_SPL
        MONARCH_HIP_CHECK(hipGetLastError());
        return MONARCH_OK;
    }
    // two partial tiles (din/16 row tiles x 4 column tiles x 64 lanes x 16 B) + the summed [64][din+1] tile
    const size_t lds = (size_t)2 * (din / 16) * 4 * 64 * 16 + (size_t)mlp1::TOK * (din + 1) * sizeof(float);
#define MONARCH_LAUNCH_MLP1(KSV, ACTV)                                                                          \
    do {                                                                                                        \
        auto kern = mlp1::mlp_order1_kernel<E, KSV, ACTV>;                                                         \
        if (lds > 64 * 1024)                                                                                    \
            MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, \
                                                  (int)lds));                                                   \
        hipLaunchKernelGGL(kern, grid, dim3(256), lds, s, (const E *)x, (E *)y, tokens, d, d_hidden,  \
                           nb, (const E *)W1, (const E *)b1, (const E *)W2, (const E *)b2,   \
                           b1_interleaved);                                                                     \
    } while (0)
#define MONARCH_LAUNCH_MLP1_ACT(KSV)                     \
    do {                                                 \
        if (act == 2) MONARCH_LAUNCH_MLP1(KSV, 2);       \
        else if (act == 1) MONARCH_LAUNCH_MLP1(KSV, 1);  \
        else MONARCH_LAUNCH_MLP1(KSV, 0);                \
    } while (0)
    switch (din / 32) {
    case 1: MONARCH_LAUNCH_MLP1_ACT(1); break;
    case 2: MONARCH_LAUNCH_MLP1_ACT(2); break;
    case 3: MONARCH_LAUNCH_MLP1_ACT(3); break;
    case 4: MONARCH_LAUNCH_MLP1_ACT(4); break;
    case 5: MONARCH_LAUNCH_MLP1_ACT(5); break;
    default: MONARCH_LAUNCH_MLP1_ACT(6); break;
    }
#undef MONARCH_LAUNCH_MLP1_ACT
#undef MONARCH_LAUNCH_MLP1
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

}  // namespace

int launch_mlp_mfma_order1(const void *x, void *y, int64_t tokens, int d, int d_hidden, int nb,
                           const void *W1, const void *b1, const void *W2, const void *b2, int act,
                           int b1_interleaved, monarch_dtype dt, hipStream_t s)
{
    if (dt == MONARCH_F16)
        return launch_typed<f16_t>(x, y, tokens, d, d_hidden, nb, W1, b1, W2, b2, act, b1_interleaved, s);
    return launch_typed<bf16_t>(x, y, tokens, d, d_hidden, nb, W1, b1, W2, b2, act, b1_interleaved, s);
}

}  // namespace monarch
