// Sequence mixer with two general (learned) order-2 Monarch matrices, Sec. 3.2 Eq. 2 and its gated form:
//   y[b,h,:] = g_out[b,h,:] o ( M2 ( K[h,:] o ( M1 ( g_in[b,h,:] o u[b,h,:] ) ) ) )
// M1 = P L1 P R1 P, M2 = P L2 P R2 P (Sec. 3.1), square, N = bs^2, factors [bs][bs][bs] shared by all channels;
// K is the kernel in the transform domain, one row per channel.  (With M1 the DFT and M2 its inverse this is
// the convolution of monarch_causal_conv; here the matrices are arbitrary real ones.)  A row never leaves the
// chip between its load and its store: both products, the kernel product and the gates are fused.
//
// Options (MixOpt) turn the same kernels into the two halves of the paper's basic M2 layer: an activation between
// the kernel product and the second matrix; u and y addressed as (B, N, H) instead of (B, H, N), so that the
// sequence mixer reads and writes the layer's (batch, position, feature) tensors without a transpose pass; and an
// epilogue y = LayerNorm(result + u) over the row (skip connection and normalisation of the dimension mixer).
#include "kernels.h"
#include "lds_dma.h"

namespace monarch {

__device__ __forceinline__ float mix_act(float v, int act) { return act == 1 ? fmaxf(v, 0.0f) : v; }

// ---- any block size: fp32 arithmetic on tiles of rows in LDS ------------------------------------------
namespace mixg {

constexpr int THREADS = 256;

// One block-diagonal factor W [bs][bs][bs] on TV rows: block k reads in[v][k * ks_in + c * cs_in] and writes
// out[v][r * rs_out + k * ks_out] (the stride pairs realise the permutations of M = P L P R P).
template <typename T, int TV>
__device__ __forceinline__ void factor(const float *in, float *out, int N, int bs, const T *W, int cs_in, int ks_in,
                                       int rs_out, int ks_out)
{
    for (int o = threadIdx.x; o < N; o += THREADS) {   // o = k bs + r
        const int k = o / bs, r = o - k * bs;
        float acc[TV];
#pragma unroll
        for (int v = 0; v < TV; ++v) acc[v] = 0.0f;
        const T *w = W + (size_t)o * bs;
        for (int c = 0; c < bs; ++c) {
            const float wv = to_f32(w[c]);
#pragma unroll
            for (int v = 0; v < TV; ++v) acc[v] = fmaf(wv, in[v * N + k * ks_in + c * cs_in], acc[v]);
        }
#pragma unroll
        for (int v = 0; v < TV; ++v) out[v * N + r * rs_out + k * ks_out] = acc[v];
    }
}

template <typename T, int TV>
__global__ __launch_bounds__(THREADS) void mixer_kernel(const T *__restrict__ u, const T *__restrict__ K,
                                                        const T *__restrict__ g_in, const T *__restrict__ g_out,
                                                        const T *__restrict__ R1, const T *__restrict__ L1,
                                                        const T *__restrict__ R2, const T *__restrict__ L2,
                                                        T *__restrict__ y, int64_t rows, int H, int bs,
                                                        const MixOpt opt)
{
    extern __shared__ float lds[];
    const int N = bs * bs;
    float *a = lds, *t = lds + TV * N;
    // element j of row r = b H + h: (B, H, N) or, transposed, (B, N, H)
    auto at = [&](int64_t r, int j) -> int64_t { return opt.transposed ? ((r / H) * N + j) * H + r % H : r * N + j; };
    const int64_t ntiles = (rows + TV - 1) / TV;
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t r0 = tile * TV;
        for (int idx = threadIdx.x; idx < TV * N; idx += THREADS) {
            const int v = idx / N, j = idx - v * N;
            float x = 0.0f;
            if (r0 + v < rows) {
                x = to_f32(u[at(r0 + v, j)]);
                if (g_in) x *= to_f32(g_in[at(r0 + v, j)]);
            }
            a[idx] = x;
        }
        __syncthreads();
        factor<T, TV>(a, t, N, bs, R1, bs, 1, bs, 1);   // block k reads a[c bs + k], writes t[r bs + k]
        __syncthreads();
        factor<T, TV>(t, a, N, bs, L1, 1, bs, bs, 1);   // block k reads t[k bs + a'], writes a[r bs + k]
        __syncthreads();
        for (int idx = threadIdx.x; idx < TV * N; idx += THREADS) {
            const int v = idx / N, j = idx - v * N;
            if (r0 + v < rows) a[idx] = mix_act(a[idx] * to_f32(K[((r0 + v) % H) * (int64_t)N + j]), opt.act);
        }
        __syncthreads();
        factor<T, TV>(a, t, N, bs, R2, bs, 1, bs, 1);
        __syncthreads();
        factor<T, TV>(t, a, N, bs, L2, 1, bs, bs, 1);
        __syncthreads();
        if (opt.layer_norm) {
            // rows of result + u; wave w normalises rows w, w + 4, ... (two passes: mean, then variance)
            for (int idx = threadIdx.x; idx < TV * N; idx += THREADS) {
                const int v = idx / N, j = idx - v * N;
                if (r0 + v < rows) {
                    float o = a[idx];
                    if (g_out) o *= to_f32(g_out[at(r0 + v, j)]);
                    a[idx] = o + to_f32(u[at(r0 + v, j)]);
                }
            }
            __syncthreads();
            const int lane = threadIdx.x & 63;
            for (int v = threadIdx.x >> 6; v < TV; v += THREADS / 64) {
                float sum = 0.0f;
                for (int j = lane; j < N; j += 64) sum += a[v * N + j];
                for (int m = 32; m; m >>= 1) sum += __shfl_xor(sum, m);
                const float mean = sum / N;
                float sq = 0.0f;
                for (int j = lane; j < N; j += 64) sq += (a[v * N + j] - mean) * (a[v * N + j] - mean);
                for (int m = 32; m; m >>= 1) sq += __shfl_xor(sq, m);
                const float rstd = rsqrtf(sq / N + opt.eps);
                if (r0 + v < rows)
                    for (int j = lane; j < N; j += 64)
                        y[at(r0 + v, j)] = from_f32<T>((a[v * N + j] - mean) * rstd * to_f32(((const T *)opt.gamma)[j]) +
                                                       to_f32(((const T *)opt.beta)[j]));
            }
        } else {
            for (int idx = threadIdx.x; idx < TV * N; idx += THREADS) {
                const int v = idx / N, j = idx - v * N;
                if (r0 + v < rows) {
                    float o = a[idx];
                    if (g_out) o *= to_f32(g_out[at(r0 + v, j)]);
                    y[at(r0 + v, j)] = from_f32<T>(o);
                }
            }
        }
        __syncthreads();
    }
}

template <typename T>
static int launch_typed(const void *u, const void *K, const void *g_in, const void *g_out, const void *R1, const void *L1,
                        const void *R2, const void *L2, void *y, int64_t rows, int H, int bs, const MixOpt &opt,
                        hipStream_t s)
{
    const int N = bs * bs;
    int tv = 8;
    while (tv > 1 && (size_t)2 * tv * N * sizeof(float) > 64 * 1024) tv >>= 1;
    const size_t lds = (size_t)2 * tv * N * sizeof(float);
    if (lds > 160 * 1024) return fail(MONARCH_ESHAPE, "a row of %d elements does not fit in LDS twice", N);
    int dev = 0, ncu = 0;
    MONARCH_HIP_CHECK(hipGetDevice(&dev));
    MONARCH_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
    const int64_t ntiles = (rows + tv - 1) / tv;
    int64_t grid = (int64_t)ncu * (lds <= 40 * 1024 ? 4 : lds <= 80 * 1024 ? 2 : 1);
    if (grid > ntiles) grid = ntiles;
#define MONARCH_LAUNCH_MIXG(TVV)                                                                                    \
    do {                                                                                                            \
        auto kern = mixer_kernel<T, TVV>;                                                                           \
        if (lds > 64 * 1024)                                                                                        \
            MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,   \
                                                  (int)lds));                                                       \
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(THREADS), lds, s, (const T *)u, (const T *)K,           \
                           (const T *)g_in, (const T *)g_out, (const T *)R1, (const T *)L1, (const T *)R2,          \
                           (const T *)L2, (T *)y, rows, H, bs, opt);                                                \
    } while (0)
    switch (tv) {
    case 8: MONARCH_LAUNCH_MIXG(8); break;
    case 4: MONARCH_LAUNCH_MIXG(4); break;
    case 2: MONARCH_LAUNCH_MIXG(2); break;
    default: MONARCH_LAUNCH_MIXG(1); break;
    }
#undef MONARCH_LAUNCH_MIXG
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

}  // namespace mixg

// ---- bs = 16 (N = 256), fp32, on the matrix cores -------------------------------------------------------
// Four block-diagonal products of 16x16x4 fp32 MFMAs per row, rows on the MFMA column index.  A workgroup (4
// waves) takes a tile of 16 rows; wave w owns the blocks 4 w .. 4 w + 3 of every factor (64 registers of
// weights for the whole kernel).  Rows of u, g_in and g_out come in by direct-to-LDS loads (a row = 1 KB = one
// wave instruction); between the factors of a Monarch matrix the rows cross between the waves through an LDS
// tile whose index map is the middle permutation; between the two matrices they sit as plain rows.
//   S1: T_a[i, v]  = sum_c R1_a[i, c] (g_in u)[v][16 c + a]          -> tile (v, i, a)
//   S2: z[v][16 k + i] = K[h_v][16 k + i] sum_a L1_i[k, a] T_a[i, v]  -> rows
//   S3, S4: the same with R2, L2 and g_out in place of K              -> rows, stored with 16-byte accesses
namespace mix16 {

typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int B = 16, N = 256, TV = 16;
constexpr int LDX = N + 4;                 // pitch of the row buffers
constexpr int RS = 18, LD = B * RS + 3;    // tile: element (v, p, q) at v LD + p RS + q
constexpr int TRANSPOSED_RUN = 8;
constexpr int STATS = 4 * TV;              // per wave and row: a partial sum (layer norm)
constexpr size_t LDS_BYTES = sizeof(float) * (3 * TV * LDX + TV * LD + STATS + 2 * N);

__device__ __forceinline__ f32x4 mfma(float a, float b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// four consecutive elements (16-byte aligned for float, 8-byte aligned for bf16) as floats, and back
__device__ __forceinline__ f32x4 ld4(const float *p) { return *reinterpret_cast<const f32x4 *>(p); }
__device__ __forceinline__ f32x4 ld4(const bf16_t *p)
{
    const uint2 w = *reinterpret_cast<const uint2 *>(p);
    return f32x4{__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xffff0000u), __uint_as_float(w.y << 16),
                 __uint_as_float(w.y & 0xffff0000u)};
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    const bf16_t a = from_f32<bf16_t>(lo), b = from_f32<bf16_t>(hi);
    return (uint32_t) * reinterpret_cast<const uint16_t *>(&a) | ((uint32_t) * reinterpret_cast<const uint16_t *>(&b) << 16);
}

// T: type of every tensor in memory; everything on chip is float.
//
// Three row buffers.  Rows of u (and g_in) wait in two of them; the third takes z between the matrices, then the
// output gates, then the rows of y (each lane overwrites the gate values it has just used).  As soon as the first
// factor has consumed a tile's inputs, the inputs of the workgroup's next tile are requested into the buffers that
// have become free (float: direct-to-LDS loads; bf16: into registers, widened into LDS after the third factor),
// together with this tile's kernel entries and output gates (registers), so that no stage of a tile waits for
// memory except the very first.  Without input gates u alternates between two buffers, which keeps this tile's u
// for the skip connection of the layer-norm epilogue.  Not prefetched: the (B, N, H) access, and the layer-norm
// epilogue combined with input gates.
template <typename T, bool GIN, bool GOUT>
__global__ __launch_bounds__(256, 2) void mixer_b16_kernel(const T *__restrict__ u, const T *__restrict__ K,
                                                           const T *__restrict__ g_in, const T *__restrict__ g_out,
                                                           const T *__restrict__ R1, const T *__restrict__ L1,
                                                           const T *__restrict__ R2, const T *__restrict__ L2,
                                                           T *__restrict__ y, int64_t rows, int H,
                                                           const MixOpt opt)
{
    constexpr bool F32 = sizeof(T) == 4;
    constexpr int NW = F32 ? 4 : 2;    // registers' worth of 16-byte pieces a lane holds of an array of a tile
    extern __shared__ __attribute__((aligned(16))) float smem[];
    float *bufA = smem;                // [TV][LDX] each
    float *bufB = bufA + TV * LDX;
    float *bufC = bufB + TV * LDX;
    float *tt = bufC + TV * LDX;       // tile between the two factors of a matrix: (v, i, a)
    float *stats = tt + TV * LD;       // [4 waves][TV]
    float *gb = stats + STATS;         // layer norm: weight [N], bias [N]
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63, l16 = lane & 15, kg = lane >> 4;
    const int b0 = 4 * wave;

    // A operands: k-step s of block q holds W[b0 + q][row l16][4 kg + s]
    float R1w[4][4], L1w[4][4], R2w[4][4], L2w[4][4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int at = ((b0 + q) * B + l16) * B + 4 * kg + s;
            R1w[q][s] = to_f32(R1[at]);
            L1w[q][s] = to_f32(L1[at]);
            R2w[q][s] = to_f32(R2[at]);
            L2w[q][s] = to_f32(L2[at]);
        }

    if (opt.layer_norm) {
        gb[threadIdx.x] = to_f32(((const T *)opt.gamma)[threadIdx.x]);
        gb[N + threadIdx.x] = to_f32(((const T *)opt.beta)[threadIdx.x]);   // (published by the first barrier of the loop)
    }

    const int64_t ntiles = (rows + TV - 1) / TV;
    // This wave's four rows of a tile (4 w .. 4 w + 3; rows past the end: the last one, never stored) as 16-byte
    // pieces: float: piece `lane` of row 4 w + i; bf16: piece lane % 32 of row 4 w + 2 i + lane / 32.
    auto piece = [&](const T *src, int64_t r0, int i) -> const T * {
        int64_t r = r0 + b0 + (F32 ? i : 2 * i + (lane >> 5));
        if (r >= rows) r = rows - 1;
        return src + r * N + (F32 ? 4 * lane : 8 * (lane & 31));
    };
    auto load_rows = [&](const T *src, int64_t r0, uint4 (&w)[NW]) {
#pragma unroll
        for (int i = 0; i < NW; ++i) w[i] = *reinterpret_cast<const uint4 *>(piece(src, r0, i));
    };
    auto park_rows = [&](const uint4 (&w)[NW], float *dst) {   // registers -> LDS rows, widened
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            if constexpr (F32) {
                *reinterpret_cast<uint4 *>(dst + (b0 + i) * LDX + 4 * lane) = w[i];
            } else {
                float *d = dst + (b0 + 2 * i + (lane >> 5)) * LDX + 8 * (lane & 31);
                *reinterpret_cast<f32x4 *>(d) = f32x4{__uint_as_float(w[i].x << 16), __uint_as_float(w[i].x & 0xffff0000u),
                                                      __uint_as_float(w[i].y << 16), __uint_as_float(w[i].y & 0xffff0000u)};
                *reinterpret_cast<f32x4 *>(d + 4) = f32x4{__uint_as_float(w[i].z << 16), __uint_as_float(w[i].z & 0xffff0000u),
                                                          __uint_as_float(w[i].w << 16), __uint_as_float(w[i].w & 0xffff0000u)};
            }
        }
    };
    auto dma_rows = [&](const T *src, int64_t r0, float *dst) {   // float only: memory -> LDS rows directly
        const uint32_t base = __builtin_amdgcn_readfirstlane(lds_address(dst));
#pragma unroll
        for (int i = 0; i < 4; ++i)
            dma_16_at(piece(src, r0, i), __builtin_amdgcn_readfirstlane(base + (uint32_t)(b0 + i) * LDX * 4));
    };
    auto fetch_now = [&](const T *src, int64_t r0, float *dst) {
        if constexpr (F32) {
            dma_rows(src, r0, dst);
        } else {
            uint4 w[NW];
            load_rows(src, r0, w);
            park_rows(w, dst);
        }
    };
    // (B, N, H) layout: the 16 rows of a tile are 16 neighbouring channels of one sequence (H is a multiple of 16):
    // 16 sizeof(T) contiguous bytes per position, i.e. TP 16-byte pieces of TE channels.  Lane l of instruction
    // w + 4 i moves piece l % TP of position (w + 4 i) 64 / TP + l / TP; in LDS the values go to (channel, position)
    // and back one by one (the banks of the 64 lanes differ).  All loads of an array are in flight before the first
    // value is stored.  A tile never crosses the end of the batch in this layout.
    constexpr int TP = (int)sizeof(T), TE = 16 / (int)sizeof(T);
    auto tile_base = [&](int64_t r0) -> int64_t { return (r0 / H) * (int64_t)N * H + r0 % H; };
    auto load_transposed = [&](const T *src, int64_t tbase, uint4 (&w)[TP]) {
#pragma unroll
        for (int i = 0; i < TP; ++i) {
            const int p = (wave + 4 * i) * (64 / TP) + lane / TP, c0 = (lane % TP) * TE;
            w[i] = *reinterpret_cast<const uint4 *>(src + tbase + (int64_t)p * H + c0);
        }
    };
    auto park_transposed = [&](const uint4 (&w)[TP], float *dst) {
#pragma unroll
        for (int i = 0; i < TP; ++i) {
            const int p = (wave + 4 * i) * (64 / TP) + lane / TP, c0 = (lane % TP) * TE;
            float *d = dst + c0 * LDX + p;
            if constexpr (F32) {
                d[0] = __uint_as_float(w[i].x); d[LDX] = __uint_as_float(w[i].y);
                d[2 * LDX] = __uint_as_float(w[i].z); d[3 * LDX] = __uint_as_float(w[i].w);
            } else {
                d[0] = __uint_as_float(w[i].x << 16); d[LDX] = __uint_as_float(w[i].x & 0xffff0000u);
                d[2 * LDX] = __uint_as_float(w[i].y << 16); d[3 * LDX] = __uint_as_float(w[i].y & 0xffff0000u);
                d[4 * LDX] = __uint_as_float(w[i].z << 16); d[5 * LDX] = __uint_as_float(w[i].z & 0xffff0000u);
                d[6 * LDX] = __uint_as_float(w[i].w << 16); d[7 * LDX] = __uint_as_float(w[i].w & 0xffff0000u);
            }
        }
    };
    auto fetch_transposed = [&](const T *src, int64_t tbase, float *dst) {
        uint4 w[TP];
        load_transposed(src, tbase, w);
        park_transposed(w, dst);
    };
    // tile number of this workgroup's it-th tile (-1: none).  (B, N, H) layout: a tile covers 64 of the bytes of a
    // position; a workgroup takes `run` neighbouring tiles one after the other, so that the other bytes of the
    // lines it has fetched are used while they are still in its L2
    const int run = opt.transposed ? opt.run : 1;
    auto tile_of = [&](int64_t it) -> int64_t {
        const int64_t first = ((int64_t)blockIdx.x + (it / run) * gridDim.x) * run;
        if (first >= ntiles) return -2;               // past the end: stop
        return first + it % run < ntiles ? first + it % run : -1;   // -1: a hole at the end of the last run
    };

    // (float rows in the (B, H, N) layout are not prefetched: the compiler's own waits for the register loads of a tile count loads in
    // issue order and would also wait for direct-to-LDS loads of the next tile issued before them; the float
    // kernel runs at the rate of a plain copy as it is)
    const bool prefetch = (!F32 || opt.transposed) && !(opt.layer_norm && GIN);
    // the kernel entries a lane multiplies in S2: K[h_v][16 (4 kg + r) + b0 .. + 3], v = l16
    f32x4 kq[4];
    auto load_kernel = [&](int64_t r0, f32x4 (&k)[4]) {
        int64_t r = r0 + l16;
        if (r >= rows) r = rows - 1;
        const T *krow = K + (r % H) * (int64_t)N + b0;
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) k[rr] = ld4(krow + 16 * (4 * kg + rr));
    };
    float *ub = bufA, *nb = bufB;      // rows of u of this tile; where the next tile's go when there are no input gates
    if (prefetch && tile_of(0) >= 0) {
        if (opt.transposed) {
            fetch_transposed(u, tile_base(tile_of(0) * TV), ub);
            if (GIN) fetch_transposed(g_in, tile_base(tile_of(0) * TV), bufB);
        } else {
            fetch_now(u, tile_of(0) * TV, ub);
            if (GIN) fetch_now(g_in, tile_of(0) * TV, bufB);
        }
    }
    for (int64_t it = 0;; ++it) {
        const int64_t tile = tile_of(it);
        if (tile == -2) break;
        if (tile < 0) continue;
        const int64_t r0 = tile * TV;
        const int64_t next = prefetch ? tile_of(it + 1) : -1;
        const int64_t tbase = tile_base(r0);
        if (prefetch) {
        } else if (opt.transposed) {
            fetch_transposed(u, tbase, ub);
            if (GIN) fetch_transposed(g_in, tbase, bufB);
        } else {
            fetch_now(u, r0, ub);
            if (GIN) fetch_now(g_in, r0, bufB);
        }
        load_kernel(r0, kq);
        if (F32) wait_loads_at_most<0>();   // the direct-to-LDS loads (bf16 rows pass through registers)
        __syncthreads();

        auto first_factor = [&](const float *rows_in, const float (&W)[4][4], bool gated) {
            f32x4 xq[4];   // [s]: elements 16 (4 kg + s) + b0 .. + 3 of row v = l16
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                xq[s] = *reinterpret_cast<const f32x4 *>(rows_in + l16 * LDX + 16 * (4 * kg + s) + b0);
                if (gated) xq[s] *= *reinterpret_cast<const f32x4 *>(bufB + l16 * LDX + 16 * (4 * kg + s) + b0);
            }
            // (the four blocks' accumulators in turn: an MFMA never waits for the one issued just before it)
            f32x4 t[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) t[q] = f32x4{0, 0, 0, 0};
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int q = 0; q < 4; ++q) t[q] = mfma(W[q][s], xq[s][q], t[q]);   // rows i = 4 kg + r of block a = b0 + q
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int r = 0; r < 4; ++r) tt[l16 * LD + (4 * kg + r) * RS + b0 + q] = t[q][r];   // (v, i, a)
        };
        auto second_factor = [&](const float (&W)[4][4], f32x4 (&out)[4]) {
            // block i = b0 + q contracts a = 4 kg + s of tile row i; result rows k = 4 kg + r: element 16 k + i
#pragma unroll
            for (int q = 0; q < 4; ++q) out[q] = f32x4{0, 0, 0, 0};
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int q = 0; q < 4; ++q) out[q] = mfma(W[q][s], tt[l16 * LD + (b0 + q) * RS + 4 * kg + s], out[q]);
        };

        first_factor(ub, R1w, GIN);
        __syncthreads();

        // requested here, to arrive while the next three stages run: this tile's output gates (into registers; float
        // rows in the (B, H, N) layout come by direct-to-LDS loads once z is consumed) ...
        static_assert(NW == TP, "one register array serves both layouts");
        uint4 gq[NW];
        if (GOUT) {
            if (opt.transposed) load_transposed(g_out, tbase, gq);
            else if (!F32) load_rows(g_out, r0, gq);
        }
        // ... and the next tile's inputs: the first factor has consumed the buffers they go to
        float *u_next = GIN ? bufA : nb;
        constexpr int PW = NW > TP ? NW : TP;
        uint4 pu[PW], pg[PW];
        if (next >= 0) {
            if (opt.transposed) {
                load_transposed(u, tile_base(next * TV), reinterpret_cast<uint4(&)[TP]>(pu));
                if (GIN) load_transposed(g_in, tile_base(next * TV), reinterpret_cast<uint4(&)[TP]>(pg));
            } else if constexpr (!F32) {
                load_rows(u, next * TV, reinterpret_cast<uint4(&)[NW]>(pu));
                if (GIN) load_rows(g_in, next * TV, reinterpret_cast<uint4(&)[NW]>(pg));
            }
        }

        f32x4 z[4];
        second_factor(L1w, z);
        // rows between the matrices: z[v][16 (4 kg + r) + b0 + q], times the kernel of the row's channel
#pragma unroll
        for (int r = 0; r < 4; ++r)
            *reinterpret_cast<f32x4 *>(bufC + l16 * LDX + 16 * (4 * kg + r) + b0) =
                f32x4{mix_act(z[0][r] * kq[r][0], opt.act), mix_act(z[1][r] * kq[r][1], opt.act),
                      mix_act(z[2][r] * kq[r][2], opt.act), mix_act(z[3][r] * kq[r][3], opt.act)};
        __syncthreads();
        first_factor(bufC, R2w, false);
        __syncthreads();   // z is consumed: the output gates take its place
        if (GOUT) {
            if (opt.transposed) {
                park_transposed(gq, bufC);
            } else if constexpr (F32) {
                dma_rows(g_out, r0, bufC);
            } else {
                park_rows(gq, bufC);
            }
        }
        if (next >= 0) {
            if (opt.transposed) {
                park_transposed(reinterpret_cast<uint4(&)[TP]>(pu), u_next);
                if (GIN) park_transposed(reinterpret_cast<uint4(&)[TP]>(pg), bufB);
            } else if constexpr (!F32) {
                park_rows(reinterpret_cast<uint4(&)[NW]>(pu), u_next);
                if (GIN) park_rows(reinterpret_cast<uint4(&)[NW]>(pg), bufB);
            }
        }
        second_factor(L2w, z);
        if (GOUT) {
            if (F32) wait_loads_at_most<0>();
            __syncthreads();
        }
        f32x4 o[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            o[r] = f32x4{z[0][r], z[1][r], z[2][r], z[3][r]};
            if (GOUT) o[r] *= *reinterpret_cast<const f32x4 *>(bufC + l16 * LDX + 16 * (4 * kg + r) + b0);
        }
        if (opt.layer_norm) {
            // skip connection (this tile's u is still in its buffer), then the row's mean and variance in two
            // passes: 16 values per lane, the 4 lane groups of a wave by shuffles, the 4 waves through LDS
            float part = 0.0f;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                o[r] += *reinterpret_cast<const f32x4 *>(ub + l16 * LDX + 16 * (4 * kg + r) + b0);
                part += o[r][0] + o[r][1] + o[r][2] + o[r][3];
            }
            part += __shfl_xor(part, 16);
            part += __shfl_xor(part, 32);
            if (kg == 0) stats[wave * TV + l16] = part;
            __syncthreads();
            const float mean = (stats[l16] + stats[TV + l16] + stats[2 * TV + l16] + stats[3 * TV + l16]) * (1.0f / N);
            __syncthreads();
            part = 0.0f;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                o[r] -= mean;
                part += o[r][0] * o[r][0] + o[r][1] * o[r][1] + o[r][2] * o[r][2] + o[r][3] * o[r][3];
            }
            part += __shfl_xor(part, 16);
            part += __shfl_xor(part, 32);
            if (kg == 0) stats[wave * TV + l16] = part;
            __syncthreads();
            const float var = (stats[l16] + stats[TV + l16] + stats[2 * TV + l16] + stats[3 * TV + l16]) * (1.0f / N);
            const float rstd = rsqrtf(var + opt.eps);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int j = 16 * (4 * kg + r) + b0;
                o[r] = o[r] * rstd * *reinterpret_cast<const f32x4 *>(gb + j) + *reinterpret_cast<const f32x4 *>(gb + N + j);
            }
        }
        // rows of y over the gates: every lane overwrites exactly the positions it has read
#pragma unroll
        for (int r = 0; r < 4; ++r) *reinterpret_cast<f32x4 *>(bufC + l16 * LDX + 16 * (4 * kg + r) + b0) = o[r];
        __syncthreads();
        if (opt.transposed) {
#pragma unroll
            for (int i = 0; i < TP; ++i) {
                const int p = (wave + 4 * i) * (64 / TP) + lane / TP, c0 = (lane % TP) * TE;
                float v[TE];
#pragma unroll
                for (int e = 0; e < TE; ++e) v[e] = bufC[(c0 + e) * LDX + p];
                T *dst = y + tbase + (int64_t)p * H + c0;
                if constexpr (F32) *reinterpret_cast<f32x4 *>(dst) = f32x4{v[0], v[1], v[2], v[3]};
                else *reinterpret_cast<uint4 *>(dst) = uint4{pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7])};
            }
        } else if constexpr (F32) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int64_t r = r0 + b0 + q;
                if (r < rows)   // (y is written once per launch, whole cache lines per instruction: streaming stores)
                    __builtin_nontemporal_store(*reinterpret_cast<const f32x4 *>(bufC + (b0 + q) * LDX + 4 * lane), reinterpret_cast<f32x4 *>(y + r * N + 4 * lane));
            }
        } else {
#pragma unroll
            for (int i = 0; i < 2; ++i) {   // two rows per instruction, 8 elements (16 bytes) per lane
                const int v = b0 + 2 * i + (lane >> 5);
                const f32x4 lo = *reinterpret_cast<const f32x4 *>(bufC + v * LDX + 8 * (lane & 31));
                const f32x4 hi = *reinterpret_cast<const f32x4 *>(bufC + v * LDX + 8 * (lane & 31) + 4);
                if (r0 + v < rows)
                    store_stream16(y + (r0 + v) * N + 8 * (lane & 31),
                                   uint4{pack_bf16(lo[0], lo[1]), pack_bf16(lo[2], lo[3]), pack_bf16(hi[0], hi[1]), pack_bf16(hi[2], hi[3])});
            }
        }
        // (no barrier here: the next tile's first barrier comes before anything of this tile's buffers is rewritten,
        // except the inputs requested above into buffers that were free)
        if (!GIN && next >= 0) {
            float *t = ub;
            ub = nb;
            nb = t;
        }

    }
}

}  // namespace mix16

bool mixer_fits(int bs) { return bs >= 1 && (size_t)2 * bs * bs * sizeof(float) <= 160 * 1024; }

int launch_mixer(const void *u, const void *K, const void *g_in, const void *g_out, const void *R1, const void *L1,
                 const void *R2, const void *L2, void *y, int64_t rows, int H, int bs, monarch_dtype dt,
                 const MixOpt &opt, hipStream_t s)
{
    if (rows == 0) return MONARCH_OK;
    if (bs == 16 && (!opt.transposed || H % 16 == 0)) {
        int dev = 0, ncu = 0;
        MONARCH_HIP_CHECK(hipGetDevice(&dev));
        MONARCH_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
        const int64_t ntiles = (rows + mix16::TV - 1) / mix16::TV;
        // runs of neighbouring tiles only when there are tiles enough to keep every workgroup busy with whole runs
        MixOpt o16 = opt;
        o16.run = 1;
        while (o16.run < mix16::TRANSPOSED_RUN && ntiles >= 2 * (int64_t)ncu * 2 * o16.run && (H / 16) % (2 * o16.run) == 0)
            o16.run *= 2;
        const int64_t nruns = opt.transposed ? (ntiles + o16.run - 1) / o16.run : ntiles;
        int64_t grid = 2 * (int64_t)ncu;
        if (grid > nruns) grid = nruns;
#define MONARCH_LAUNCH_MIX16(T, GI, GO)                                                                            \
    do {                                                                                                           \
        auto kern = mix16::mixer_b16_kernel<T, GI, GO>;                                                            \
        MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,      \
                                              (int)mix16::LDS_BYTES));                                             \
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), mix16::LDS_BYTES, s, (const T *)u, (const T *)K, \
                           (const T *)g_in, (const T *)g_out, (const T *)R1, (const T *)L1, (const T *)R2,         \
                           (const T *)L2, (T *)y, rows, H, o16);                                                   \
    } while (0)
#define MONARCH_LAUNCH_MIX16_GATES(T)                                                                              \
    do {                                                                                                           \
        if (g_in && g_out) MONARCH_LAUNCH_MIX16(T, true, true);                                                    \
        else if (g_in) MONARCH_LAUNCH_MIX16(T, true, false);                                                       \
        else if (g_out) MONARCH_LAUNCH_MIX16(T, false, true);                                                      \
        else MONARCH_LAUNCH_MIX16(T, false, false);                                                                \
    } while (0)
        if (dt == MONARCH_F32) MONARCH_LAUNCH_MIX16_GATES(float);
        else MONARCH_LAUNCH_MIX16_GATES(bf16_t);
#undef MONARCH_LAUNCH_MIX16_GATES
#undef MONARCH_LAUNCH_MIX16
        MONARCH_HIP_CHECK(hipGetLastError());
        return MONARCH_OK;
    }
    // blocks of 32 or 64: in place on the matrix cores
    if (mixer_inplace_takes(bs, H, dt, opt)) return launch_mixer_inplace(u, K, g_in, g_out, R1, L1, R2, L2, y, rows, H, bs, dt, opt, s);
    if (dt == MONARCH_F32) return mixg::launch_typed<float>(u, K, g_in, g_out, R1, L1, R2, L2, y, rows, H, bs, opt, s);
    return mixg::launch_typed<bf16_t>(u, K, g_in, g_out, R1, L1, R2, L2, y, rows, H, bs, opt, s);
}

}  // namespace monarch
