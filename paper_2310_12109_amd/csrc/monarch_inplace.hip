// Square order-2 Monarch products with blocks of 32 x 32 or 64 x 64 (N = 1024 or 4096) on the fp32 matrix
// instruction (16x16x4), fp32 or bf16 tensors, fp32 arithmetic:
//   monarch_matmul   y = P L P R P x                                    (Sec. 3.1)
//   monarch_mixer    y = g_out o M2 (K o M1 (g_in o u))                  (Sec. 3.2 Eq. 2 in its gated form)
//   monarch_matmul_backward                  dx = M^T dy, dR, dL            (what training the matrices of Sec. 3.1 needs)
// A workgroup holds a tile of rows in LDS (element hi b + lo of a row at hi SH + lo) and every block-diagonal
// factor works IN PLACE: block k reads the b elements of a row that it contracts (one digit of the index, the other
// digit being the block's number) and writes its b results to the same places.  With x at (c, k):
//   R: block k contracts c (stride SH)  ->  (r, k);     L: block r contracts k (stride 1)  ->  (r, s) = y[s b + r]
// so the three permutations of M = P L P R P cost nothing and the product ends transposed in the tile.  The mixer's
// second matrix takes that layout as it is (R2: block k' = s contracts c' = r with stride 1, L2: block r' contracts
// k' with stride SH) and ends in natural order.  Rows sit on the MFMA column index.  The factors (b^3 floats each) stay
// in L2: a block's matrix is read as the A operand, 16 bytes per lane (lane (row, group g) takes columns
// (b/4) g .. of its row, the contraction index of MFMA j being (b/4) g + j), the next row tile's weights requested
// while the current one is multiplied.
#include "kernels.h"

namespace monarch {

namespace inpl {

typedef __attribute__((ext_vector_type(4))) float f32x4;

__device__ __forceinline__ f32x4 mfma(float a, float b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0); }
__device__ __forceinline__ f32x4 ld4(const float *p) { return *reinterpret_cast<const f32x4 *>(p); }
__device__ __forceinline__ f32x4 ld4(const bf16_t *p)
{
    const uint2 w = *reinterpret_cast<const uint2 *>(p);
    return f32x4{__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xffff0000u), __uint_as_float(w.y << 16),
                 __uint_as_float(w.y & 0xffff0000u)};
}
__device__ __forceinline__ float ld1(const float *p) { return *p; }
__device__ __forceinline__ float ld1(const bf16_t *p) { return __uint_as_float((uint32_t)*reinterpret_cast<const uint16_t *>(p) << 16); }
__device__ __forceinline__ void st4(float *p, f32x4 v) { *reinterpret_cast<f32x4 *>(p) = v; }
// the same for rows that a launch reads or writes once, a wave instruction covering whole cache lines: streaming
// accesses (the plain product: -4.8 % at b = 32, -3.5 % at b = 64 in fp32; the mixer kernel keeps ordinary accesses:
// with the layer's transposed pieces, which take a cache line in several instructions, streaming cost 11 %)
__device__ __forceinline__ f32x4 ld4s(const float *p) { return __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p)); }
__device__ __forceinline__ f32x4 ld4s(const bf16_t *p)
{
    const uint2 w = load_stream8(p);
    return f32x4{__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xffff0000u), __uint_as_float(w.y << 16),
                 __uint_as_float(w.y & 0xffff0000u)};
}
__device__ __forceinline__ void st4s(float *p, f32x4 v) { __builtin_nontemporal_store(v, reinterpret_cast<f32x4 *>(p)); }
__device__ __forceinline__ void st4(bf16_t *p, f32x4 v)
{
    const bf16_t h[4] = {from_f32<bf16_t>(v[0]), from_f32<bf16_t>(v[1]), from_f32<bf16_t>(v[2]), from_f32<bf16_t>(v[3])};
    *reinterpret_cast<uint2 *>(p) = *reinterpret_cast<const uint2 *>(h);
}
__device__ __forceinline__ void st4s(bf16_t *p, f32x4 v)
{
    const bf16_t h[4] = {from_f32<bf16_t>(v[0]), from_f32<bf16_t>(v[1]), from_f32<bf16_t>(v[2]), from_f32<bf16_t>(v[3])};
    store_stream8(p, *reinterpret_cast<const uint2 *>(h));
}

// b = 32: tiles of 16 rows (74 KB: two workgroups of 8 waves per compute unit); b = 64: tiles of 8 rows (139 KB, one
// workgroup of 16 waves; columns 8..15 of the MFMA repeat the rows).  SH = b + 4: four lane groups that read rows
// (b/4) g of a column are 16 banks apart; the row pitch is 1 (mod 64).
template <int BS>
struct Geo {
    static constexpr int N = BS * BS, SH = BS + 4, TV = BS == 32 ? 16 : 8, ROWP = BS * SH + 1;
    static constexpr int THREADS = BS == 32 ? 512 : 1024, WAVES = THREADS / 64, NBW = BS / WAVES;
    static constexpr int Q = BS / 4, RT = BS / 16;   // contraction indices per lane group; row tiles of a block
    static constexpr size_t LDS_BYTES = sizeof(float) * TV * ROWP;
};

// One factor in place.  Block blk contracts the digit that has stride SK; its other digit puts it at at(blk).
// TRANS: the transposed blocks (lane (row i, group g) takes W[blk][(b/4) g + j][i]: a column of the block, 4-byte
// loads that run along i across the 16 lanes of a group).
template <typename T, int BS, int SK, bool TRANS = false, typename At>
__device__ __forceinline__ void stage(float *tile, const T *__restrict__ W, int wave, int lane, At at)
{
    typedef Geo<BS> G;
    const int l16 = lane & 15, kg = lane >> 4;
    float *mine = tile + (l16 & (G::TV - 1)) * G::ROWP;
    constexpr int ITEMS = G::NBW * G::RT, WV = G::Q / 4;   // (block, row tile) pairs of this wave; 16-byte pieces per lane
    f32x4 w[2][WV];
    float anchor = 0.0f;
    // (the pointer passes through an empty asm that names the latest result, so that the compiler keeps each
    // request where it is written instead of hoisting all of a stage's loads to its top)
    auto request = [&](int item, f32x4 (&dst)[WV]) {
        const T *src = W;
        asm volatile("" : "+s"(src) : "v"(anchor));
        const int blk = wave * G::NBW + item / G::RT, rt = item % G::RT;
        if constexpr (TRANS) {
            const T *col = src + ((size_t)blk * BS + G::Q * kg) * BS + 16 * rt + l16;
#pragma unroll
            for (int p = 0; p < WV; ++p)
#pragma unroll
                for (int e = 0; e < 4; ++e) dst[p][e] = ld1(col + (size_t)(4 * p + e) * BS);
        } else {
            const T *row = src + ((size_t)blk * BS + 16 * rt + l16) * BS + G::Q * kg;
#pragma unroll
            for (int p = 0; p < WV; ++p) dst[p] = ld4(row + 4 * p);
        }
    };
    request(0, w[0]);
#pragma unroll
    for (int u = 0; u < G::NBW; ++u) {
        float *e = mine + at(wave * G::NBW + u);
        float bv[G::Q];
#pragma unroll
        for (int j = 0; j < G::Q; ++j) bv[j] = e[(G::Q * kg + j) * SK];
        f32x4 acc[G::RT];
#pragma unroll
        for (int rt = 0; rt < G::RT; ++rt) {
            const int item = u * G::RT + rt;
            if (item + 1 < ITEMS) request(item + 1, w[(item + 1) & 1]);
            f32x4 a = {0, 0, 0, 0};
#pragma unroll
            for (int j = 0; j < G::Q; ++j) a = mfma(w[item & 1][j >> 2][j & 3], bv[j], a);
            acc[rt] = a;
            anchor = a[0];
        }
        // every input of the block has been read: the results take their places
        if (l16 < G::TV) {
#pragma unroll
            for (int rt = 0; rt < G::RT; ++rt)
#pragma unroll
                for (int r = 0; r < 4; ++r) e[(16 * rt + 4 * kg + r) * SK] = acc[rt][r];
        }
    }
}

template <typename T, int BS>
__global__ __launch_bounds__(Geo<BS>::THREADS, BS == 32 ? 2 : 1) void matmul_kernel(const T *__restrict__ x, const T *__restrict__ R,
                                                                                  const T *__restrict__ L, T *__restrict__ y, int64_t batch)
{
    typedef Geo<BS> G;
    extern __shared__ __attribute__((aligned(16))) float tile[];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int64_t ntiles = (batch + G::TV - 1) / G::TV;
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int64_t v0 = t * G::TV;
        for (int piece = threadIdx.x; piece < G::TV * G::N / 4; piece += G::THREADS) {
            const int v = piece / (G::N / 4), i = 4 * (piece % (G::N / 4));
            int64_t r = v0 + v;
            if (r >= batch) r = batch - 1;   // (rows past the end: computed, never stored)
            const f32x4 val = ld4s(x + r * G::N + i);
            float *d = tile + v * G::ROWP + (i / BS) * G::SH + i % BS;
            d[0] = val[0]; d[1] = val[1]; d[2] = val[2]; d[3] = val[3];
        }
        __syncthreads();
        stage<T, BS, G::SH>(tile, R, wave, lane, [](int k) { return k; });
        __syncthreads();
        stage<T, BS, 1>(tile, L, wave, lane, [](int r) { return r * G::SH; });
        __syncthreads();
        // y[s b + r] sits at (r, s): a thread stores r = 4 q .. 4 q + 3 of one s
        for (int piece = threadIdx.x; piece < G::TV * G::N / 4; piece += G::THREADS) {
            const int v = piece / (G::N / 4), m = 4 * (piece % (G::N / 4));
            const float *sp = tile + v * G::ROWP + (m % BS) * G::SH + m / BS;
            if (v0 + v < batch) st4s(y + (v0 + v) * G::N + m, f32x4{sp[0], sp[G::SH], sp[2 * G::SH], sp[3 * G::SH]});
        }
        __syncthreads();
    }
}

// opt: the options of the basic M2 layer (Sec. 3.2): an activation after the kernel product, rows that run along the
// middle index of a (B, N, H) tensor (transposed: a tile's TV rows are TV neighbouring h of one batch entry, moved in
// pieces of four rows of one position), and the skip connection and layer norm over the row at the store.
template <typename T, int BS, bool GIN, bool GOUT>
__global__ __launch_bounds__(Geo<BS>::THREADS, BS == 32 ? 2 : 1) void mixer_kernel(
    const T *__restrict__ u, const T *__restrict__ K, const T *__restrict__ g_in, const T *__restrict__ g_out,
    const T *__restrict__ R1, const T *__restrict__ L1, const T *__restrict__ R2, const T *__restrict__ L2, T *__restrict__ y,
    int64_t rows, int H, const MixOpt opt)
{
    typedef Geo<BS> G;
    extern __shared__ __attribute__((aligned(16))) float tile[];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int64_t ntiles = (rows + G::TV - 1) / G::TV;
    constexpr int PIECES = G::TV * G::N / 4;
    // piece p of a tile: four elements and where they sit.  Plain rows: elements i .. i + 3 of row v; transposed: element i
    // of rows v .. v + 3 (neighbouring h of one batch entry: contiguous in memory).
    auto where = [&](int p, int64_t v0, int &v, int &i) -> int64_t {
        if (opt.transposed) {
            i = p / (G::TV / 4);
            v = 4 * (p % (G::TV / 4));
            // (rows is a multiple of TV here and a tile stays inside one batch entry: v0 = bt H + h0)
            const int64_t bt = v0 / H, h0 = v0 - bt * H;
            return (bt * G::N + i) * H + h0 + v;
        }
        v = p / (G::N / 4);
        i = 4 * (p % (G::N / 4));
        int64_t r = v0 + v;
        if (r >= rows) r = rows - 1;   // (rows past the end: computed, never stored)
        return r * G::N + i;
    };
    // the four tile words of a piece: natural position (hi, lo) = (i / b, i % b)
    auto put = [&](int v, int i, f32x4 val) {
        if (opt.transposed) {
            float *d = tile + v * G::ROWP + (i / BS) * G::SH + i % BS;
            d[0] = val[0]; d[G::ROWP] = val[1]; d[2 * G::ROWP] = val[2]; d[3 * G::ROWP] = val[3];
        } else {
            float *d = tile + v * G::ROWP + (i / BS) * G::SH + i % BS;
            d[0] = val[0]; d[1] = val[1]; d[2] = val[2]; d[3] = val[3];
        }
    };
    auto get = [&](int v, int i) -> f32x4 {
        const float *d = tile + v * G::ROWP + (i / BS) * G::SH + i % BS;
        if (opt.transposed) return f32x4{d[0], d[G::ROWP], d[2 * G::ROWP], d[3 * G::ROWP]};
        return f32x4{d[0], d[1], d[2], d[3]};
    };
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int64_t v0 = t * G::TV;
        for (int piece = threadIdx.x; piece < PIECES; piece += G::THREADS) {
            int v, i;
            const int64_t at = where(piece, v0, v, i);
            f32x4 val = ld4(u + at);
            if (GIN) val *= ld4(g_in + at);
            put(v, i, val);
        }
        __syncthreads();
        stage<T, BS, G::SH>(tile, R1, wave, lane, [](int k) { return k; });
        __syncthreads();
        stage<T, BS, 1>(tile, L1, wave, lane, [](int r) { return r * G::SH; });
        __syncthreads();
        // kernel product: entry m = s b + r of the transform domain sits at (r, s)
        for (int piece = threadIdx.x; piece < PIECES; piece += G::THREADS) {
            const int v = piece / (G::N / 4), m = 4 * (piece % (G::N / 4));
            int64_t r = v0 + v;
            if (r >= rows) r = rows - 1;
            const f32x4 kv = ld4(K + (r % H) * G::N + m);
            float *sp = tile + v * G::ROWP + (m % BS) * G::SH + m / BS;
            f32x4 p = {sp[0] * kv[0], sp[G::SH] * kv[1], sp[2 * G::SH] * kv[2], sp[3 * G::SH] * kv[3]};
            if (opt.act) p = f32x4{fmaxf(p[0], 0.0f), fmaxf(p[1], 0.0f), fmaxf(p[2], 0.0f), fmaxf(p[3], 0.0f)};
            sp[0] = p[0]; sp[G::SH] = p[1]; sp[2 * G::SH] = p[2]; sp[3 * G::SH] = p[3];
        }
        __syncthreads();
        stage<T, BS, 1>(tile, R2, wave, lane, [](int k) { return k * G::SH; });
        __syncthreads();
        stage<T, BS, G::SH>(tile, L2, wave, lane, [](int r) { return r; });
        __syncthreads();
        if (opt.layer_norm) {
            // result (gated) + u back into the tile, then a wave per row: mean, variance, scale and shift
            for (int piece = threadIdx.x; piece < PIECES; piece += G::THREADS) {
                int v, i;
                const int64_t at = where(piece, v0, v, i);
                f32x4 val = get(v, i);
                if (GOUT) val *= ld4(g_out + at);
                put(v, i, val + ld4(u + at));
            }
            __syncthreads();
            for (int v = wave; v < G::TV; v += G::WAVES) {
                const float *row = tile + v * G::ROWP;
                float sum = 0.0f;
                for (int j = lane; j < G::N; j += 64) sum += row[(j / BS) * G::SH + j % BS];
                for (int m = 32; m; m >>= 1) sum += __shfl_xor(sum, m);
                const float mean = sum / G::N;
                float sq = 0.0f;
                for (int j = lane; j < G::N; j += 64) {
                    const float dlt = row[(j / BS) * G::SH + j % BS] - mean;
                    sq += dlt * dlt;
                }
                for (int m = 32; m; m >>= 1) sq += __shfl_xor(sq, m);
                const float rstd = rsqrtf(sq / G::N + opt.eps);
                const int64_t r = v0 + v;
                if (r < rows)
                    for (int j = lane; j < G::N; j += 64) {
                        const int64_t at = opt.transposed ? ((v0 / H) * G::N + j) * H + v0 % H + v : r * G::N + j;
                        y[at] = from_f32<T>((row[(j / BS) * G::SH + j % BS] - mean) * rstd * to_f32(((const T *)opt.gamma)[j]) +
                                            to_f32(((const T *)opt.beta)[j]));
                    }
            }
        } else {
            for (int piece = threadIdx.x; piece < PIECES; piece += G::THREADS) {
                int v, i;
                const int64_t at = where(piece, v0, v, i);
                if (v0 + v < rows) {
                    f32x4 val = get(v, i);
                    if (GOUT) val *= ld4(g_out + at);
                    st4(y + at, val);
                }
            }
        }
        __syncthreads();
    }
}

// ---- gradients (blocks of 32) ----------------------------------------------------------------------------------
// With S = sum_v <dy_v, M x_v>, mid = R-stage of x at (r, k) and dy loaded at (r, s):
//   dmid(r, k) = sum_s L[r][s][k] dy(r, s)    (block r of L transposed contracts s, stride 1)
//   dx(c, k)   = sum_r R[k][r][c] dmid(r, k)  (block k of R transposed contracts r, stride SH)
//   dL[r][s][k] = sum_v dy_v(r, s) mid_v(r, k),   dR[k][r][c] = sum_v dmid_v(r, k) x_v(c, k).
// Two tiles of 16 rows (forward values and gradients, 148 KB): a factor's gradient is, per block and 16 x 16 piece
// of it, four MFMAs whose contraction index is the row of the tile; the sums of a wave's four blocks (64 registers)
// stay in registers over all tiles of the workgroup and are added to the caller's cleared buffer once.  Two
// launches, because x is overwritten by mid and dy by dmid: one gives dx and dL, the other dR.

// sum[u][it][jt] += (rows 16 it .. of side A)^T (rows 16 jt .. of side B) of block wave NBW + u, over the tile's rows
template <int BS, int SK, typename At>
__device__ __forceinline__ void outer(const float *ta, const float *tb, int wave, int lane, At at,
                                      f32x4 (&sum)[Geo<BS>::NBW][Geo<BS>::RT][Geo<BS>::RT])
{
    typedef Geo<BS> G;
    const int l16 = lane & 15, kg = lane >> 4;
#pragma unroll
    for (int u = 0; u < G::NBW; ++u) {
        const int off = at(wave * G::NBW + u);
#pragma unroll
        for (int q = 0; q < G::TV / 4; ++q) {   // the MFMA's contraction index kg is row 4 q + kg of the tile
            const float *ra = ta + (4 * q + kg) * G::ROWP + off, *rb = tb + (4 * q + kg) * G::ROWP + off;
            float a[G::RT], b[G::RT];
#pragma unroll
            for (int it = 0; it < G::RT; ++it) {
                a[it] = ra[(16 * it + l16) * SK];
                b[it] = rb[(16 * it + l16) * SK];
            }
#pragma unroll
            for (int it = 0; it < G::RT; ++it)
#pragma unroll
                for (int jt = 0; jt < G::RT; ++jt) sum[u][it][jt] = mfma(a[it], b[jt], sum[u][it][jt]);
        }
    }
}

template <int BS>
__device__ __forceinline__ void flush(float *dW, int wave, int lane, const f32x4 (&sum)[Geo<BS>::NBW][Geo<BS>::RT][Geo<BS>::RT])
{
    typedef Geo<BS> G;
    const int l16 = lane & 15, kg = lane >> 4;
#pragma unroll
    for (int u = 0; u < G::NBW; ++u)
#pragma unroll
        for (int it = 0; it < G::RT; ++it)
#pragma unroll
            for (int jt = 0; jt < G::RT; ++jt)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    atomicAdd(dW + ((size_t)(wave * G::NBW + u) * BS + 16 * it + 4 * kg + r) * BS + 16 * jt + l16, sum[u][it][jt][r]);
}

// x -> fw tile at (c, k); dy -> gr tile at (r, s), zero for the rows past the batch (their x is a copy of the last row)
template <typename T, int BS>
__device__ __forceinline__ void load_pair(float *fw, float *gr, const T *x, const T *dy, int64_t v0, int64_t batch, bool want_x)
{
    typedef Geo<BS> G;
    for (int piece = threadIdx.x; piece < G::TV * G::N / 4; piece += G::THREADS) {
        const int v = piece / (G::N / 4), i = 4 * (piece % (G::N / 4));
        const bool live = v0 + v < batch;
        const int64_t r = live ? v0 + v : batch - 1;
        if (want_x) {
            const f32x4 val = ld4(x + r * G::N + i);
            float *d = fw + v * G::ROWP + (i / BS) * G::SH + i % BS;
            d[0] = val[0]; d[1] = val[1]; d[2] = val[2]; d[3] = val[3];
        }
        f32x4 g = ld4(dy + r * G::N + i);
        if (!live) g = f32x4{0, 0, 0, 0};
        float *sp = gr + v * G::ROWP + (i % BS) * G::SH + i / BS;   // dy[s b + r] at (r, s): i / b = s, i % b = r .. r + 3
        sp[0] = g[0]; sp[G::SH] = g[1]; sp[2 * G::SH] = g[2]; sp[3 * G::SH] = g[3];
    }
}

template <typename T, int BS, bool DX, bool DL>
__global__ __launch_bounds__(Geo<BS>::THREADS, 1) void backward_dx_dl_kernel(const T *__restrict__ x, const T *__restrict__ R,
                                                                               const T *__restrict__ L, const T *__restrict__ dy,
                                                                               T *__restrict__ dx, float *__restrict__ dL, int64_t batch)
{
    typedef Geo<BS> G;
    extern __shared__ __attribute__((aligned(16))) float tile[];
    float *fw = tile, *gr = tile + G::TV * G::ROWP;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    f32x4 sum[G::NBW][G::RT][G::RT];
#pragma unroll
    for (int u = 0; u < G::NBW; ++u)
#pragma unroll
        for (int it = 0; it < G::RT; ++it)
#pragma unroll
            for (int jt = 0; jt < G::RT; ++jt) sum[u][it][jt] = f32x4{0, 0, 0, 0};
    const int64_t ntiles = (batch + G::TV - 1) / G::TV;
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int64_t v0 = t * G::TV;
        load_pair<T, BS>(fw, gr, x, dy, v0, batch, DL);
        __syncthreads();
        if constexpr (DL) {
            stage<T, BS, G::SH>(fw, R, wave, lane, [](int k) { return k; });   // x -> mid
            __syncthreads();
            outer<BS, 1>(gr, fw, wave, lane, [](int r) { return r * G::SH; }, sum);   // dL[r][s][k]: dy(r, s) x mid(r, k)
            __syncthreads();
        }
        if constexpr (DX) {
            stage<T, BS, 1, true>(gr, L, wave, lane, [](int r) { return r * G::SH; });   // dy -> dmid
            __syncthreads();
            stage<T, BS, G::SH, true>(gr, R, wave, lane, [](int k) { return k; });       // dmid -> dx at (c, k)
            __syncthreads();
            for (int piece = threadIdx.x; piece < G::TV * G::N / 4; piece += G::THREADS) {
                const int v = piece / (G::N / 4), i = 4 * (piece % (G::N / 4));
                const float *sp = gr + v * G::ROWP + (i / BS) * G::SH + i % BS;
                if (v0 + v < batch) st4(dx + (v0 + v) * G::N + i, f32x4{sp[0], sp[1], sp[2], sp[3]});
            }
            __syncthreads();
        }
    }
    if constexpr (DL) flush<BS>(dL, wave, lane, sum);
}

template <typename T, int BS>
__global__ __launch_bounds__(Geo<BS>::THREADS, 1) void backward_dr_kernel(const T *__restrict__ x, const T *__restrict__ L,
                                                                            const T *__restrict__ dy, float *__restrict__ dR, int64_t batch)
{
    typedef Geo<BS> G;
    extern __shared__ __attribute__((aligned(16))) float tile[];
    float *fw = tile, *gr = tile + G::TV * G::ROWP;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    f32x4 sum[G::NBW][G::RT][G::RT];
#pragma unroll
    for (int u = 0; u < G::NBW; ++u)
#pragma unroll
        for (int it = 0; it < G::RT; ++it)
#pragma unroll
            for (int jt = 0; jt < G::RT; ++jt) sum[u][it][jt] = f32x4{0, 0, 0, 0};
    const int64_t ntiles = (batch + G::TV - 1) / G::TV;
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        load_pair<T, BS>(fw, gr, x, dy, t * G::TV, batch, true);
        __syncthreads();
        stage<T, BS, 1, true>(gr, L, wave, lane, [](int r) { return r * G::SH; });   // dy -> dmid at (r, k)
        __syncthreads();
        outer<BS, G::SH>(gr, fw, wave, lane, [](int k) { return k; }, sum);          // dR[k][r][c]: dmid(r, k) x x(c, k)
        __syncthreads();
    }
    flush<BS>(dR, wave, lane, sum);
}

// ---- gradients (blocks of 64) ----------------------------------------------------------------------------------
// The factor gradients (b^3 = 262144 floats each) do not fit in a workgroup's registers, and two tiles of eight rows
// do not fit in LDS.  Three launches:
//   dx: one tile of eight rows, the transposed stages of L and R (as the forward product, reversed);
//   dL: workgroup (group g, slice) sums the 16 blocks r = 16 g .. 16 g + 15, one per wave, over the tiles of its
//       slice of the rows: x whole (tile of four rows), the R stage restricted to the output rows r of the group
//       (one row tile per block k), dy only at (r, s) with r in the group (a compact tile);
//   dR: the same with the 16 blocks k of a group: dy whole, the transposed L stage restricted to the outputs k of
//       the group, x only at (c, k) with k in the group.
// A factor's gradient is then one MFMA per block and 16 x 16 piece (contraction index = the tile's four rows).
constexpr int TV64 = 4;                 // rows of a gradient tile at b = 64
constexpr int CP64 = 16 * 68 + 1;       // floats per row of the compact tile holding (r, s), r in a group of 16: r' 68 + s
constexpr int CX64 = 64 * 20 + 1;       // floats per row of the compact tile holding (c, k), k in a group of 16: c 20 + k'

// One factor in place, restricted to row tile rt0 of every block's outputs (the other positions keep their inputs).
template <typename T, int BS, int SK, bool TRANS, typename At>
__device__ __forceinline__ void stage_one(float *tile, const T *__restrict__ W, int wave, int lane, At at, int rt0, int tv)
{
    typedef Geo<BS> G;
    const int l16 = lane & 15, kg = lane >> 4;
    float *mine = tile + (l16 & (tv - 1)) * G::ROWP;
    constexpr int WV = G::Q / 4;
    f32x4 w[2][WV];
    float anchor = 0.0f;
    auto request = [&](int u, f32x4 (&dst)[WV]) {
        const T *src = W;
        asm volatile("" : "+s"(src) : "v"(anchor));
        const int blk = wave * G::NBW + u;
        if constexpr (TRANS) {
            const T *col = src + ((size_t)blk * BS + G::Q * kg) * BS + 16 * rt0 + l16;
#pragma unroll
            for (int p = 0; p < WV; ++p)
#pragma unroll
                for (int e = 0; e < 4; ++e) dst[p][e] = ld1(col + (size_t)(4 * p + e) * BS);
        } else {
            const T *row = src + ((size_t)blk * BS + 16 * rt0 + l16) * BS + G::Q * kg;
#pragma unroll
            for (int p = 0; p < WV; ++p) dst[p] = ld4(row + 4 * p);
        }
    };
    request(0, w[0]);
#pragma unroll
    for (int u = 0; u < G::NBW; ++u) {
        float *e = mine + at(wave * G::NBW + u);
        float bv[G::Q];
#pragma unroll
        for (int j = 0; j < G::Q; ++j) bv[j] = e[(G::Q * kg + j) * SK];
        if (u + 1 < G::NBW) request(u + 1, w[(u + 1) & 1]);
        f32x4 a = {0, 0, 0, 0};
#pragma unroll
        for (int j = 0; j < G::Q; ++j) a = mfma(w[u & 1][j >> 2][j & 3], bv[j], a);
        anchor = a[0];
        if (l16 < tv) {
#pragma unroll
            for (int r = 0; r < 4; ++r) e[(16 * rt0 + 4 * kg + r) * SK] = a[r];
        }
    }
}

template <typename T>
__global__ __launch_bounds__(1024, 1) void backward64_dx_kernel(const T *__restrict__ R, const T *__restrict__ L, const T *__restrict__ dy,
                                                                  T *__restrict__ dx, int64_t batch)
{
    typedef Geo<64> G;
    constexpr int BS = 64;
    extern __shared__ __attribute__((aligned(16))) float tile[];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int64_t ntiles = (batch + G::TV - 1) / G::TV;
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int64_t v0 = t * G::TV;
        for (int piece = threadIdx.x; piece < G::TV * G::N / 4; piece += G::THREADS) {
            const int v = piece / (G::N / 4), i = 4 * (piece % (G::N / 4));
            int64_t r = v0 + v;
            if (r >= batch) r = batch - 1;   // (rows past the end: computed, never stored)
            const f32x4 g = ld4(dy + r * G::N + i);
            float *sp = tile + v * G::ROWP + (i % BS) * G::SH + i / BS;   // dy[s b + r] at (r, s)
            sp[0] = g[0]; sp[G::SH] = g[1]; sp[2 * G::SH] = g[2]; sp[3 * G::SH] = g[3];
        }
        __syncthreads();
        stage<T, BS, 1, true>(tile, L, wave, lane, [](int r) { return r * G::SH; });   // dy -> dmid at (r, k)
        __syncthreads();
        stage<T, BS, G::SH, true>(tile, R, wave, lane, [](int k) { return k; });       // dmid -> dx at (c, k)
        __syncthreads();
        for (int piece = threadIdx.x; piece < G::TV * G::N / 4; piece += G::THREADS) {
            const int v = piece / (G::N / 4), i = 4 * (piece % (G::N / 4));
            const float *sp = tile + v * G::ROWP + (i / BS) * G::SH + i % BS;
            if (v0 + v < batch) st4(dx + (v0 + v) * G::N + i, f32x4{sp[0], sp[1], sp[2], sp[3]});
        }
        __syncthreads();
    }
}

// WHICH = 0: dL (group of blocks r), 1: dR (group of blocks k).  blockIdx.x = 4 slice + group.
template <typename T, int WHICH>
__global__ __launch_bounds__(1024, 1) void backward64_factor_kernel(const T *__restrict__ x, const T *__restrict__ W,
                                                                      const T *__restrict__ dy, float *__restrict__ dW, int64_t batch)
{
    typedef Geo<64> G;
    constexpr int BS = 64, TV = TV64, CP = WHICH == 0 ? CP64 : CX64;
    extern __shared__ __attribute__((aligned(16))) float tile[];
    float *full = tile, *part = tile + TV * G::ROWP;   // dL: full = x -> mid, part = dy(r in group, s); dR: full = dy -> dmid, part = x(c, k in group)
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int l16 = lane & 15, kg = lane >> 4;
    const int group = blockIdx.x & 3, slice = blockIdx.x >> 2, nslices = gridDim.x >> 2;
    f32x4 sum[4][4];
#pragma unroll
    for (int it = 0; it < 4; ++it)
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) sum[it][jt] = f32x4{0, 0, 0, 0};
    const int64_t ntiles = (batch + TV - 1) / TV;
    for (int64_t t = slice; t < ntiles; t += nslices) {
        const int64_t v0 = t * TV;
        // the whole rows of one operand, 16 elements (64 bytes) per 64 of the other
        for (int piece = threadIdx.x; piece < TV * G::N / 4; piece += G::THREADS) {
            const int v = piece / (G::N / 4), i = 4 * (piece % (G::N / 4));
            const bool live = v0 + v < batch;
            const int64_t r = live ? v0 + v : batch - 1;
            if (WHICH == 0) {
                const f32x4 val = ld4(x + r * G::N + i);
                float *d = full + v * G::ROWP + (i / BS) * G::SH + i % BS;
                d[0] = val[0]; d[1] = val[1]; d[2] = val[2]; d[3] = val[3];
            } else {
                f32x4 g = ld4(dy + r * G::N + i);
                if (!live) g = f32x4{0, 0, 0, 0};
                float *sp = full + v * G::ROWP + (i % BS) * G::SH + i / BS;
                sp[0] = g[0]; sp[G::SH] = g[1]; sp[2 * G::SH] = g[2]; sp[3 * G::SH] = g[3];
            }
        }
        for (int piece = threadIdx.x; piece < TV * 64 * 4; piece += G::THREADS) {   // (one piece per thread)
            const int v = piece >> 8, hi = (piece >> 2) & 63, q = piece & 3;   // element hi b + 16 group + 4 q ..
            const bool live = v0 + v < batch;
            const int64_t r = live ? v0 + v : batch - 1;
            const int i = hi * BS + 16 * group + 4 * q;
            if (WHICH == 0) {   // dy[s b + r], s = hi, r = 16 group + 4 q + e  ->  (r', s) at r' 68 + s
                f32x4 g = ld4(dy + r * G::N + i);
                if (!live) g = f32x4{0, 0, 0, 0};
                float *sp = part + v * CP + (4 * q) * 68 + hi;
                sp[0] = g[0]; sp[68] = g[1]; sp[2 * 68] = g[2]; sp[3 * 68] = g[3];
            } else {            // x[c b + k], c = hi, k = 16 group + 4 q + e  ->  (c, k') at c 20 + k'
                const f32x4 val = ld4(x + r * G::N + i);
                float *d = part + v * CP + hi * 20 + 4 * q;
                d[0] = val[0]; d[1] = val[1]; d[2] = val[2]; d[3] = val[3];
            }
        }
        __syncthreads();
        if (WHICH == 0) stage_one<T, BS, G::SH, false>(full, W, wave, lane, [](int k) { return k; }, group, TV);        // mid(r, k), r in the group
        else stage_one<T, BS, 1, true>(full, W, wave, lane, [](int r) { return r * G::SH; }, group, TV);                // dmid(r, k), k in the group
        __syncthreads();
        // this wave's block: the MFMA's contraction index kg is row kg of the tiles
        {
            const int blk = 16 * group + wave;
            float a[4], b[4];
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                if (WHICH == 0) {   // dL[r][s][k]: dy(r, s) from the compact tile, mid(r, k) from the full one
                    a[it] = part[kg * CP + wave * 68 + 16 * it + l16];
                    b[it] = full[kg * G::ROWP + blk * G::SH + 16 * it + l16];
                } else {            // dR[k][r][c]: dmid(r, k) from the full tile, x(c, k) from the compact one
                    a[it] = full[kg * G::ROWP + (16 * it + l16) * G::SH + blk];
                    b[it] = part[kg * CP + (16 * it + l16) * 20 + wave];
                }
            }
#pragma unroll
            for (int it = 0; it < 4; ++it)
#pragma unroll
                for (int jt = 0; jt < 4; ++jt) sum[it][jt] = mfma(a[it], b[jt], sum[it][jt]);
        }
        __syncthreads();
    }
    const int blk = 16 * group + wave;
#pragma unroll
    for (int it = 0; it < 4; ++it)
#pragma unroll
        for (int jt = 0; jt < 4; ++jt)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                atomicAdd(dW + ((size_t)blk * BS + 16 * it + 4 * kg + r) * BS + 16 * jt + l16, sum[it][jt][r]);
}

// ---- the polynomial-parameterised Monarch convolution (blocks of 32 and 64) --------------------------------------
// y = g_out o Re( M2 ( Kf o M1 (g_in o u, 0) ) )[0:n] with complex block-diagonal factors (appendix: the blocky
// Monarch convolution): the mixer's four stages on two planes of the tile (real and imaginary parts), a complex
// product being four real MFMA chains, two when the input is real (first stage) or only the real part is kept (last
// stage, which also skips the row tiles of its outputs past n).  The factors are complex float32 [block][row][column]:
// a lane reads the (b/4) complex columns of its row as (b/2) consecutive floats.
template <int BS>
struct CGeo {   // rows of a tile: two planes of TV rows fit in LDS
    static constexpr int TV = BS == 32 ? 16 : 4;
    static constexpr size_t LDS_BYTES = 2 * sizeof(float) * TV * Geo<BS>::ROWP;
};

// RTMAX: row tiles of every block's outputs that are computed (the others keep their inputs).
template <int BS, int SK, bool REAL_IN, bool REAL_OUT, int RTMAX, typename At>
__device__ __forceinline__ void cstage(float *tre, float *tim, const float2 *__restrict__ W, int wave, int lane, At at)
{
    typedef Geo<BS> G;
    constexpr int TV = CGeo<BS>::TV;
    const int l16 = lane & 15, kg = lane >> 4;
    float *mre = tre + (l16 & (TV - 1)) * G::ROWP, *mim = tim + (l16 & (TV - 1)) * G::ROWP;
    // a lane's Q complex columns of a row come in halves of 8 (4 pieces of 16 bytes), the next half requested while the
    // current one is multiplied
    constexpr int HALVES = G::Q / 8, WV = 4;
    f32x4 w[2][WV];
    float anchor = 0.0f;
    constexpr int ITEMS = G::NBW * RTMAX * HALVES;
    auto request = [&](int item, f32x4 (&dst)[WV]) {
        const float2 *src = W;
        asm volatile("" : "+s"(src) : "v"(anchor));
        const int half = item % HALVES, rt = (item / HALVES) % RTMAX, blk = wave * G::NBW + item / (HALVES * RTMAX);
        const float *row = reinterpret_cast<const float *>(src + ((size_t)blk * BS + 16 * rt + l16) * BS + G::Q * kg + 8 * half);
#pragma unroll
        for (int p = 0; p < WV; ++p) dst[p] = ld4(row + 4 * p);
    };
    request(0, w[0]);
#pragma unroll
    for (int u = 0; u < G::NBW; ++u) {
        const int off = at(wave * G::NBW + u);
        float *ere = mre + off, *eim = mim + off;
        float bre[G::Q], bim[G::Q];
#pragma unroll
        for (int j = 0; j < G::Q; ++j) {
            bre[j] = ere[(G::Q * kg + j) * SK];
            if constexpr (!REAL_IN) bim[j] = eim[(G::Q * kg + j) * SK];
        }
        // (every input of the block is in registers by now: a row tile's results take their places at once)
#pragma unroll
        for (int rt = 0; rt < RTMAX; ++rt) {
            f32x4 ar = {0, 0, 0, 0}, ai = {0, 0, 0, 0}, sub = {0, 0, 0, 0};   // real part = ar - sub
#pragma unroll
            for (int half = 0; half < HALVES; ++half) {
                const int item = (u * RTMAX + rt) * HALVES + half;
                if (item + 1 < ITEMS) request(item + 1, w[(item + 1) & 1]);
                const f32x4 (&wc)[WV] = w[item & 1];
#pragma unroll
                for (int jj = 0; jj < 8; ++jj) {
                    const int j = 8 * half + jj;
                    const float wre = wc[jj >> 1][2 * (jj & 1)], wim = wc[jj >> 1][2 * (jj & 1) + 1];
                    ar = mfma(wre, bre[j], ar);
                    if constexpr (!REAL_IN) sub = mfma(wim, bim[j], sub);
                    if constexpr (!REAL_OUT) {
                        ai = mfma(wim, bre[j], ai);
                        if constexpr (!REAL_IN) ai = mfma(wre, bim[j], ai);
                    }
                }
            }
            ar -= sub;
            anchor = ar[0];
            if (l16 < TV) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    ere[(16 * rt + 4 * kg + r) * SK] = ar[r];
                    if constexpr (!REAL_OUT) eim[(16 * rt + 4 * kg + r) * SK] = ai[r];
                }
            }
        }
    }
}

template <typename T, int BS, bool GIN, bool GOUT>
__global__ __launch_bounds__(Geo<BS>::THREADS, 1) void blocky_kernel(
    const T *__restrict__ u, const T *__restrict__ g_in, const T *__restrict__ g_out, const float2 *__restrict__ R1,
    const float2 *__restrict__ L1, const float2 *__restrict__ R2, const float2 *__restrict__ L2, const float2 *__restrict__ Kf,
    T *__restrict__ y, int64_t rows, int H, int n)
{
    typedef Geo<BS> G;
    constexpr int TV = CGeo<BS>::TV;
    extern __shared__ __attribute__((aligned(16))) float tile[];
    float *tre = tile, *tim = tile + TV * G::ROWP;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int64_t ntiles = (rows + TV - 1) / TV;
    const int live_rt = ((n + BS - 1) / BS + 15) / 16;   // row tiles of the last stage that hold outputs below n
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int64_t v0 = t * TV;
        for (int piece = threadIdx.x; piece < TV * G::N / 4; piece += G::THREADS) {
            const int v = piece / (G::N / 4), i = 4 * (piece % (G::N / 4));
            int64_t r = v0 + v;
            if (r >= rows) r = rows - 1;   // (rows past the end: computed, never stored)
            f32x4 val = {0, 0, 0, 0};      // (n is a multiple of 4: a piece is inside the row or past it)
            if (i < n) {
                val = ld4(u + r * n + i);
                if (GIN) val *= ld4(g_in + r * n + i);
            }
            float *d = tre + v * G::ROWP + (i / BS) * G::SH + i % BS;
            d[0] = val[0]; d[1] = val[1]; d[2] = val[2]; d[3] = val[3];
        }
        __syncthreads();
        cstage<BS, G::SH, true, false, G::RT>(tre, tim, R1, wave, lane, [](int k) { return k; });
        __syncthreads();
        cstage<BS, 1, false, false, G::RT>(tre, tim, L1, wave, lane, [](int r) { return r * G::SH; });
        __syncthreads();
        // kernel product: entry m = s b + r of the transform domain sits at (r, s)
        for (int piece = threadIdx.x; piece < TV * G::N / 4; piece += G::THREADS) {
            const int v = piece / (G::N / 4), m = 4 * (piece % (G::N / 4));
            int64_t r = v0 + v;
            if (r >= rows) r = rows - 1;
            const float *kp = reinterpret_cast<const float *>(Kf + (r % H) * (int64_t)G::N + m);
            const f32x4 k01 = ld4(kp), k23 = ld4(kp + 4);
            const float kre[4] = {k01[0], k01[2], k23[0], k23[2]}, kim[4] = {k01[1], k01[3], k23[1], k23[3]};
            const int at = v * G::ROWP + (m % BS) * G::SH + m / BS;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float xr = tre[at + e * G::SH], xi = tim[at + e * G::SH];
                tre[at + e * G::SH] = xr * kre[e] - xi * kim[e];
                tim[at + e * G::SH] = xr * kim[e] + xi * kre[e];
            }
        }
        __syncthreads();
        cstage<BS, 1, false, false, G::RT>(tre, tim, R2, wave, lane, [](int k) { return k * G::SH; });
        __syncthreads();
        // (only the row tiles of the outputs below n)
        if (live_rt == 1) cstage<BS, G::SH, false, true, 1>(tre, tim, L2, wave, lane, [](int r) { return r; });
        else if (live_rt == 2 || G::RT == 2) cstage<BS, G::SH, false, true, 2>(tre, tim, L2, wave, lane, [](int r) { return r; });
        else if (live_rt == 3) cstage<BS, G::SH, false, true, (G::RT > 2 ? 3 : 2)>(tre, tim, L2, wave, lane, [](int r) { return r; });
        else cstage<BS, G::SH, false, true, G::RT>(tre, tim, L2, wave, lane, [](int r) { return r; });
        __syncthreads();
        for (int piece = threadIdx.x; piece < TV * G::N / 4; piece += G::THREADS) {
            const int v = piece / (G::N / 4), i = 4 * (piece % (G::N / 4));
            if (v0 + v < rows && i < n) {
                const float *sp = tre + v * G::ROWP + (i / BS) * G::SH + i % BS;
                f32x4 val = {sp[0], sp[1], sp[2], sp[3]};
                if (GOUT) val *= ld4(g_out + (v0 + v) * n + i);
                st4(y + (v0 + v) * n + i, val);
            }
        }
        __syncthreads();
    }
}

template <int BS>
static int grid_for(int64_t ntiles, int64_t *grid)
{
    int dev = 0, ncu = 0;
    MONARCH_HIP_CHECK(hipGetDevice(&dev));
    MONARCH_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
    *grid = (int64_t)ncu * (BS == 32 ? 2 : 1);
    if (*grid > ntiles) *grid = ntiles;
    return MONARCH_OK;
}

template <typename T, int BS>
static int launch_matmul(const void *x, const void *R, const void *L, void *y, int64_t batch, hipStream_t s)
{
    typedef Geo<BS> G;
    int64_t grid = 0;
    if (int rc = grid_for<BS>((batch + G::TV - 1) / G::TV, &grid)) return rc;
    auto kern = matmul_kernel<T, BS>;
    MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)G::LDS_BYTES));
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(G::THREADS), G::LDS_BYTES, s, (const T *)x, (const T *)R, (const T *)L, (T *)y, batch);
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

template <typename T, int BS, bool GIN, bool GOUT>
static int launch_mixer_g(const void *u, const void *K, const void *g_in, const void *g_out, const void *R1, const void *L1,
                          const void *R2, const void *L2, void *y, int64_t rows, int H, const MixOpt &opt, hipStream_t s)
{
    typedef Geo<BS> G;
    int64_t grid = 0;
    if (int rc = grid_for<BS>((rows + G::TV - 1) / G::TV, &grid)) return rc;
    auto kern = mixer_kernel<T, BS, GIN, GOUT>;
    MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)G::LDS_BYTES));
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(G::THREADS), G::LDS_BYTES, s, (const T *)u, (const T *)K, (const T *)g_in,
                       (const T *)g_out, (const T *)R1, (const T *)L1, (const T *)R2, (const T *)L2, (T *)y, rows, H, opt);
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

template <typename T, int BS>
static int launch_mixer_t(const void *u, const void *K, const void *g_in, const void *g_out, const void *R1, const void *L1,
                          const void *R2, const void *L2, void *y, int64_t rows, int H, const MixOpt &opt, hipStream_t s)
{
    if (g_in && g_out) return launch_mixer_g<T, BS, true, true>(u, K, g_in, g_out, R1, L1, R2, L2, y, rows, H, opt, s);
    if (g_in) return launch_mixer_g<T, BS, true, false>(u, K, g_in, g_out, R1, L1, R2, L2, y, rows, H, opt, s);
    if (g_out) return launch_mixer_g<T, BS, false, true>(u, K, g_in, g_out, R1, L1, R2, L2, y, rows, H, opt, s);
    return launch_mixer_g<T, BS, false, false>(u, K, g_in, g_out, R1, L1, R2, L2, y, rows, H, opt, s);
}


template <typename T, int BS>
static int launch_backward(const void *x, const void *R, const void *L, const void *dy, void *dx, float *dR, float *dL, int64_t batch,
                           hipStream_t s)
{
    typedef Geo<BS> G;
    const size_t lds = 2 * G::LDS_BYTES;
    int dev = 0, ncu = 0;
    MONARCH_HIP_CHECK(hipGetDevice(&dev));
    MONARCH_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
    const int64_t ntiles = (batch + G::TV - 1) / G::TV;
    const unsigned grid = (unsigned)(ntiles < ncu ? ntiles : ncu);   // one workgroup per compute unit
#define MONARCH_INPL_BWD(KERN, ...)                                                                                        \
    do {                                                                                                                   \
        auto kern = KERN;                                                                                                  \
        MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));  \
        hipLaunchKernelGGL(kern, dim3(grid), dim3(G::THREADS), lds, s, __VA_ARGS__);                                       \
        MONARCH_HIP_CHECK(hipGetLastError());                                                                              \
    } while (0)
    if (dx && dL) MONARCH_INPL_BWD((backward_dx_dl_kernel<T, BS, true, true>), (const T *)x, (const T *)R, (const T *)L, (const T *)dy, (T *)dx, dL, batch);
    else if (dx) MONARCH_INPL_BWD((backward_dx_dl_kernel<T, BS, true, false>), (const T *)x, (const T *)R, (const T *)L, (const T *)dy, (T *)dx, dL, batch);
    else if (dL) MONARCH_INPL_BWD((backward_dx_dl_kernel<T, BS, false, true>), (const T *)x, (const T *)R, (const T *)L, (const T *)dy, (T *)dx, dL, batch);
    if (dR) MONARCH_INPL_BWD((backward_dr_kernel<T, BS>), (const T *)x, (const T *)L, (const T *)dy, dR, batch);
#undef MONARCH_INPL_BWD
    return MONARCH_OK;
}


template <typename T>
static int launch_backward64(const void *x, const void *R, const void *L, const void *dy, void *dx, float *dR, float *dL, int64_t batch,
                             hipStream_t s)
{
    typedef Geo<64> G;
    int dev = 0, ncu = 0;
    MONARCH_HIP_CHECK(hipGetDevice(&dev));
    MONARCH_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
    if (dx) {
        const int64_t ntiles = (batch + G::TV - 1) / G::TV;
        const unsigned grid = (unsigned)(ntiles < ncu ? ntiles : ncu);
        auto kern = backward64_dx_kernel<T>;
        MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)G::LDS_BYTES));
        hipLaunchKernelGGL(kern, dim3(grid), dim3(1024), G::LDS_BYTES, s, (const T *)R, (const T *)L, (const T *)dy, (T *)dx, batch);
        MONARCH_HIP_CHECK(hipGetLastError());
    }
    const int64_t ntiles = (batch + TV64 - 1) / TV64;
    int64_t slices = ncu / 4 > 0 ? ncu / 4 : 1;   // four groups of blocks per slice of the rows: one workgroup per compute unit
    if (slices > ntiles) slices = ntiles;
    if (dL) {
        const size_t lds = sizeof(float) * TV64 * (G::ROWP + CP64);
        auto kern = backward64_factor_kernel<T, 0>;
        MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(kern, dim3((unsigned)(4 * slices)), dim3(1024), lds, s, (const T *)x, (const T *)R, (const T *)dy, dL, batch);
        MONARCH_HIP_CHECK(hipGetLastError());
    }
    if (dR) {
        const size_t lds = sizeof(float) * TV64 * (G::ROWP + CX64);
        auto kern = backward64_factor_kernel<T, 1>;
        MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        hipLaunchKernelGGL(kern, dim3((unsigned)(4 * slices)), dim3(1024), lds, s, (const T *)x, (const T *)L, (const T *)dy, dR, batch);
        MONARCH_HIP_CHECK(hipGetLastError());
    }
    return MONARCH_OK;
}


template <typename T, int BS>
static int launch_blocky_t(const void *u, const void *g_in, const void *g_out, const float2 *R1, const float2 *L1, const float2 *R2,
                           const float2 *L2, const float2 *Kf, void *y, int64_t rows, int H, int n, hipStream_t s)
{
    typedef Geo<BS> G;
    int dev = 0, ncu = 0;
    MONARCH_HIP_CHECK(hipGetDevice(&dev));
    MONARCH_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
    const int64_t ntiles = (rows + CGeo<BS>::TV - 1) / CGeo<BS>::TV;
    const unsigned grid = (unsigned)(ntiles < ncu ? ntiles : ncu);   // one workgroup per compute unit
#define MONARCH_INPL_BLOCKY(GI, GO)                                                                                        \
    do {                                                                                                                   \
        auto kern = blocky_kernel<T, BS, GI, GO>;                                                                          \
        MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)CGeo<BS>::LDS_BYTES)); \
        hipLaunchKernelGGL(kern, dim3(grid), dim3(G::THREADS), CGeo<BS>::LDS_BYTES, s, (const T *)u, (const T *)g_in, (const T *)g_out, \
                           R1, L1, R2, L2, Kf, (T *)y, rows, H, n);                                                        \
    } while (0)
    if (g_in && g_out) MONARCH_INPL_BLOCKY(true, true);
    else if (g_in) MONARCH_INPL_BLOCKY(true, false);
    else if (g_out) MONARCH_INPL_BLOCKY(false, true);
    else MONARCH_INPL_BLOCKY(false, false);
#undef MONARCH_INPL_BLOCKY
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

}  // namespace inpl

bool monarch_inplace_supported(int bs, monarch_dtype dt) { return (bs == 32 || bs == 64) && (dt == MONARCH_F32 || dt == MONARCH_BF16); }

int launch_matmul_inplace(const void *x, const void *R, const void *L, void *y, int64_t batch, int bs, monarch_dtype dt, hipStream_t s)
{
    if (batch == 0) return MONARCH_OK;
    if (bs == 32) return dt == MONARCH_F32 ? inpl::launch_matmul<float, 32>(x, R, L, y, batch, s) : inpl::launch_matmul<bf16_t, 32>(x, R, L, y, batch, s);
    return dt == MONARCH_F32 ? inpl::launch_matmul<float, 64>(x, R, L, y, batch, s) : inpl::launch_matmul<bf16_t, 64>(x, R, L, y, batch, s);
}

// transposed access needs whole tiles inside a batch entry
bool mixer_inplace_takes(int bs, int H, monarch_dtype dt, const MixOpt &opt)
{
    if (!monarch_inplace_supported(bs, dt) || opt.act > 1) return false;
    return !opt.transposed || H % (bs == 32 ? inpl::Geo<32>::TV : inpl::Geo<64>::TV) == 0;
}

int launch_mixer_inplace(const void *u, const void *K, const void *g_in, const void *g_out, const void *R1, const void *L1,
                         const void *R2, const void *L2, void *y, int64_t rows, int H, int bs, monarch_dtype dt, const MixOpt &opt,
                         hipStream_t s)
{
    if (rows == 0) return MONARCH_OK;
    if (bs == 32)
        return dt == MONARCH_F32 ? inpl::launch_mixer_t<float, 32>(u, K, g_in, g_out, R1, L1, R2, L2, y, rows, H, opt, s)
                                 : inpl::launch_mixer_t<bf16_t, 32>(u, K, g_in, g_out, R1, L1, R2, L2, y, rows, H, opt, s);
    return dt == MONARCH_F32 ? inpl::launch_mixer_t<float, 64>(u, K, g_in, g_out, R1, L1, R2, L2, y, rows, H, opt, s)
                             : inpl::launch_mixer_t<bf16_t, 64>(u, K, g_in, g_out, R1, L1, R2, L2, y, rows, H, opt, s);
}

bool monarch_inplace_backward_supported(int bs, monarch_dtype dt) { return (bs == 32 || bs == 64) && (dt == MONARCH_F32 || dt == MONARCH_BF16); }

// dR and dL must have been cleared; batch > 0.
int launch_matmul_backward_inplace(const void *x, const void *R, const void *L, const void *dy, void *dx, float *dR, float *dL,
                                   int64_t batch, int bs, monarch_dtype dt, hipStream_t s)
{
    if (bs == 64)
        return dt == MONARCH_F32 ? inpl::launch_backward64<float>(x, R, L, dy, dx, dR, dL, batch, s)
                                 : inpl::launch_backward64<bf16_t>(x, R, L, dy, dx, dR, dL, batch, s);
    return dt == MONARCH_F32 ? inpl::launch_backward<float, 32>(x, R, L, dy, dx, dR, dL, batch, s)
                             : inpl::launch_backward<bf16_t, 32>(x, R, L, dy, dx, dR, dL, batch, s);
}

// rows of a multiple of 4 elements (16-byte pieces of fp32 rows, 8-byte pieces of bf16 rows)
bool blocky_inplace_takes(int bs, int n, monarch_dtype dt) { return monarch_inplace_supported(bs, dt) && n >= 4 && n % 4 == 0; }

int launch_blocky_inplace(const void *u, const void *g_in, const void *g_out, const float2 *R1, const float2 *L1, const float2 *R2,
                          const float2 *L2, const float2 *Kf, void *y, int64_t rows, int H, int n, int bs, monarch_dtype dt, hipStream_t s)
{
    if (bs == 32)
        return dt == MONARCH_F32 ? inpl::launch_blocky_t<float, 32>(u, g_in, g_out, R1, L1, R2, L2, Kf, y, rows, H, n, s)
                                 : inpl::launch_blocky_t<bf16_t, 32>(u, g_in, g_out, R1, L1, R2, L2, Kf, y, rows, H, n, s);
    return dt == MONARCH_F32 ? inpl::launch_blocky_t<float, 64>(u, g_in, g_out, R1, L1, R2, L2, Kf, y, rows, H, n, s)
                             : inpl::launch_blocky_t<bf16_t, 64>(u, g_in, g_out, R1, L1, R2, L2, Kf, y, rows, H, n, s);
}

}  // namespace monarch
