// Square order-2 Monarch products with blocks of 32 x 32 or 64 x 64 (N = 1024 or 4096) on the fp32 matrix
// instruction (16x16x4), fp32 or bf16 tensors, fp32 arithmetic:
//   monarch_matmul   y = P L P R P x                                    (Sec. 3.1)
//   monarch_mixer    y = g_out o M2 (K o M1 (g_in o u))                  (Sec. 3.2 Eq. 2 in its gated form)
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
__device__ __forceinline__ void st4(float *p, f32x4 v) { *reinterpret_cast<f32x4 *>(p) = v; }
__device__ __forceinline__ void st4(bf16_t *p, f32x4 v)
{
    const bf16_t h[4] = {from_f32<bf16_t>(v[0]), from_f32<bf16_t>(v[1]), from_f32<bf16_t>(v[2]), from_f32<bf16_t>(v[3])};
    *reinterpret_cast<uint2 *>(p) = *reinterpret_cast<const uint2 *>(h);
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
template <typename T, int BS, int SK, typename At>
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
        const T *row = src + ((size_t)blk * BS + 16 * rt + l16) * BS + G::Q * kg;
#pragma unroll
        for (int p = 0; p < WV; ++p) dst[p] = ld4(row + 4 * p);
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
            const f32x4 val = ld4(x + r * G::N + i);
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
            if (v0 + v < batch) st4(y + (v0 + v) * G::N + m, f32x4{sp[0], sp[G::SH], sp[2 * G::SH], sp[3 * G::SH]});
        }
        __syncthreads();
    }
}

template <typename T, int BS, bool GIN, bool GOUT>
__global__ __launch_bounds__(Geo<BS>::THREADS, BS == 32 ? 2 : 1) void mixer_kernel(
    const T *__restrict__ u, const T *__restrict__ K, const T *__restrict__ g_in, const T *__restrict__ g_out,
    const T *__restrict__ R1, const T *__restrict__ L1, const T *__restrict__ R2, const T *__restrict__ L2, T *__restrict__ y,
    int64_t rows, int H)
{
    typedef Geo<BS> G;
    extern __shared__ __attribute__((aligned(16))) float tile[];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int64_t ntiles = (rows + G::TV - 1) / G::TV;
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int64_t v0 = t * G::TV;
        for (int piece = threadIdx.x; piece < G::TV * G::N / 4; piece += G::THREADS) {
            const int v = piece / (G::N / 4), i = 4 * (piece % (G::N / 4));
            int64_t r = v0 + v;
            if (r >= rows) r = rows - 1;
            f32x4 val = ld4(u + r * G::N + i);
            if (GIN) val *= ld4(g_in + r * G::N + i);
            float *d = tile + v * G::ROWP + (i / BS) * G::SH + i % BS;
            d[0] = val[0]; d[1] = val[1]; d[2] = val[2]; d[3] = val[3];
        }
        __syncthreads();
        stage<T, BS, G::SH>(tile, R1, wave, lane, [](int k) { return k; });
        __syncthreads();
        stage<T, BS, 1>(tile, L1, wave, lane, [](int r) { return r * G::SH; });
        __syncthreads();
        // kernel product: entry m = s b + r of the transform domain sits at (r, s)
        for (int piece = threadIdx.x; piece < G::TV * G::N / 4; piece += G::THREADS) {
            const int v = piece / (G::N / 4), m = 4 * (piece % (G::N / 4));
            int64_t r = v0 + v;
            if (r >= rows) r = rows - 1;
            const f32x4 kv = ld4(K + (r % H) * G::N + m);
            float *sp = tile + v * G::ROWP + (m % BS) * G::SH + m / BS;
            sp[0] *= kv[0]; sp[G::SH] *= kv[1]; sp[2 * G::SH] *= kv[2]; sp[3 * G::SH] *= kv[3];
        }
        __syncthreads();
        stage<T, BS, 1>(tile, R2, wave, lane, [](int k) { return k * G::SH; });
        __syncthreads();
        stage<T, BS, G::SH>(tile, L2, wave, lane, [](int r) { return r; });
        __syncthreads();
        for (int piece = threadIdx.x; piece < G::TV * G::N / 4; piece += G::THREADS) {
            const int v = piece / (G::N / 4), i = 4 * (piece % (G::N / 4));
            if (v0 + v < rows) {
                const float *sp = tile + v * G::ROWP + (i / BS) * G::SH + i % BS;
                f32x4 val = {sp[0], sp[1], sp[2], sp[3]};
                if (GOUT) val *= ld4(g_out + (v0 + v) * G::N + i);
                st4(y + (v0 + v) * G::N + i, val);
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
                          const void *R2, const void *L2, void *y, int64_t rows, int H, hipStream_t s)
{
    typedef Geo<BS> G;
    int64_t grid = 0;
    if (int rc = grid_for<BS>((rows + G::TV - 1) / G::TV, &grid)) return rc;
    auto kern = mixer_kernel<T, BS, GIN, GOUT>;
    MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)G::LDS_BYTES));
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(G::THREADS), G::LDS_BYTES, s, (const T *)u, (const T *)K, (const T *)g_in,
                       (const T *)g_out, (const T *)R1, (const T *)L1, (const T *)R2, (const T *)L2, (T *)y, rows, H);
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

template <typename T, int BS>
static int launch_mixer_t(const void *u, const void *K, const void *g_in, const void *g_out, const void *R1, const void *L1,
                          const void *R2, const void *L2, void *y, int64_t rows, int H, hipStream_t s)
{
    if (g_in && g_out) return launch_mixer_g<T, BS, true, true>(u, K, g_in, g_out, R1, L1, R2, L2, y, rows, H, s);
    if (g_in) return launch_mixer_g<T, BS, true, false>(u, K, g_in, g_out, R1, L1, R2, L2, y, rows, H, s);
    if (g_out) return launch_mixer_g<T, BS, false, true>(u, K, g_in, g_out, R1, L1, R2, L2, y, rows, H, s);
    return launch_mixer_g<T, BS, false, false>(u, K, g_in, g_out, R1, L1, R2, L2, y, rows, H, s);
}

}  // namespace inpl

bool monarch_inplace_supported(int bs, monarch_dtype dt) { return (bs == 32 || bs == 64) && (dt == MONARCH_F32 || dt == MONARCH_BF16); }

int launch_matmul_inplace(const void *x, const void *R, const void *L, void *y, int64_t batch, int bs, monarch_dtype dt, hipStream_t s)
{
    if (batch == 0) return MONARCH_OK;
    if (bs == 32) return dt == MONARCH_F32 ? inpl::launch_matmul<float, 32>(x, R, L, y, batch, s) : inpl::launch_matmul<bf16_t, 32>(x, R, L, y, batch, s);
    return dt == MONARCH_F32 ? inpl::launch_matmul<float, 64>(x, R, L, y, batch, s) : inpl::launch_matmul<bf16_t, 64>(x, R, L, y, batch, s);
}

int launch_mixer_inplace(const void *u, const void *K, const void *g_in, const void *g_out, const void *R1, const void *L1,
                         const void *R2, const void *L2, void *y, int64_t rows, int H, int bs, monarch_dtype dt, hipStream_t s)
{
    if (rows == 0) return MONARCH_OK;
    if (bs == 32)
        return dt == MONARCH_F32 ? inpl::launch_mixer_t<float, 32>(u, K, g_in, g_out, R1, L1, R2, L2, y, rows, H, s)
                                 : inpl::launch_mixer_t<bf16_t, 32>(u, K, g_in, g_out, R1, L1, R2, L2, y, rows, H, s);
    return dt == MONARCH_F32 ? inpl::launch_mixer_t<float, 64>(u, K, g_in, g_out, R1, L1, R2, L2, y, rows, H, s)
                             : inpl::launch_mixer_t<bf16_t, 64>(u, K, g_in, g_out, R1, L1, R2, L2, y, rows, H, s);
}

}  // namespace monarch
