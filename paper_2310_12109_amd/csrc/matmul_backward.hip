// Gradients of the order-2 Monarch product y = P3 L P2 R P1 x (Sec. 3.1) with respect to x, R and L, given
// dy, by the chain rule through the five steps of the product:
//   forward   t0 = P1 x,  t1 = R t0,  t2 = P2 t1,  (t3 = L t2,  y = P3 t3)
//   backward  g3 = P3^T dy,  dL_k += g3_k t2_k^T,  g2 = L^T g3,  g1 = P2^T g2,  dR_k += g1_k t0_k^T,
//             dx = P1^T R^T g1
// fp32 arithmetic on tiles of vectors held in LDS; the permutations are LDS index maps (t0 and g3 are
// written permuted, t2 and g1 are produced permuted).  Workgroups are persistent and walk over the tiles;
// the parameter gradients, sums over the whole batch, are accumulated per workgroup (in registers when a
// thread's share of the entries is at most EPT, else added to memory after every tile) and leave with one
// floating-point atomic add per entry.  The caller's dR / dL are cleared by a fill kernel first.
#include "kernels.h"
#include "lds_dma.h"

namespace monarch {

namespace mmb {

constexpr int THREADS = 256, EPT = 32;

__global__ void fill_zero_kernel(float *a, size_t na, float *b, size_t nb)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < na + nb; i += stride) {
        if (i < na) a[i] = 0.0f;
        else b[i - na] = 0.0f;
    }
}

struct Dims {
    int nbR, r_out, r_in, nbL, l_out, l_in;
};

// KEEP: this thread's entries of dR / dL stay in registers over all tiles of the workgroup.
template <typename T, int TV, bool KEEP>
__global__ __launch_bounds__(THREADS) void matmul_backward_kernel(
    const T *__restrict__ x, const T *__restrict__ R, const T *__restrict__ L, const T *__restrict__ dy,
    T *__restrict__ dx, float *__restrict__ dR, float *__restrict__ dL, int64_t batch, const Dims d)
{
    extern __shared__ float lds[];
    const int nbR = d.nbR, r_out = d.r_out, r_in = d.r_in, nbL = d.nbL, l_out = d.l_out, l_in = d.l_in;
    const int d_in = nbR * r_in, d_mid = nbR * r_out, d_out = nbL * l_out;
    float *t0 = lds;                  // [TV][d_in]   t0[k r_in + c]  = x[c nbR + k]
    float *g3 = t0 + TV * d_in;       // [TV][d_out]  g3[k l_out + r] = dy[r nbL + k]
    float *t2 = g3 + TV * d_out;      // [TV][d_mid]  input of L: t2[r nbR + k] = (R t0)[k r_out + r]
    float *g1 = t2 + TV * d_mid;      // [TV][d_mid]  gradient of R's output: g1[k r_out + r] = (L^T g3)[r nbR + k]
    const int tid = threadIdx.x;
    const int nR = nbR * r_out * r_in, nL = nbL * l_out * l_in;
    const int nRw = dR ? nR : 0, nLw = dL ? nL : 0;   // entries wanted
    const int64_t ntiles = (batch + TV - 1) / TV;

    float keep[KEEP ? EPT : 1];
#pragma unroll
    for (int i = 0; i < (KEEP ? EPT : 1); ++i) keep[i] = 0.0f;

    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t v0 = tile * TV;
        for (int idx = tid; idx < TV * d_in; idx += THREADS) {
            const int v = idx / d_in, j = idx - v * d_in;   // j = c nbR + k
            const int c = j / nbR, k = j - c * nbR;
            t0[v * d_in + k * r_in + c] = v0 + v < batch ? to_f32(x[(v0 + v) * d_in + j]) : 0.0f;
        }
        for (int idx = tid; idx < TV * d_out; idx += THREADS) {
            const int v = idx / d_out, i = idx - v * d_out;   // i = r nbL + k
            const int r = i / nbL, k = i - r * nbL;
            g3[v * d_out + k * l_out + r] = v0 + v < batch ? to_f32(dy[(v0 + v) * d_out + i]) : 0.0f;
        }
        __syncthreads();
        for (int o = tid; o < d_mid; o += THREADS) {   // o = k r_out + r
            const int k = o / r_out, r = o - k * r_out;
            float acc[TV];
#pragma unroll
            for (int v = 0; v < TV; ++v) acc[v] = 0.0f;
            const T *w = R + (size_t)o * r_in;
            for (int c = 0; c < r_in; ++c) {
                const float wv = to_f32(w[c]);
#pragma unroll
                for (int v = 0; v < TV; ++v) acc[v] = fmaf(wv, t0[v * d_in + k * r_in + c], acc[v]);
            }
#pragma unroll
            for (int v = 0; v < TV; ++v) t2[v * d_mid + r * nbR + k] = acc[v];
        }
        for (int o = tid; o < d_mid; o += THREADS) {   // o = k' l_in + a = r nbR + k
            const int kk = o / l_in, a = o - kk * l_in;
            float acc[TV];
#pragma unroll
            for (int v = 0; v < TV; ++v) acc[v] = 0.0f;
            const T *w = L + (size_t)kk * l_out * l_in + a;
            for (int r = 0; r < l_out; ++r) {
                const float wv = to_f32(w[(size_t)r * l_in]);
#pragma unroll
                for (int v = 0; v < TV; ++v) acc[v] = fmaf(wv, g3[v * d_out + kk * l_out + r], acc[v]);
            }
            const int r = o / nbR, k = o - r * nbR;
#pragma unroll
            for (int v = 0; v < TV; ++v) g1[v * d_mid + k * r_out + r] = acc[v];
        }
        __syncthreads();
        if (dx) {
            for (int o = tid; o < d_in; o += THREADS) {   // o = k r_in + c
                const int k = o / r_in, c = o - k * r_in;
                float acc[TV];
#pragma unroll
                for (int v = 0; v < TV; ++v) acc[v] = 0.0f;
                const T *w = R + (size_t)k * r_out * r_in + c;
                for (int r = 0; r < r_out; ++r) {
                    const float wv = to_f32(w[(size_t)r * r_in]);
#pragma unroll
                    for (int v = 0; v < TV; ++v) acc[v] = fmaf(wv, g1[v * d_mid + k * r_out + r], acc[v]);
                }
#pragma unroll
                for (int v = 0; v < TV; ++v)
                    if (v0 + v < batch) dx[(v0 + v) * d_in + c * nbR + k] = from_f32<T>(acc[v]);
            }
        }
        // entry e < nRw: dR[k][r][c] (e = (k r_out + r) r_in + c); then dL[k][r][a]
        int slot = 0;
        for (int e = tid; e < nRw + nLw; e += THREADS, ++slot) {
            float s = 0.0f;
            if (e < nRw) {
                const int o = e / r_in, c = e - o * r_in, k = o / r_out;
#pragma unroll
                for (int v = 0; v < TV; ++v) s = fmaf(g1[v * d_mid + o], t0[v * d_in + k * r_in + c], s);
            } else {
                const int el = e - nRw, o = el / l_in, a = el - o * l_in, k = o / l_out;
#pragma unroll
                for (int v = 0; v < TV; ++v) s = fmaf(g3[v * d_out + o], t2[v * d_mid + k * l_in + a], s);
            }
            if (KEEP) {
#pragma unroll
                for (int i = 0; i < EPT; ++i)   // (constant register index: no scratch memory)
                    if (i == slot) keep[i] += s;
            } else {
                atomicAdd(e < nRw ? dR + e : dL + (e - nRw), s);
            }
        }
        __syncthreads();
    }
    if (KEEP) {
#pragma unroll
        for (int i = 0; i < EPT; ++i) {
            const int e = tid + i * THREADS;
            if (e < nRw + nLw) atomicAdd(e < nRw ? dR + e : dL + (e - nRw), keep[i]);
        }
    }
}

static size_t lds_bytes(const Dims &d, int tv)
{
    return (size_t)tv * ((size_t)d.nbR * d.r_in + (size_t)d.nbL * d.l_out + 2 * (size_t)d.nbR * d.r_out) * sizeof(float);
}

template <typename T>
static int launch_typed(const void *x, const void *R, const void *L, const void *dy, void *dx, float *dR, float *dL,
                        int64_t batch, const Dims &d, hipStream_t s)
{
    int tv = 8;
    while (tv > 1 && lds_bytes(d, tv) > 64 * 1024) tv >>= 1;
    const size_t lds = lds_bytes(d, tv);
    if (lds > 160 * 1024) return fail(MONARCH_ESHAPE, "a row of the backward pass does not fit in LDS");
    int dev = 0, ncu = 0;
    MONARCH_HIP_CHECK(hipGetDevice(&dev));
    MONARCH_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
    const int64_t ntiles = (batch + tv - 1) / tv;
    int64_t grid = (int64_t)ncu * (lds <= 40 * 1024 ? 4 : lds <= 80 * 1024 ? 2 : 1);
    if (grid > ntiles) grid = ntiles;
    const size_t nR = dR ? (size_t)d.nbR * d.r_out * d.r_in : 0, nL = dL ? (size_t)d.nbL * d.l_out * d.l_in : 0;
    if (nR + nL) {
        hipLaunchKernelGGL(fill_zero_kernel, dim3(64), dim3(256), 0, s, dR, nR, dL, nL);
        MONARCH_HIP_CHECK(hipGetLastError());
    }
    if (ntiles == 0) return MONARCH_OK;   // empty batch: the parameter gradients are the zeros just written
    const bool keep = nR + nL <= (size_t)EPT * THREADS;
#define MONARCH_LAUNCH_MMB(TVV, KEEPV)                                                                              \
    do {                                                                                                            \
        auto kern = matmul_backward_kernel<T, TVV, KEEPV>;                                                          \
        if (lds > 64 * 1024)                                                                                        \
            MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,   \
                                                  (int)lds));                                                       \
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(THREADS), lds, s, (const T *)x, (const T *)R,           \
                           (const T *)L, (const T *)dy, (T *)dx, dR, dL, batch, d);                                 \
    } while (0)
#define MONARCH_LAUNCH_MMB_TV(KEEPV)                     \
    do {                                                 \
        switch (tv) {                                    \
        case 8: MONARCH_LAUNCH_MMB(8, KEEPV); break;     \
        case 4: MONARCH_LAUNCH_MMB(4, KEEPV); break;     \
        case 2: MONARCH_LAUNCH_MMB(2, KEEPV); break;     \
        default: MONARCH_LAUNCH_MMB(1, KEEPV); break;    \
        }                                                \
    } while (0)
    if (keep) MONARCH_LAUNCH_MMB_TV(true);
    else MONARCH_LAUNCH_MMB_TV(false);
#undef MONARCH_LAUNCH_MMB_TV
#undef MONARCH_LAUNCH_MMB
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

}  // namespace mmb

// ---- square case b = 16 (N = 256), fp32, on the matrix cores -------------------------------------------
// With x[v][16 c + a] and dy[v][16 k + i] (Sec. 3.1; blocks R_a, L_i of 16 x 16):
//   T_a[i, v]  = sum_c R_a[i, c] x[v][16 c + a]          first factor, recomputed
//   G_i[a, v]  = sum_k L_i[k, a] dy[v][16 k + i]         gradient of T_a[i, v]
//   dL_i[k, a] = sum_v dy[v][16 k + i] T_a[i, v]
//   dR_a[i, c] = sum_v G_i[a, v] x[v][16 c + a]
//   dx[v][16 c + a] = sum_i R_a[i, c] G_i[a, v]
// all of them 16x16x4 fp32 MFMAs.  A workgroup (4 waves) takes one tile of 16 vectors at a time; wave w owns the
// blocks 4 w .. 4 w + 3 of every product, so its share of the weights (and of dR, dL, accumulated over all the
// workgroup's tiles) stays in registers.  The rows of x and dy come in by direct-to-LDS loads (one vector,
// 1 KB, per wave instruction); T and G cross between the waves through two LDS tiles whose index maps are the
// middle permutation; dx leaves through LDS as whole rows.  Products over the vectors of a tile need their
// operands transposed (a lane per feature, vectors on the contraction index): those are the reads of the x /
// dy rows at [vector][feature] and of the T / G tiles along their other index.
namespace mmb16 {

typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int B = 16, N = 256, TV = 16;
constexpr int LDX = N + 4;                 // row pitch of the x / dy tiles: 16-byte aligned, one 16-byte slot off
constexpr int RS = 18, LD = B * RS + 3;    // T / G tiles: element (v, p, q) at v LD + p RS + q
constexpr size_t LDS_BYTES = sizeof(float) * (2 * TV * LDX + 2 * TV * LD);

__device__ __forceinline__ f32x4 mfma(float a, float b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    const bf16_t a = from_f32<bf16_t>(lo), b = from_f32<bf16_t>(hi);
    return (uint32_t) * reinterpret_cast<const uint16_t *>(&a) | ((uint32_t) * reinterpret_cast<const uint16_t *>(&b) << 16);
}

// T: type of x, R, L, dy and dx in memory (dR, dL are always float).  float rows arrive by direct-to-LDS loads;
// bf16 rows (512 bytes, two per wave instruction) pass through registers and are widened into LDS.
template <typename T>
__global__ __launch_bounds__(256, 2) void matmul_backward_b16_kernel(
    const T *__restrict__ x, const T *__restrict__ R, const T *__restrict__ L,
    const T *__restrict__ dy, T *__restrict__ dx, float *__restrict__ dR, float *__restrict__ dL,
    int64_t batch)
{
    constexpr bool F32 = sizeof(T) == 4;
    extern __shared__ __attribute__((aligned(16))) float smem[];
    float *xs = smem;                      // [TV][LDX]
    float *gs = xs + TV * LDX;             // [TV][LDX]  dy rows, later the dx rows
    float *tt = gs + TV * LDX;             // T: (v, i, a)
    float *gt = tt + TV * LD;              // G: (v, a, i)
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63, l16 = lane & 15, kg = lane >> 4;
    const int b0 = 4 * wave;   // this wave's blocks

    // k-step s of an MFMA contracts the index 4 kg + s
    float Rw[4][4], Rt[4][4], Lt[4][4];   // [block - b0][s]: R_a[l16][4kg+s], R_a[4kg+s][l16], L_i[4kg+s][l16]
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            Rw[q][s] = to_f32(R[((b0 + q) * B + l16) * B + 4 * kg + s]);
            Rt[q][s] = to_f32(R[((b0 + q) * B + 4 * kg + s) * B + l16]);
            Lt[q][s] = to_f32(L[((b0 + q) * B + 4 * kg + s) * B + l16]);
        }
    f32x4 accL[4], accR[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) accL[q] = accR[q] = f32x4{0, 0, 0, 0};

    const int64_t ntiles = (batch + TV - 1) / TV;
    const uint32_t xs_addr = lds_address(xs), gs_addr = lds_address(gs);
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t v0 = tile * TV;
        // rows in: wave w fetches vectors 4 w .. 4 w + 3 of x and of dy (rows past the batch: the last one)
        if constexpr (F32) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                int64_t v = v0 + b0 + q;
                if (v >= batch) v = batch - 1;
                dma_16_at(x + v * N + 4 * lane, xs_addr + (uint32_t)(b0 + q) * LDX * 4);
                dma_16_at(dy + v * N + 4 * lane, gs_addr + (uint32_t)(b0 + q) * LDX * 4);
            }
            wait_loads_at_most<0>();
        } else {
            uint4 w[4];   // lanes 0..31: vector 2 i, lanes 32..63: vector 2 i + 1; 8 elements per lane
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                int64_t v = v0 + b0 + 2 * i + (lane >> 5);
                if (v >= batch) v = batch - 1;
                w[i] = *reinterpret_cast<const uint4 *>(x + v * N + 8 * (lane & 31));
                w[2 + i] = *reinterpret_cast<const uint4 *>(dy + v * N + 8 * (lane & 31));
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float *d = (i < 2 ? xs : gs) + (b0 + 2 * (i & 1) + (lane >> 5)) * LDX + 8 * (lane & 31);
                *reinterpret_cast<f32x4 *>(d) = f32x4{__uint_as_float(w[i].x << 16), __uint_as_float(w[i].x & 0xffff0000u),
                                                      __uint_as_float(w[i].y << 16), __uint_as_float(w[i].y & 0xffff0000u)};
                *reinterpret_cast<f32x4 *>(d + 4) = f32x4{__uint_as_float(w[i].z << 16), __uint_as_float(w[i].z & 0xffff0000u),
                                                          __uint_as_float(w[i].w << 16), __uint_as_float(w[i].w & 0xffff0000u)};
            }
        }
        if (v0 + TV > batch) {   // ragged tile: the missing vectors must not reach dR, dL
            __syncthreads();
            for (int idx = threadIdx.x; idx < TV * N; idx += 256) {
                const int v = idx / N;
                if (v0 + v >= batch) gs[v * LDX + (idx - v * N)] = 0.0f;
            }
        }
        __syncthreads();

        // T_a (blocks a of this wave) and G_i (blocks i of this wave); the lane is vector v = l16
        {
            f32x4 xq[4], gq[4];   // [s]: features 16 (4 kg + s) + b0 .. + 3
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                xq[s] = *reinterpret_cast<const f32x4 *>(xs + l16 * LDX + 16 * (4 * kg + s) + b0);
                gq[s] = *reinterpret_cast<const f32x4 *>(gs + l16 * LDX + 16 * (4 * kg + s) + b0);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                f32x4 t = {0, 0, 0, 0}, g = {0, 0, 0, 0};
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    t = mfma(Rw[q][s], xq[s][q], t);   // rows i = 4 kg + r
                    g = mfma(Lt[q][s], gq[s][q], g);   // rows a = 4 kg + r
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    tt[l16 * LD + (4 * kg + r) * RS + b0 + q] = t[r];   // (v, i, a = b0 + q)
                    gt[l16 * LD + (4 * kg + r) * RS + b0 + q] = g[r];   // (v, a, i = b0 + q)
                }
            }
        }
        __syncthreads();

        // dL_i += dy_i T_i^T and dR_a += G_a x_a^T over the 16 vectors: k-step s contracts v = 4 kg + s
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int v = 4 * kg + s;
            const f32x4 ga = *reinterpret_cast<const f32x4 *>(gs + v * LDX + 16 * l16 + b0);   // dy[v][16 k + i], k = l16
            const f32x4 xb = *reinterpret_cast<const f32x4 *>(xs + v * LDX + 16 * l16 + b0);   // x[v][16 c + a], c = l16
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                accL[q] = mfma(ga[q], tt[v * LD + (b0 + q) * RS + l16], accL[q]);   // B: T_a[i][v], a = l16
                accR[q] = mfma(gt[v * LD + (b0 + q) * RS + l16], xb[q], accR[q]);   // A: G_i[a][v], i = l16
            }
        }
        // dx_a[c, v] = sum_i R_a[i, c] G_i[a, v]: rows c = 4 kg + r, column v = l16
        f32x4 dxa[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            f32x4 acc = {0, 0, 0, 0};
#pragma unroll
            for (int s = 0; s < 4; ++s) acc = mfma(Rt[q][s], gt[l16 * LD + (b0 + q) * RS + 4 * kg + s], acc);
            dxa[q] = acc;
        }
        __syncthreads();   // every wave is done with the dy rows: they become the dx rows
        if (dx) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
                *reinterpret_cast<f32x4 *>(gs + l16 * LDX + 16 * (4 * kg + r) + b0) = f32x4{dxa[0][r], dxa[1][r], dxa[2][r], dxa[3][r]};
            __syncthreads();
            if constexpr (F32) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int64_t v = v0 + b0 + q;
                    if (v < batch)   // (dx is written once per launch: streaming stores)
                        __builtin_nontemporal_store(*reinterpret_cast<const f32x4 *>(gs + (b0 + q) * LDX + 4 * lane), reinterpret_cast<f32x4 *>(dx + v * N + 4 * lane));
                }
            } else {
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int vv = b0 + 2 * i + (lane >> 5);
                    const f32x4 lo = *reinterpret_cast<const f32x4 *>(gs + vv * LDX + 8 * (lane & 31));
                    const f32x4 hi = *reinterpret_cast<const f32x4 *>(gs + vv * LDX + 8 * (lane & 31) + 4);
                    if (v0 + vv < batch)
                        store_stream16(dx + (v0 + vv) * N + 8 * (lane & 31),
                                       uint4{pack_bf16(lo[0], lo[1]), pack_bf16(lo[2], lo[3]), pack_bf16(hi[0], hi[1]), pack_bf16(hi[2], hi[3])});
                }
            }
            __syncthreads();   // before the next tile's rows land
        }
    }
    // accL[q][r] = dL_i[k = 4 kg + r][a = l16], accR[q][r] = dR_a[i = 4 kg + r][c = l16]
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if (dL) atomicAdd(dL + ((b0 + q) * B + 4 * kg + r) * B + l16, accL[q][r]);
            if (dR) atomicAdd(dR + ((b0 + q) * B + 4 * kg + r) * B + l16, accR[q][r]);
        }
}

}  // namespace mmb16

bool matmul_backward_b16_supported(int nbR, int r_out, int r_in, int nbL, int l_out, int l_in, monarch_dtype dt)
{
    return (dt == MONARCH_F32 || dt == MONARCH_BF16) && nbR == 16 && r_out == 16 && r_in == 16 && nbL == 16 && l_out == 16 &&
           l_in == 16;
}

static int launch_matmul_backward_b16(const void *x, const void *R, const void *L, const void *dy, void *dx, float *dR,
                                      float *dL, int64_t batch, monarch_dtype dt, hipStream_t s)
{
    if (dR || dL) {
        hipLaunchKernelGGL(mmb::fill_zero_kernel, dim3(16), dim3(256), 0, s, dR, dR ? (size_t)4096 : 0, dL, dL ? (size_t)4096 : 0);
        MONARCH_HIP_CHECK(hipGetLastError());
    }
    const int64_t ntiles = (batch + mmb16::TV - 1) / mmb16::TV;
    if (ntiles == 0) return MONARCH_OK;
    int dev = 0, ncu = 0;
    MONARCH_HIP_CHECK(hipGetDevice(&dev));
    MONARCH_HIP_CHECK(hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev));
    int64_t grid = 2 * (int64_t)ncu;   // two workgroups (69 KB of LDS each) per compute unit
    if (grid > ntiles) grid = ntiles;
    if (dt == MONARCH_F32) {
        MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)mmb16::matmul_backward_b16_kernel<float>,
                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)mmb16::LDS_BYTES));
        hipLaunchKernelGGL(mmb16::matmul_backward_b16_kernel<float>, dim3((unsigned)grid), dim3(256), mmb16::LDS_BYTES, s,
                           (const float *)x, (const float *)R, (const float *)L, (const float *)dy, (float *)dx, dR, dL, batch);
    } else {
        MONARCH_HIP_CHECK(hipFuncSetAttribute((const void *)mmb16::matmul_backward_b16_kernel<bf16_t>,
                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)mmb16::LDS_BYTES));
        hipLaunchKernelGGL(mmb16::matmul_backward_b16_kernel<bf16_t>, dim3((unsigned)grid), dim3(256), mmb16::LDS_BYTES, s,
                           (const bf16_t *)x, (const bf16_t *)R, (const bf16_t *)L, (const bf16_t *)dy, (bf16_t *)dx, dR, dL,
                           batch);
    }
    MONARCH_HIP_CHECK(hipGetLastError());
    return MONARCH_OK;
}

bool matmul_backward_fits(int nbR, int r_out, int r_in, int nbL, int l_out, int l_in)
{
    const mmb::Dims d = {nbR, r_out, r_in, nbL, l_out, l_in};
    return mmb::lds_bytes(d, 1) <= 160 * 1024;
}

int launch_matmul_backward(const void *x, const void *R, const void *L, const void *dy, void *dx, float *dR,
                           float *dL, int64_t batch, int nbR, int r_out, int r_in, int nbL, int l_out, int l_in,
                           monarch_dtype dt, hipStream_t s)
{
    if (matmul_backward_b16_supported(nbR, r_out, r_in, nbL, l_out, l_in, dt))
        return launch_matmul_backward_b16(x, R, L, dy, dx, dR, dL, batch, dt, s);
    const int bs = nbR;
    if ((bs == 32 || bs == 64) && r_out == bs && r_in == bs && nbL == bs && l_out == bs && l_in == bs && monarch_inplace_backward_supported(bs, dt)) {
        // square blocks of 32 or 64: both factors and their gradients on the fp32 matrix instruction, in place on LDS tiles
        const size_t nw = (size_t)bs * bs * bs;
        if (dR || dL) {
            hipLaunchKernelGGL(mmb::fill_zero_kernel, dim3(256), dim3(256), 0, s, dR, dR ? nw : 0, dL, dL ? nw : 0);
            MONARCH_HIP_CHECK(hipGetLastError());
        }
        if (batch == 0) return MONARCH_OK;
        return launch_matmul_backward_inplace(x, R, L, dy, dx, dR, dL, batch, bs, dt, s);
    }
    const mmb::Dims d = {nbR, r_out, r_in, nbL, l_out, l_in};
    if (dt == MONARCH_F32) return mmb::launch_typed<float>(x, R, L, dy, dx, dR, dL, batch, d, s);
    return mmb::launch_typed<bf16_t>(x, R, L, dy, dx, dR, dL, batch, d, s);
}

}  // namespace monarch
