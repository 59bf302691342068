// Host-side launchers of the HIP kernels; argument checks are done by the callers in api.hip.
#pragma once

#include "common.h"

namespace monarch {

// ---- generic fp32-arithmetic kernels (any shape) -------------------------------------------

// y = act(P3 L P2 R P1 x + bias) (order 2) or y = act(diag(R) x + bias) (order 1: L ignored).
// x: (batch, d_in) of type dt_in, y: (batch, d_out) of type dt_out, weights/bias of type dt_w.
int launch_matmul_generic(const void *x, const void *R, const void *L, const void *bias, void *y,
                          int64_t batch, int nbR, int r_out, int r_in, int nbL, int l_out, int l_in,
                          int order, int act, monarch_dtype dt_in, monarch_dtype dt_w,
                          monarch_dtype dt_out, hipStream_t s);
// Largest d_in/d_out + d_mid the generic kernel can hold on chip.
bool matmul_generic_fits(int d_in, int d_mid, int d_out);

// C32: complex fp32 (re, im); C16: complex as a packed bf16 pair (MFMA passes only); REAL / CPLX: the
// caller's element type.  *_PAIR: two real rows travel as one complex row (MFMA only).
// LD_C16_HERM_MULK: rows and kernels were both paired across channels (z = a + i b, kz = ka + i kb, natural
// order, packed bf16, kz in `kf`): the Hermitian halves are separated on load, A Ka + i B Kb is formed and conjugated.
enum FftLoad { LD_C32 = 0, LD_C32_CONJ = 1, LD_C32_CONJ_MULK = 2, LD_REAL = 3, LD_CPLX = 4,
               LD_C16 = 5, LD_C16_CONJ_MULK = 6, LD_REAL_PAIR = 7, LD_C16_HERM_MULK = 8 };
enum FftStore { ST_C32 = 0, ST_C32_NATURAL = 1, ST_CPLX_CONJ_SCALE = 2, ST_REAL_SCALE_GATE = 3,
                ST_C16 = 4, ST_C16_NATURAL = 5, ST_REAL_PAIR = 6 };

struct FftPass {
    const void *in;      // see FftLoad
    void *out;           // see FftStore
    const void *gate;    // LD_REAL: optional per-element gate (same layout as in); ST_REAL_SCALE_GATE: optional output gate
    const float2 *kf;    // LD_C32_CONJ_MULK: spectrum (H, N)
    int64_t rows;
    int N;               // transform length
    int O, f, S;         // the row is viewed as [O][f][S]; this pass contracts the middle digit
    int nf;              // number of factors of the whole transform and the factors themselves
    int factors[3];
    int n_valid;         // LD_REAL: entries at positions >= n_valid are zero; ST_REAL: only t < n_valid is stored
    int H;               // *_CONJ_MULK: row r uses kf row r % H
    int pair_stride;     // *_PAIR: complex row rc packs real rows first = (rc / ps) * 2 ps + rc % ps (re) and first + ps (im):
                         // ps = H pairs batch entries 2 b2, 2 b2 + 1 of a channel, ps = 1 pairs neighbouring rows
    int64_t real_rows;   // *_PAIR: number of real rows (the last complex rows may have no second member)
    float scale;         // store scale (1/N for the inverse)
    int load, store;
    monarch_dtype dt;    // element type of typed loads/stores
};
int launch_fft_pass(const FftPass &p, hipStream_t s);

// Same pass on the matrix cores: bf16 operands, fp32 accumulation, factors 16/32/64/128, every pass
// but the last storing ST_C16 and every pass but the first loading LD_C16.
bool fft_mfma_supported(int N, const int *factors, int nf, monarch_dtype dt);
int launch_fft_pass_mfma(const FftPass &p, hipStream_t s);
// The fp32 version (16x16x4 MFMA): rows stay complex fp32 (LD_C32 / ST_C32) between passes.
bool fft_mfma_f32_supported(int N, const int *factors, int nf, monarch_dtype dt);
int launch_fft_pass_mfma_f32(const FftPass &p, hipStream_t s);

// ---- fp32 MFMA Monarch multiply --------------------------------------------------------------

// Square order-2 Monarch with 16 blocks of 16 x 16 (N = 256), fp32 storage and arithmetic.
bool matmul_mfma_b16_supported(int nbR, int r_out, int r_in, int nbL, int l_out, int l_in, monarch_dtype dt);
int launch_matmul_mfma_b16(const void *x, const void *R, const void *L, void *y, int64_t batch, monarch_dtype dt,
                           hipStream_t s);

// Two factors at once on chunks of f1 x f2 complex numbers held in LDS (bf16; see fft2_lds.hip).  The
// spectrum is left in the forward's in-place order (position [j1][j2] = frequency j2 f1 + j1) and the
// inverse consumes that order.  Loads: LD_REAL / LD_REAL_PAIR (whole rows, two factors) or LD_C16 forward,
// LD_C16_CONJ_MULK / LD_C16_HERM_MULK inverse (kf: packed bf16 pairs in the same order); stores: ST_C16, or
// ST_REAL_SCALE_GATE / ST_REAL_PAIR for the inverse of a two-factor transform.  A real load together with a
// real store runs the whole convolution of a two-factor row in one kernel: forward, times kf, inverse.
struct Fft2Args {
    const void *in;
    void *out;
    const void *gate;
    const void *gate_out;   // fused convolution (real load and real store): gate = input gate, gate_out = output gate
    const void *kf;
    int64_t rows;        // complex rows
    int N, O, f1, f2;    // row length, chunks per row, chunk = f1 x f2
    int n_valid;         // real rows: their length (zero padded / truncated)
    int H, pair_stride;
    int64_t real_rows;
    float scale;
    int load, store, inverse;
    int tw_outer;        // inverse of a three-factor transform: times omega_N^(o (f2 j + col)) after the chunk, o = chunk index
};
// gradients of the order-2 product (csrc/matmul_backward.hip); any of dx, dR, dL may be null
bool matmul_backward_fits(int nbR, int r_out, int r_in, int nbL, int l_out, int l_in);
int launch_matmul_backward(const void *x, const void *R, const void *L, const void *dy, void *dx, float *dR,
                           float *dL, int64_t batch, int nbR, int r_out, int r_in, int nbL, int l_out, int l_in,
                           monarch_dtype dt, hipStream_t s);
// the gated-convolution layer: dense projections (rocBLAS), short depthwise convolutions, the gated long convolution
// (csrc/hyena_layer.hip), with head_dim > 1 the outer products of the heads around it; ws: hyena_layer_workspace_bytes
size_t hyena_layer_workspace_bytes(int B, int n, int d, int klen, int nfft, const int *factors, int nf, int head_dim, monarch_dtype dt);
int launch_hyena_layer(const void *u, const void *W_in, const void *b_in, const void *k_short, const void *k_long, const void *W_out,
                       const void *b_out, void *y, int B, int n, int d, int taps, int klen, int nfft, const int *factors, int nf,
                       int causal, int head_dim, monarch_dtype dt, void *ws, size_t ws_bytes, hipStream_t s);
// square order-2 products with blocks of 32 or 64, in place on LDS tiles, fp32 MFMA (csrc/monarch_inplace.hip):
// the plain product and the gated mixer (g_in, g_out may be null); fp32 or bf16 tensors
bool monarch_inplace_supported(int bs, monarch_dtype dt);
int launch_matmul_inplace(const void *x, const void *R, const void *L, void *y, int64_t batch, int bs, monarch_dtype dt, hipStream_t s);
// Gradients of the square product with blocks of 32 (dx = M^T dy, dR, dL added to cleared buffers); batch > 0.
bool monarch_inplace_backward_supported(int bs, monarch_dtype dt);
int launch_matmul_backward_inplace(const void *x, const void *R, const void *L, const void *dy, void *dx, float *dR, float *dL,
                                   int64_t batch, int bs, monarch_dtype dt, hipStream_t s);
// sequence mixer with two general square order-2 Monarch matrices (csrc/mixer.hip); g_in, g_out may be null
struct MixOpt {
    int act = 0;             // between the kernel product and the second matrix: 0 none, 1 ReLU
    int transposed = 0;      // u, gates and y are (B, N, H) instead of (B, H, N)
    int run = 1;             // (set by the launcher) neighbouring tiles a workgroup takes in a row, transposed access
    int layer_norm = 0;      // y = LayerNorm(result + u) over the row, with gamma, beta (type dt, N entries), eps
    const void *gamma = nullptr, *beta = nullptr;
    float eps = 0.0f;
};
bool mixer_inplace_takes(int bs, int H, monarch_dtype dt, const MixOpt &opt);
int launch_mixer_inplace(const void *u, const void *K, const void *g_in, const void *g_out, const void *R1, const void *L1,
                         const void *R2, const void *L2, void *y, int64_t rows, int H, int bs, monarch_dtype dt, const MixOpt &opt,
                         hipStream_t s);
// the polynomial-parameterised convolution with blocks of 32 or 64 on the same tiles (complex factors of a prepared state)
bool blocky_inplace_takes(int bs, int n, monarch_dtype dt);
int launch_blocky_inplace(const void *u, const void *g_in, const void *g_out, const float2 *R1, const float2 *L1, const float2 *R2,
                          const float2 *L2, const float2 *Kf, void *y, int64_t rows, int H, int n, int bs, monarch_dtype dt, hipStream_t s);
bool mixer_fits(int bs);
int launch_mixer(const void *u, const void *K, const void *g_in, const void *g_out, const void *R1, const void *L1,
                 const void *R2, const void *L2, void *y, int64_t rows, int H, int bs, monarch_dtype dt,
                 const MixOpt &opt, hipStream_t s);
// gradients of the sequence mixer (csrc/mixer_backward.hip); ws: mixer_backward_workspace_bytes
size_t mixer_backward_workspace_bytes(int64_t B, int H, int bs, monarch_dtype dt);
int launch_mixer_backward(const void *u, const void *K, const void *g_in, const void *g_out, const void *R1,
                          const void *L1, const void *R2, const void *L2, const void *dy, void *du, float *dK, void *dg_in,
                          void *dg_out, float *dR1, float *dL1, float *dR2, float *dL2, int64_t B, int H, int bs,
                          monarch_dtype dt, void *ws, hipStream_t s);
// general order-3 Monarch product and its gradients (csrc/matmul3.hip); any of dx, dB1, dB2, dB3 may be null
bool matmul3_fits(int b);
int launch_matmul3(const void *x, const void *B1, const void *B2, const void *B3, void *y, int64_t batch, int b,
                   monarch_dtype dt, hipStream_t s);
int launch_matmul3_backward(const void *x, const void *B1, const void *B2, const void *B3, const void *dy, void *dx,
                            float *dB1, float *dB2, float *dB3, int64_t batch, int b, monarch_dtype dt, hipStream_t s);
// general order-p Monarch product and its gradients (csrc/matmulp.hip); B: (p, b^(p-1), b, b); dx or dB may be null
int matmulp_length(int b, int p, bool backward);   // b^p, or 0 for a shape the kernels do not take
int launch_matmulp(const void *x, const void *B, void *y, int64_t batch, int b, int p, monarch_dtype dt, hipStream_t s);
int launch_matmulp_backward(const void *x, const void *B, const void *dy, void *dx, float *dB, int64_t batch, int b, int p,
                            monarch_dtype dt, hipStream_t s);
// polynomial-parameterised Monarch convolution (csrc/blocky.hip): parameter phase and per-batch phase
bool blocky_fits(int bs);
size_t blocky_state_bytes(int H, int bs);
void blocky_state_offsets(int H, int bs, size_t out[5]);   // byte offsets of R1, L1, R2, L2, Kf
int launch_blocky_prepare(const float *Lt, const float *Rt, const float *k, int H, int klen, int bs, int mask,
                          void *state, hipStream_t s);
int launch_blocky_conv(const void *u, const void *g_in, const void *g_out, const void *state, void *y, int64_t rows,
                       int H, int n, int bs, monarch_dtype dt, hipStream_t s);
bool fft2_lds_supported(int f1, int f2, monarch_dtype dt);
int launch_fft2_lds(const Fft2Args &p, hipStream_t s);
// Three factors, rows pairing two channels: both forward chunk transforms (row in `in`, kernel row in `kf`, each after
// its strided pass), the Hermitian separation with the products, and the inverse chunk transform, in one launch.
bool conv3_middle_supported(int O, int f1, int f2, monarch_dtype dt);
int launch_conv3_middle(const Fft2Args &p, hipStream_t s);

// ---- fused bf16 MFMA kernels ---------------------------------------------------------------

// nfft = 2048 = 64 x 32, n <= 1024, klen <= 1024 (both multiples of 8), bf16 or fp16 I/O.
bool conv_mfma_2048_supported(int n, int klen, const int *factors, int nf, monarch_dtype dt);
int launch_conv_mfma_2048(const void *u, const void *k, const void *g_in, const void *g_out, void *y,
                          int B, int H, int n, int klen, monarch_dtype dt, hipStream_t s);
// the d_h^2 long convolutions per head of the gated-convolution layer with heads, outer products formed on the loads
int launch_conv_mfma_2048_heads(const void *v, const void *k, const void *x2, void *yv, int B, int heads, int dh, int n, int klen,
                                monarch_dtype dt, hipStream_t s);

// nfft = 16384 = 128 x 128, n <= 8192, klen <= 8192 (both multiples of 8), bf16 I/O; no workspace.
bool conv_mfma_16k_supported(int n, int klen, const int *factors, int nf, monarch_dtype dt);
int launch_conv_mfma_16k(const void *u, const void *k, const void *g_in, const void *g_out, void *y,
                         int B, int H, int n, int klen, hipStream_t s);

// Fused causal convolution, nfft = 2048 = 64 x 32, fp32 tensors and fp32 matrix-core arithmetic; n, klen <= 1024,
// multiples of 4 (csrc/conv_f32_2048.hip)
bool conv_f32_2048_supported(int n, int klen, const int *factors, int nf, monarch_dtype dt);
int launch_conv_f32_2048(const void *u, const void *k, const void *g_in, const void *g_out, void *y,
                         int B, int H, int n, int klen, hipStream_t s);

// nfft = 256 = 16 x 16, n <= 128, klen <= 256, bf16 I/O; no workspace.
bool conv_mfma_256_supported(int n, int klen, const int *factors, int nf, monarch_dtype dt);
int launch_conv_mfma_256(const void *u, const void *k, const void *g_in, const void *g_out, void *y,
                         int B, int H, int n, int klen, hipStream_t s);

// Block-diagonal MLP (order 1), bf16 or fp16, d/nb a multiple of 32 up to 192, d_hidden/nb a multiple of 32.
bool mlp_mfma_order1_supported(int d, int d_hidden, int nb, monarch_dtype dt);
// b1_interleaved: hidden unit h of block k reads b1[h nb + k] instead of b1[k (d_hidden / nb) + h].
int launch_mlp_mfma_order1(const void *x, void *y, int64_t tokens, int d, int d_hidden, int nb,
                           const void *W1, const void *b1, const void *W2, const void *b2, int act,
                           int b1_interleaved, monarch_dtype dt, hipStream_t s);

// One block-diagonal factor (nb blocks of r_out x r_in, r_in a multiple of 32 up to 192, r_out a
// multiple of 16) of a rectangular order-2 Monarch with the permutations around it, bf16.
// mode 0: first factor (reads in[c nb + k]); 1: second factor on an already permuted input;
// 2: second factor on the previous factor's natural [block][row] output.  Writes out[r nb + k] (+ bias).
bool factor_mfma_supported(int nb, int r_out, int r_in, monarch_dtype dt);
int launch_factor_mfma(const void *in, void *out, int64_t tokens, int nb, int r_out, int r_in, const void *W,
                       const void *bias, int mode, monarch_dtype dt, hipStream_t s);

}  // namespace monarch
