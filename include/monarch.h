/*
 * monarch.h -- C ABI of the MI355X (gfx950) Monarch Mixer hot-path library.
 *
 * The library implements the Monarch matrix multiply of Monarch Mixer (M2,
 * arXiv 2310.12109, Sec. 3.1) and its two uses in an M2 layer (Sec. 3.2):
 * the Monarch-factored DFT inside the causal gated long convolution (Eq. 2,
 * Thm 3) and the block-diagonal / Monarch MLP (Eq. 3).
 *
 * Common rules for every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller (the library
 *     never frees or keeps it), densely packed in the stated row-major layout
 *     and 16-byte aligned.  `factors` arrays and `host_out` are HOST pointers.
 *   - Calls are asynchronous on `stream` (a hipStream_t passed as an opaque
 *     pointer; NULL is the null stream) and never synchronise the device.
 *   - `ws` is caller-provided device scratch of at least the size the matching
 *     *_workspace_bytes query returns (may be NULL when that size is 0).  Its
 *     contents are undefined after the call; calls sharing one ws must not overlap.
 *   - Output buffers must not alias inputs.
 *   - Return value: MONARCH_OK (0) or a negative error code.  All argument and
 *     shape checks happen before any device work, so a failing call has no side
 *     effect.  monarch_last_error() gives a thread-local message for the last
 *     failure.  The library never throws, aborts or prints.
 *   - I/O element types: MONARCH_F32, MONARCH_BF16 or MONARCH_F16 on the four
 *     hot-path operations (monarch_matmul, monarch_fft / monarch_ifft,
 *     monarch_causal_conv and its _static variant, monarch_mlp); the other entry
 *     points take F32 and BF16 and return MONARCH_EDTYPE for F16.  Arithmetic
 *     accumulates in fp32 always.
 *   - Index conventions: 0-based; omega_N = exp(+2*pi*i/N) (the paper's sign);
 *     sigma_(b,N)(i1*b+i0) = i0*(N/b)+i1 and (P_(b,N) x)[i] = x[sigma(i)]
 *     (appendix notation); block-diagonal factors are stored [block][out][in].
 */
#ifndef MONARCH_H
#define MONARCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { MONARCH_F32 = 0, MONARCH_BF16 = 1, MONARCH_F16 = 2 } monarch_dtype;

enum {
    MONARCH_OK = 0,
    MONARCH_EINVAL = -1,     /* null pointer, misalignment, aliasing, bad flag      */
    MONARCH_ESHAPE = -2,     /* sizes inconsistent, non-factorable or unsupported   */
    MONARCH_EDTYPE = -3,     /* element type not supported by this entry point      */
    MONARCH_EWORKSPACE = -4, /* ws is NULL or smaller than the query says           */
    MONARCH_EHIP = -5        /* a HIP call failed; message holds hipGetErrorString  */
};

typedef void *monarch_stream_t;

/* Human-readable name of an error code (static storage). */
const char *monarch_strerror(int code);
/* Message of the last failing call on this thread ("" if none). */
const char *monarch_last_error(void);

/*
 * Permutation sigma_(b,N) of Sec. 3.1 / appendix notation, as indices:
 * host_out[i1*b + i0] = i0*(N/b) + i1.  Host-only helper (no device work) so
 * that index maps can be checked bit-exactly.  host_out: N int32 on the host.
 * Errors: EINVAL (null), ESHAPE (b <= 0, N <= 0 or b does not divide N).
 */
int monarch_permutation_index(int b, int N, int32_t *host_out);

/*
 * Order-2 Monarch matrix multiply (Sec. 3.1, M = P L P R P), batched:
 *   y[v,:] = P3 * L * P2 * R * P1 * x[v,:],   v in [0, batch).
 * R: [nbR][r_out][r_in] is applied first, L: [nbL][l_out][l_in] second, with
 * d_in = nbR*r_in, d_mid = nbR*r_out = nbL*l_in, d_out = nbL*l_out and
 * P1 = P_(r_in,d_in), P2 = P_(nbR,d_mid), P3 = P_(nbL,d_out).  The paper's
 * square case has all six sizes equal to b = sqrt(N).
 * x: (batch, d_in), y: (batch, d_out), R, L, x, y all of type dt.
 * Errors: EINVAL, ESHAPE (d_mid mismatch, sizes < 1, a row too large for the
 * on-chip tile: (max(d_in, d_out) + d_mid) * 4 bytes beyond 160 KB), EDTYPE, EHIP.
 */
int monarch_matmul(const void *x, const void *R, const void *L, void *y, int64_t batch,
                   int nbR, int r_out, int r_in, int nbL, int l_out, int l_in,
                   monarch_dtype dt, void *ws, size_t ws_bytes, monarch_stream_t stream);
size_t monarch_matmul_workspace_bytes(int64_t batch, int nbR, int r_out, int r_in,
                                      int nbL, int l_out, int l_in, monarch_dtype dt);

/*
 * Gradients of monarch_matmul (Sec. 3.1, M = P L P R P; the chain rule through the five factors of the
 * product), for a training step: with S = sum_v <dy[v,:], y[v,:]>,
 *   dx[v,:] = M^T dy[v,:]                       (batch, d_in), type dt
 *   dR[k][r][c] = dS / dR[k][r][c],  dL alike   shaped like R and L, always float32 (sums over the batch)
 * x, R, L as in monarch_matmul; dy: (batch, d_out) of type dt.  Any of dx, dR, dL may be NULL (not computed);
 * dR and dL are overwritten, not accumulated into.  The sums over the batch are formed with floating-point
 * atomic adds, so their last bits depend on the order in which workgroups finish.
 * Errors: EINVAL (null x, R, L, dy with batch > 0; misalignment; an output overlapping an input), ESHAPE (as
 * monarch_matmul; rows of (d_in + d_out + 2 d_mid) * 4 bytes beyond 160 KB), EDTYPE, EHIP.
 */
int monarch_matmul_backward(const void *x, const void *R, const void *L, const void *dy,
                            void *dx, float *dR, float *dL, int64_t batch,
                            int nbR, int r_out, int r_in, int nbL, int l_out, int l_in,
                            monarch_dtype dt, void *ws, size_t ws_bytes, monarch_stream_t stream);
size_t monarch_matmul_backward_workspace_bytes(int64_t batch, int nbR, int r_out, int r_in,
                                               int nbL, int l_out, int l_in, monarch_dtype dt);

/*
 * General (learned) order-3 Monarch product and its gradients (Sec. 3.1: higher-order Monarch matrices; appendix
 * definition of order-p Monarch matrices, p = 3).  N = b^3; B1, B2, B3: [b*b blocks][b][b], B1 applied first;
 *   M = P^R B3 P_(b,b^2,N) B2 P_(b^2,b^3,N) B1 P^R,   P^R the reversal of the three base-b digits of an index.
 * With j = j2 b^2 + j1 b + j0 (input), m = m2 b^2 + m1 b + m0 (output) and block (p, q) = block p b + q:
 *   t1[(j0,j1), m0] = sum_j2 B1[(j0,j1)][m0, j2] x[j]
 *   t2[(m0,j0), m1] = sum_j1 B2[(m0,j0)][m1, j1] t1[(j0,j1), m0]
 *   y[m]            = sum_j0 B3[(m0,m1)][m2, j0] t2[(m0,j0), m1]
 * (the factors of the order-3 Monarch DFT of monarch_fft are of this form with complex blocks).
 * monarch_matmul3: x, y: (batch, N); x, y and the factors of type dt, fp32 arithmetic.
 * monarch_matmul3_backward: with S = sum_v <dy[v,:], y[v,:]>: dx = M^T dy (type dt) and dB1, dB2, dB3 = dS/dB
 * (always float32, overwritten; sums over the batch by floating-point atomic adds: the last bits depend on the
 * order of the additions).  Any of dx, dB1, dB2, dB3 may be NULL (not computed).
 * Errors: EINVAL (null required pointer with batch > 0, misalignment, overlap), ESHAPE (batch < 0, b outside
 * [1, 16]), EDTYPE, EHIP.
 */
int monarch_matmul3(const void *x, const void *B1, const void *B2, const void *B3, void *y, int64_t batch, int b,
                    monarch_dtype dt, monarch_stream_t stream);
int monarch_matmul3_backward(const void *x, const void *B1, const void *B2, const void *B3, const void *dy, void *dx,
                             float *dB1, float *dB2, float *dB3, int64_t batch, int b, monarch_dtype dt,
                             monarch_stream_t stream);

/*
 * General (learned) order-p Monarch product and its gradients (Sec. 3.1: higher-order Monarch matrices; appendix
 * definition of the p-variate Monarch matrix and the lemma that numbers the blocks of its factors).  N = b^p;
 * B: (p, b^(p-1), b, b), the p block-diagonal factors one after the other, B[0] applied first;
 *   M = P^R B_p P B_(p-1) P ... P B_1 P^R,   P^R the reversal of the p base-b digits of an index.
 * With j = sum_a j_a b^a (input) and m = sum_a m_a b^a (output), factor s = 1 .. p consumes the input digit j_(p-s)
 * and produces the output digit m_(s-1); its blocks are numbered by (m_0 .. m_(s-2), j_0 .. j_(p-s-1)), most
 * significant first (the digits produced so far, then the input digits not yet consumed):
 *   t_s[(m_0 .. m_(s-2), j_0 .. j_(p-s-1)), m_(s-1)] =
 *       sum_c B_s[(m_0 .. m_(s-2), j_0 .. j_(p-s-1))][m_(s-1), c] t_(s-1)[(m_0 .. m_(s-3), j_0 .. j_(p-s-1), c), m_(s-2)]
 * t_0[(j_0 .. j_(p-1))] = x[j], y[m] = t_p[(m_0 .. m_(p-1))].  p = 2 is monarch_matmul's P L P R P with square blocks
 * (R = B_1, L = B_2), p = 3 is monarch_matmul3.
 * monarch_matmulp: x, y: (batch, N); x, y and B of type dt, fp32 arithmetic.
 * monarch_matmulp_backward: with S = sum_v <dy[v,:], y[v,:]>: dx = M^T dy (type dt) and dB = dS/dB (shaped like B,
 * always float32, overwritten; sums over the batch by floating-point atomic adds: the last bits depend on the order
 * of the additions).  dx or dB may be NULL (not computed).
 * Shapes: 2 <= p <= 12, 2 <= b <= 16, b^p <= 4096.
 * Errors: EINVAL (null required pointer with batch > 0, misalignment, overlap), ESHAPE, EDTYPE, EHIP.
 */
int monarch_matmulp(const void *x, const void *B, void *y, int64_t batch, int b, int p, monarch_dtype dt,
                    monarch_stream_t stream);
int monarch_matmulp_backward(const void *x, const void *B, const void *dy, void *dx, float *dB, int64_t batch, int b,
                             int p, monarch_dtype dt, monarch_stream_t stream);

/*
 * Sequence mixer with two general (learned) square order-2 Monarch matrices (Sec. 3.2, Eq. 2, in its gated
 * form): for every sequence b in [0, B) and channel h in [0, H)
 *   y[b,h,:] = g_out[b,h,:] o ( M2 ( K[h,:] o ( M1 ( g_in[b,h,:] o u[b,h,:] ) ) ) ),
 * M1 = P L1 P R1 P and M2 = P L2 P R2 P as in monarch_matmul with all six sizes equal to bs, N = bs^2,
 * both shared by all channels; o is the elementwise product.  With M1 the DFT and M2 its inverse this is the
 * convolution of monarch_causal_conv; here the matrices are arbitrary real ones and K lives in M1's range.
 * u, g_in, g_out, y: (B, H, N); K: (H, N); R1, L1, R2, L2: [bs][bs][bs]; all device memory of type dt, the
 * arithmetic is float32.  g_in and / or g_out may be NULL (no gate).  Nothing is written outside y; a row
 * stays on chip from its load to its store.
 * Errors: EINVAL (a null required pointer with B * H > 0, misalignment, y overlapping an input), ESHAPE
 * (B < 0, H < 1, bs < 1, 2 * bs^2 * 4 bytes beyond 160 KB), EDTYPE, EHIP.
 */
int monarch_mixer(const void *u, const void *K, const void *g_in, const void *g_out,
                  const void *R1, const void *L1, const void *R2, const void *L2, void *y,
                  int64_t B, int H, int bs, monarch_dtype dt, void *ws, size_t ws_bytes, monarch_stream_t stream);
size_t monarch_mixer_workspace_bytes(int64_t B, int H, int bs, monarch_dtype dt);

/*
 * Gradients of monarch_mixer (Sec. 3.2 Eq. 2, gated form; the chain rule through gate, M1, kernel product, M2,
 * gate), for a training step: with S = sum <dy, y>,
 *   du, dg_in, dg_out: (B, H, N), type dt;   dK: (H, N) float32 (a sum over the sequences);
 *   dR1, dL1, dR2, dL2: [bs][bs][bs] float32 (sums over all rows, by floating-point atomic adds: the last bits depend
 *   on the order of the additions).  All are overwritten.  Any of them may be NULL (not computed); dg_in / dg_out
 *   need their gate.
 * Composed from the order-2 product and its gradient kernels with elementwise kernels between them; the
 * intermediate rows (type dt) travel through ws: monarch_mixer_backward_workspace_bytes(B, H, bs, dt) bytes of
 * device memory of the caller (five arrays of the size of u).
 * Errors: EINVAL (null required pointer with B * H > 0, a gate's gradient without the gate, misalignment, overlap),
 * ESHAPE, EWORKSPACE, EDTYPE, EHIP.
 */
int monarch_mixer_backward(const void *u, const void *K, const void *g_in, const void *g_out,
                           const void *R1, const void *L1, const void *R2, const void *L2, const void *dy,
                           void *du, float *dK, void *dg_in, void *dg_out,
                           float *dR1, float *dL1, float *dR2, float *dL2,
                           int64_t B, int H, int bs, monarch_dtype dt, void *ws, size_t ws_bytes, monarch_stream_t stream);
size_t monarch_mixer_backward_workspace_bytes(int64_t B, int H, int bs, monarch_dtype dt);

/*
 * The basic M2 layer (Sec. 3.2: Eq. 2 for the sequence axis and its counterpart for the feature axis, with the
 * non-linearity, skip connection and layer normalisation of the paper's basic implementation):
 *   X~ = ( M2 act( K_n o (M1 X^T) ) )^T           per sequence; K_n: (d, n), one kernel row per feature
 *   Y  = M4 act( k_d o (M3 X~) )                  per position;  k_d: (d,)
 *   y  = LayerNorm(Y + X~)                        over the features: biased variance, eps, weight gamma, bias beta
 * x, y: (B, n, d), n = bn^2, d = bd^2.  M1, M2 = P L P R P with blocks [bn][bn][bn] (R applied first, as in
 * monarch_matmul); M3, M4 with blocks [bd][bd][bd].  act: 0 none, 1 ReLU.  All tensors device memory of type dt,
 * float32 arithmetic.  Two kernels: the sequence mixer reads x and writes X~ in (B, n, d) order directly (no
 * transpose pass), the dimension mixer fuses the skip connection and the normalisation into its store.  ws holds
 * X~: monarch_m2_layer_workspace_bytes(B, n, d, dt) bytes of device memory, owned by the caller.
 * Errors: EINVAL (null or misaligned pointer, act, eps, overlap of x, y, ws), ESHAPE (B < 0, block sizes),
 * EWORKSPACE, EDTYPE, EHIP.
 */
int monarch_m2_layer(const void *x, void *y, int64_t B, int bn, int bd,
                     const void *R1, const void *L1, const void *R2, const void *L2, const void *n_kernel,
                     const void *R3, const void *L3, const void *R4, const void *L4, const void *d_kernel,
                     const void *ln_gamma, const void *ln_beta, float eps, int act,
                     monarch_dtype dt, void *ws, size_t ws_bytes, monarch_stream_t stream);
size_t monarch_m2_layer_workspace_bytes(int64_t B, int n, int d, monarch_dtype dt);

/*
 * The gated-convolution layer of the paper's models (appendix algorithm "M2 Hyena layer with heads" at head
 * dimension 1; with causal = 0 the bidirectional gated convolution of the M2-BERT sequence mixer, Sec. 5):
 *   [X1; X2; V] = W_in u[b,t,:] + b_in            W_in: (3d, d), rows 0..d-1 give X1, d..2d-1 X2, 2d..3d-1 V
 *   X1~, X2~, V~: x~[c,t] = sum_{tau < taps} k_short[c,tau] x[c,t-tau]   (causal depthwise, k_short: (3d, taps))
 *   O = X1~ o conv(k_long, X2~ o V~)              monarch_causal_conv over the sequence, k_long: (d, klen),
 *                                                 nfft / factors / causal as there
 *   y[b,t,:] = W_out O[b,:,t] + b_out             W_out: (d, d)
 * u, y: (B, n, d); everything of type dt (MONARCH_F32 or MONARCH_BF16, fp32 accumulation); b_in, b_out may be
 * NULL.  n a multiple of 8, 1 <= taps <= 8.  The dense projections are plain GEMMs and run in rocBLAS, which the
 * library loads on the first call of this entry point (MONARCH_EHIP if it cannot); that library may allocate
 * device memory of its own on first use.  ws: monarch_hyena_layer_workspace_bytes.
 * Errors: EINVAL (null or misaligned pointer, overlap), ESHAPE (as monarch_causal_conv; n not a multiple of 8;
 * taps outside [1, 8]), EDTYPE, EWORKSPACE, EHIP.
 */
int monarch_hyena_layer(const void *u, const void *W_in, const void *b_in, const void *k_short, const void *k_long,
                        const void *W_out, const void *b_out, void *y, int B, int n, int d, int taps, int klen, int nfft,
                        const int *factors, int nf, int causal, monarch_dtype dt, void *ws, size_t ws_bytes,
                        monarch_stream_t stream);
size_t monarch_hyena_layer_workspace_bytes(int B, int n, int d, int klen, int nfft, const int *factors, int nf,
                                           monarch_dtype dt);

/*
 * The same layer with heads (appendix algorithm "M2 Hyena layer with heads"): the d features form d / head_dim heads
 * of head_dim consecutive features, the long kernel has one row per head (k_long: (d / head_dim, klen)), and per batch
 * entry, head and position, with i, j < head_dim numbering the features of the head,
 *   XV[i][j] = conv(k_long[head], X2~[i] o V~[j])      the outer product of the head, convolved along the sequence
 *   O[j]     = sum_i X1~[i] o XV[i][j]                  multiplied by X1~ position by position
 * Projections, short convolutions and the output projection as in monarch_hyena_layer, which is this entry point at
 * head_dim = 1.  The products X2~[i] o V~[j] and their convolutions go through the workspace as tensors of
 * head_dim times the activation size each (rounded to dt there); the sum over i is formed in fp32.
 * 1 <= head_dim <= 64, head_dim divides d.  ws: monarch_hyena_heads_layer_workspace_bytes.
 * Errors: as monarch_hyena_layer; ESHAPE for a head dimension that is out of range or does not divide d.
 */
int monarch_hyena_heads_layer(const void *u, const void *W_in, const void *b_in, const void *k_short, const void *k_long,
                              const void *W_out, const void *b_out, void *y, int B, int n, int d, int taps, int klen, int nfft,
                              const int *factors, int nf, int causal, int head_dim, monarch_dtype dt, void *ws,
                              size_t ws_bytes, monarch_stream_t stream);
size_t monarch_hyena_heads_layer_workspace_bytes(int B, int n, int d, int klen, int nfft, const int *factors, int nf,
                                                 int head_dim, monarch_dtype dt);

/*
 * Convolution with a polynomial-parameterised ("blocky") Monarch matrix (appendix: the blocky Monarch algorithm,
 * the masking lemma for causality, the blocky Monarch convolution and its causality theorem).
 *
 * Parameters: coefficient matrices Lt, Rt (N x bs, row-major, float32, N = bs^2).  With w_m = exp(+2 pi i / m)
 * they define the complex block-diagonal factors
 *   R_{j1}[i0, j0] = sum_{a < bs} Rt[j1 bs + a, j0] w_bs^(i0 a),   L_{i0}[i1, j1] = sum_{a < N} Lt[a, j1] w_N^((i1 bs + i0) a),
 * M = P L P R P as in monarch_matmul, and per sequence b and channel h
 *   y[b,h,0:n] = g_out[b,h,:] o Re( M^-1 ( (M (k[h,:], 0)) o (M (g_in[b,h,:] o u[b,h,:], 0)) ) )[0:n],
 * M^-1 = P R^-1 P L^-1 P with blockwise inverses.  Identity coefficients (every block of Rt and the top block of
 * Lt the identity, the rest zero) give the DFT and the circular convolution of length N.  mask = 1 zeroes the
 * coefficients the lemma zeroes (of Lt all but the entries [a, j1], j1 <= a < bs; of each block of Rt the entries
 * [a, j0] with a < j0, and with a >= bs/2 in a column j0 < bs/2): then the map is causal in u for
 * n, klen <= bs * floor(bs / 2).
 *
 * monarch_blocky_prepare (once per parameter update): evaluates the factors in float64, inverts the blocks
 * (Gauss-Jordan, partial pivoting, float64), transforms the kernels k (H, klen; float32), and writes all of it as
 * complex float32 into `state` (device memory of the caller, monarch_blocky_state_bytes(H, bs) bytes; see
 * monarch_blocky_state_offsets).  A singular block yields non-finite values in the state and in every later output.
 * monarch_blocky_conv (per batch): u, g_in, g_out, y: (B, H, n) of type dt, n <= N; gates may be NULL; reads the
 * state, writes nothing but y; complex float32 arithmetic, rows stay on chip from load to store.
 * Errors: EINVAL (null or misaligned pointers, mask not 0 / 1, overlap), ESHAPE (bs outside [2, 64], klen or n
 * beyond N, klen beyond bs * floor(bs / 2) with the mask), EWORKSPACE (state too small), EDTYPE, EHIP.
 */
size_t monarch_blocky_state_bytes(int H, int bs);
/* For inspection and tests: byte offsets, within a prepared state, of the complex float32 arrays R1, L1 (factors
 * of M), R2, L2 (factors of M^-1, R2 = blockwise L^-1 applied first), each [bs][bs][bs], and Kf (H, N), written to
 * host_out[0..4] (host memory). */
int monarch_blocky_state_offsets(int H, int bs, size_t *host_out);
int monarch_blocky_prepare(const float *Lt, const float *Rt, const float *k, int H, int klen, int bs, int mask,
                           void *state, size_t state_bytes, monarch_stream_t stream);
int monarch_blocky_conv(const void *u, const void *g_in, const void *g_out, const void *state, size_t state_bytes,
                        void *y, int64_t B, int H, int n, int bs, monarch_dtype dt, monarch_stream_t stream);

/*
 * Monarch-factored DFT (appendix, DFT corollary; order 3 per the p-variate
 * section):  X[r,:] = F_N x[r,:],  F_N[m,j] = omega_N^(m j), unnormalised,
 * natural output order.  N = factors[0]*...*factors[nf-1], nf in {2,3}; the
 * first block-diagonal factor contracts the most significant input digit
 * (size factors[0]), twiddles are folded into the later factors.
 * x: rows x N reals of type dt (real_input = 1) or rows x N interleaved
 * (re,im) pairs of type dt (real_input = 0).  X: rows x N interleaved fp32.
 * monarch_ifft is the exact inverse (minus sign, 1/N included); X is
 * interleaved fp32, x is real (real_output = 1, imaginary part dropped) or
 * interleaved complex, of type dt.
 * Errors: EINVAL, ESHAPE (nf not 2 or 3, product != N, factor < 2, N > 2^24),
 * EDTYPE, EWORKSPACE, EHIP.
 */
int monarch_fft(const void *x, void *X, int64_t rows, int N, const int *factors, int nf,
                int real_input, monarch_dtype dt, void *ws, size_t ws_bytes, monarch_stream_t stream);
int monarch_ifft(const void *X, void *x, int64_t rows, int N, const int *factors, int nf,
                 int real_output, monarch_dtype dt, void *ws, size_t ws_bytes, monarch_stream_t stream);
size_t monarch_fft_workspace_bytes(int64_t rows, int N, const int *factors, int nf, monarch_dtype dt);

/*
 * Gated long convolution through the Monarch DFT (Sec. 3.2 Eq. 2 with the
 * gated form of the same section; Thm 3; appendix review of FFT convolution):
 *   y[b,h,t] = g_out[b,h,t] * sum_s k[h,(t-s)] * (g_in[b,h,s] * u[b,h,s]),  t in [0,n),
 * computed as  F^-1( (F k') o (F u') )  with k', u' zero-padded to nfft and F
 * the Monarch DFT with the given factors (nfft = prod factors).
 *   causal = 1: taps k[h,0..klen-1] at lags 0..klen-1, sum over s <= t; needs
 *               nfft >= n + klen - 1 (no wrap-around), klen <= n.
 *   causal = 0: circular convolution of length nfft truncated to n: lag
 *               (t-s) mod nfft, so negative lags live at the end of k
 *               (klen <= nfft); this is the bidirectional kernel of M2-BERT.
 * u, y, g_in, g_out: (B,H,n); k: (H,klen); all of type dt.  g_in and/or g_out
 * may be NULL (no gate).
 * Errors: EINVAL, ESHAPE (as monarch_fft; n > nfft; aliasing sizes), EDTYPE,
 * EWORKSPACE, EHIP.
 */
int monarch_causal_conv(const void *u, const void *k, const void *g_in, const void *g_out, void *y,
                        int B, int H, int n, int klen, int nfft, const int *factors, int nf,
                        int causal, monarch_dtype dt, void *ws, size_t ws_bytes,
                        monarch_stream_t stream);
size_t monarch_causal_conv_workspace_bytes(int B, int H, int n, int klen, int nfft,
                                           const int *factors, int nf, monarch_dtype dt);

/*
 * monarch_causal_conv for callers that cannot allocate device memory or pass a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid allocation.  Same arguments, results and errors as monarch_causal_conv
 * without ws / ws_bytes; the scratch memory the multi-pass paths need (row
 * buffers between the passes, the spectrum of k) is a static device array of
 * MONARCH_STATIC_SCRATCH_BYTES inside the library, which every GPU the library
 * runs on holds until the process ends.  The call allocates nothing and frees
 * nothing.  A shape whose monarch_causal_conv_workspace_bytes exceeds
 * MONARCH_STATIC_SCRATCH_BYTES returns MONARCH_EWORKSPACE (no device work).
 * All calls on one GPU share that GPU's array: calls that overlap in time on
 * one GPU (different streams, different threads) race and give undefined
 * results; serialise them.  Nothing in the array needs to start at zero.
 */
#define MONARCH_STATIC_SCRATCH_BYTES (32u << 20)
int monarch_causal_conv_static(const void *u, const void *k, const void *g_in, const void *g_out, void *y,
                               int B, int H, int n, int klen, int nfft, const int *factors, int nf,
                               int causal, monarch_dtype dt, monarch_stream_t stream);

/*
 * Monarch MLP, the dimension mixer (Sec. 3.2 Eq. 3):
 *   y[t,:] = W2 * act(W1 * x[t,:] + b1) + b2,   t in [0, tokens),
 * W1: d -> d_hidden, W2: d_hidden -> d.
 *   order 1: Wi = diag of nb blocks (the M2-BERT dimension mixer);
 *            W1_R: [nb][d_hidden/nb][d/nb], W2_R: [nb][d/nb][d_hidden/nb];
 *            W1_L, W2_L must be NULL.
 *   order 2: Wi = P L P R P as in monarch_matmul with nb blocks per factor and
 *            inner widths mid1, mid2 (0 means d):
 *            W1_R: [nb][mid1/nb][d/nb], W1_L: [nb][d_hidden/nb][mid1/nb],
 *            W2_R: [nb][mid2/nb][d_hidden/nb], W2_L: [nb][d/nb][mid2/nb].
 * act: 0 none, 1 ReLU, 2 GELU (erf form: z * Phi(z); the 16-bit matrix-core
 * kernels evaluate Phi by a polynomial in fp16 with |Phi error| <= 1e-3, an
 * absolute bound: the result is within 1e-3 |z| of z Phi(z), and 0 below
 * z = -3.25).  b1
 * (d_hidden) and b2 (d) may be NULL.  x, y: (tokens, d); everything of type dt.
 * Errors: EINVAL, ESHAPE (nb does not divide the widths, order not 1 or 2,
 * widths beyond the on-chip tile), EDTYPE, EWORKSPACE, EHIP.
 */
int monarch_mlp(const void *x, void *y, int64_t tokens, int d, int d_hidden, int nb, int order,
                const void *W1_R, const void *W1_L, const void *b1,
                const void *W2_R, const void *W2_L, const void *b2,
                int mid1, int mid2, int act, monarch_dtype dt, void *ws, size_t ws_bytes,
                monarch_stream_t stream);
size_t monarch_mlp_workspace_bytes(int64_t tokens, int d, int d_hidden, int nb, int order,
                                   int mid1, int mid2, monarch_dtype dt);

#ifdef __cplusplus
}
#endif
#endif /* MONARCH_H */
