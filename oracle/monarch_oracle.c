/*
 * CPU oracle for the Monarch Mixer hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the plain, slow, double-precision statement of what every entry
 * point of the GPU library has to compute.  It is written from the paper
 * (Monarch Mixer, arXiv 2310.12109) and shares no code, header, table or
 * constant with the HIP path.  Only the tests, the smoke check and the
 * cpu_baseline leg of the benchmark may call it; the product never does.
 *
 * Conventions (all indices 0-based, matrices row-major):
 *   sigma_(b,N)(i1*b + i0) = i0*(N/b) + i1        (Appendix, Notation, item 6)
 *   P_(b,N) has e_sigma(i) as its i-th row, so (P x)[i] = x[sigma(i)]:
 *   view x as a (b x N/b) row-major matrix, transpose it, flatten it (Sec. 3.1).
 *   omega_N = exp(+2*pi*i/N), F_N[m,j] = omega_N^(m*j)   (Appendix, DFT corollary).
 *   Block-diagonal factors are stored [block][out][in] (Appendix listing, einsum "bnm").
 *
 * Every function is the definition written out; nothing is blocked, fused or
 * reordered.  OpenMP is used only to run independent rows on several cores.
 */
#include <complex.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef double complex cplx;

#define TWO_PI 6.283185307179586476925286766559

/* omega_N^e with the integer exponent reduced mod N first, so that the angle
 * handed to cos/sin stays in [0, 2*pi) whatever the size of m*j. */
static cplx omega_pow(int64_t N, int64_t e)
{
    int64_t r = e % N;
    if (r < 0) r += N;
    double ang = TWO_PI * (double)r / (double)N;
    return cos(ang) + I * sin(ang);
}

/* ------------------------------------------------------------------------- */
/* Permutation (Sec. 3.1; Appendix, Notation item 6)                         */
/* ------------------------------------------------------------------------- */

/* sigma[i1*b + i0] = i0*(N/b) + i1 for 0 <= i0 < b, 0 <= i1 < N/b.  Returns 0,
 * or -1 when b does not divide N. */
int oracle_perm(int b, int N, int32_t *sigma)
{
    if (b <= 0 || N <= 0 || N % b != 0) return -1;
    int q = N / b;
    for (int i1 = 0; i1 < q; ++i1)
        for (int i0 = 0; i0 < b; ++i0)
            sigma[i1 * b + i0] = i0 * q + i1;
    return 0;
}

/* Dense N x N matrix of P_(b,N): row i is the unit vector e_sigma(i). */
static void dense_perm(int b, int N, double *P)
{
    int32_t *s = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    oracle_perm(b, N, s);
    memset(P, 0, sizeof(double) * (size_t)N * (size_t)N);
    for (int i = 0; i < N; ++i) P[(size_t)i * N + s[i]] = 1.0;
    free(s);
}

static void dense_perm_c(int b, int N, cplx *P)
{
    int32_t *s = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    oracle_perm(b, N, s);
    for (size_t t = 0; t < (size_t)N * N; ++t) P[t] = 0.0;
    for (int i = 0; i < N; ++i) P[(size_t)i * N + s[i]] = 1.0;
    free(s);
}

/* ------------------------------------------------------------------------- */
/* Block-diagonal factor and dense products                                  */
/* ------------------------------------------------------------------------- */

/* W is [nb][out][in]; D becomes the (nb*out) x (nb*in) matrix diag(W_0..W_{nb-1}). */
static void dense_blockdiag(const double *W, int nb, int out, int in, double *D)
{
    size_t rows = (size_t)nb * out, cols = (size_t)nb * in;
    memset(D, 0, sizeof(double) * rows * cols);
    for (int k = 0; k < nb; ++k)
        for (int r = 0; r < out; ++r)
            for (int c = 0; c < in; ++c)
                D[((size_t)k * out + r) * cols + (size_t)k * in + c] =
                    W[((size_t)k * out + r) * in + c];
}

static void dense_blockdiag_c(const cplx *W, int nb, int out, int in, cplx *D)
{
    size_t rows = (size_t)nb * out, cols = (size_t)nb * in;
    for (size_t t = 0; t < rows * cols; ++t) D[t] = 0.0;
    for (int k = 0; k < nb; ++k)
        for (int r = 0; r < out; ++r)
            for (int c = 0; c < in; ++c)
                D[((size_t)k * out + r) * cols + (size_t)k * in + c] =
                    W[((size_t)k * out + r) * in + c];
}

/* C (m x n) = A (m x k) * B (k x n), the textbook triple loop.  Exact zeros of
 * A are skipped: they contribute exactly nothing, and permutation and
 * block-diagonal matrices are mostly zeros. */
static void dense_mul(const double *A, const double *B, double *C, int m, int k, int n)
{
#pragma omp parallel for schedule(static)
    for (int i = 0; i < m; ++i) {
        double *c = C + (size_t)i * n;
        for (int j = 0; j < n; ++j) c[j] = 0.0;
        for (int l = 0; l < k; ++l) {
            double a = A[(size_t)i * k + l];
            if (a == 0.0) continue;
            const double *b = B + (size_t)l * n;
            for (int j = 0; j < n; ++j) c[j] += a * b[j];
        }
    }
}

static void dense_mul_c(const cplx *A, const cplx *B, cplx *C, int m, int k, int n)
{
#pragma omp parallel for schedule(static)
    for (int i = 0; i < m; ++i) {
        cplx *c = C + (size_t)i * n;
        for (int j = 0; j < n; ++j) c[j] = 0.0;
        for (int l = 0; l < k; ++l) {
            cplx a = A[(size_t)i * k + l];
            if (a == 0.0) continue;
            const cplx *b = B + (size_t)l * n;
            for (int j = 0; j < n; ++j) c[j] += a * b[j];
        }
    }
}

/* ------------------------------------------------------------------------- */
/* Order-2 Monarch matrix  M = P3 * L * P2 * R * P1   (Sec. 3.1)             */
/* ------------------------------------------------------------------------- */

/*
 * R: [nbR][r_out][r_in] is applied first, L: [nbL][l_out][l_in] second.
 * d_in = nbR*r_in, d_mid = nbR*r_out = nbL*l_in, d_out = nbL*l_out.
 * P1 = P_(r_in, d_in), P2 = P_(nbR, d_mid), P3 = P_(nbL, d_out).  In the
 * paper's square case all six sizes equal b = sqrt(N) and P1 = P2 = P3 = P_(b,N).
 * M is d_out x d_in.  Returns 0, -1 on inconsistent sizes.
 */
int oracle_monarch_dense(const double *R, const double *L, int nbR, int r_out, int r_in,
                         int nbL, int l_out, int l_in, double *M)
{
    if (nbR <= 0 || r_out <= 0 || r_in <= 0 || nbL <= 0 || l_out <= 0 || l_in <= 0) return -1;
    if ((int64_t)nbR * r_out != (int64_t)nbL * l_in) return -1;
    int d_in = nbR * r_in, d_mid = nbR * r_out, d_out = nbL * l_out;

    double *P1 = (double *)malloc(sizeof(double) * (size_t)d_in * d_in);
    double *Rd = (double *)malloc(sizeof(double) * (size_t)d_mid * d_in);
    double *P2 = (double *)malloc(sizeof(double) * (size_t)d_mid * d_mid);
    double *Ld = (double *)malloc(sizeof(double) * (size_t)d_out * d_mid);
    double *P3 = (double *)malloc(sizeof(double) * (size_t)d_out * d_out);
    double *T1 = (double *)malloc(sizeof(double) * (size_t)d_mid * d_in);
    double *T2 = (double *)malloc(sizeof(double) * (size_t)d_mid * d_in);
    double *T3 = (double *)malloc(sizeof(double) * (size_t)d_out * d_in);

    dense_perm(r_in, d_in, P1);
    dense_blockdiag(R, nbR, r_out, r_in, Rd);
    dense_perm(nbR, d_mid, P2);
    dense_blockdiag(L, nbL, l_out, l_in, Ld);
    dense_perm(nbL, d_out, P3);

    dense_mul(Rd, P1, T1, d_mid, d_in, d_in);   /* R P1          */
    dense_mul(P2, T1, T2, d_mid, d_mid, d_in);  /* P2 R P1       */
    dense_mul(Ld, T2, T3, d_out, d_mid, d_in);  /* L P2 R P1     */
    dense_mul(P3, T3, M, d_out, d_out, d_in);   /* P3 L P2 R P1  */

    free(P1); free(Rd); free(P2); free(Ld); free(P3); free(T1); free(T2); free(T3);
    return 0;
}

/* The same product with complex factors (needed for the DFT instance). */
int oracle_monarch_dense_c(const cplx *R, const cplx *L, int nbR, int r_out, int r_in,
                           int nbL, int l_out, int l_in, cplx *M)
{
    if (nbR <= 0 || r_out <= 0 || r_in <= 0 || nbL <= 0 || l_out <= 0 || l_in <= 0) return -1;
    if ((int64_t)nbR * r_out != (int64_t)nbL * l_in) return -1;
    int d_in = nbR * r_in, d_mid = nbR * r_out, d_out = nbL * l_out;

    cplx *P1 = (cplx *)malloc(sizeof(cplx) * (size_t)d_in * d_in);
    cplx *Rd = (cplx *)malloc(sizeof(cplx) * (size_t)d_mid * d_in);
    cplx *P2 = (cplx *)malloc(sizeof(cplx) * (size_t)d_mid * d_mid);
    cplx *Ld = (cplx *)malloc(sizeof(cplx) * (size_t)d_out * d_mid);
    cplx *P3 = (cplx *)malloc(sizeof(cplx) * (size_t)d_out * d_out);
    cplx *T1 = (cplx *)malloc(sizeof(cplx) * (size_t)d_mid * d_in);
    cplx *T2 = (cplx *)malloc(sizeof(cplx) * (size_t)d_mid * d_in);
    cplx *T3 = (cplx *)malloc(sizeof(cplx) * (size_t)d_out * d_in);

    dense_perm_c(r_in, d_in, P1);
    dense_blockdiag_c(R, nbR, r_out, r_in, Rd);
    dense_perm_c(nbR, d_mid, P2);
    dense_blockdiag_c(L, nbL, l_out, l_in, Ld);
    dense_perm_c(nbL, d_out, P3);

    dense_mul_c(Rd, P1, T1, d_mid, d_in, d_in);
    dense_mul_c(P2, T1, T2, d_mid, d_mid, d_in);
    dense_mul_c(Ld, T2, T3, d_out, d_mid, d_in);
    dense_mul_c(P3, T3, M, d_out, d_out, d_in);

    free(P1); free(Rd); free(P2); free(Ld); free(P3); free(T1); free(T2); free(T3);
    return 0;
}

/* y[v,:] = M x[v,:] for v < batch, with M materialised densely as above.
 * x is batch x d_in, y is batch x d_out. */
int oracle_matmul(const double *x, const double *R, const double *L, double *y, int64_t batch,
                  int nbR, int r_out, int r_in, int nbL, int l_out, int l_in)
{
    int d_in = nbR * r_in, d_out = nbL * l_out;
    double *M = (double *)malloc(sizeof(double) * (size_t)d_out * d_in);
    int rc = oracle_monarch_dense(R, L, nbR, r_out, r_in, nbL, l_out, l_in, M);
    if (rc != 0) { free(M); return rc; }
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < batch; ++v)
        for (int i = 0; i < d_out; ++i) {
            double s = 0.0;
            for (int j = 0; j < d_in; ++j) s += M[(size_t)i * d_in + j] * x[(size_t)v * d_in + j];
            y[(size_t)v * d_out + i] = s;
        }
    free(M);
    return 0;
}

/*
 * Gradients of S = sum_v <dy[v,:], M x[v,:]> with M = P3 L P2 R P1 (Sec. 3.1), by the chain rule through the
 * five steps of the product, each step's adjoint written out (own derivation; the paper states the forward
 * product only):
 *   forward   t0 = P1 x,  t1 = R t0,  t2 = P2 t1,  t3 = L t2,  y = P3 t3
 *   backward  g3 = P3^T dy,  dL_k += g3_k t2_k^T,  g2 = L^T g3,  g1 = P2^T g2,  dR_k += g1_k t0_k^T,
 *             g0 = R^T g1,  dx = P1^T g0
 * x: batch x d_in, dy: batch x d_out, dx: batch x d_in, dR: like R, dL: like L (sums over the batch).
 * Any of dx, dR, dL may be NULL.  Returns 0, -1 on inconsistent sizes.
 */
int oracle_matmul_backward(const double *x, const double *R, const double *L, const double *dy,
                           double *dx, double *dR, double *dL, int64_t batch,
                           int nbR, int r_out, int r_in, int nbL, int l_out, int l_in)
{
    if (nbR <= 0 || r_out <= 0 || r_in <= 0 || nbL <= 0 || l_out <= 0 || l_in <= 0) return -1;
    if ((int64_t)nbR * r_out != (int64_t)nbL * l_in) return -1;
    int d_in = nbR * r_in, d_mid = nbR * r_out, d_out = nbL * l_out;
    int32_t *s1 = (int32_t *)malloc(sizeof(int32_t) * (size_t)d_in);
    int32_t *s2 = (int32_t *)malloc(sizeof(int32_t) * (size_t)d_mid);
    int32_t *s3 = (int32_t *)malloc(sizeof(int32_t) * (size_t)d_out);
    oracle_perm(r_in, d_in, s1);    /* (P1 x)[i] = x[s1[i]] */
    oracle_perm(nbR, d_mid, s2);
    oracle_perm(nbL, d_out, s3);
    if (dR) memset(dR, 0, sizeof(double) * (size_t)nbR * r_out * r_in);
    if (dL) memset(dL, 0, sizeof(double) * (size_t)nbL * l_out * l_in);
    double *t0 = (double *)malloc(sizeof(double) * (size_t)d_in);
    double *t1 = (double *)malloc(sizeof(double) * (size_t)d_mid);
    double *t2 = (double *)malloc(sizeof(double) * (size_t)d_mid);
    double *g3 = (double *)malloc(sizeof(double) * (size_t)d_out);
    double *g2 = (double *)malloc(sizeof(double) * (size_t)d_mid);
    double *g1 = (double *)malloc(sizeof(double) * (size_t)d_mid);
    double *g0 = (double *)malloc(sizeof(double) * (size_t)d_in);
    for (int64_t v = 0; v < batch; ++v) {   /* (serial: the parameter gradients are sums over v) */
        const double *xv = x + (size_t)v * d_in, *dyv = dy + (size_t)v * d_out;
        for (int i = 0; i < d_in; ++i) t0[i] = xv[s1[i]];
        for (int k = 0; k < nbR; ++k)
            for (int r = 0; r < r_out; ++r) {
                double acc = 0.0;
                for (int c = 0; c < r_in; ++c) acc += R[((size_t)k * r_out + r) * r_in + c] * t0[k * r_in + c];
                t1[k * r_out + r] = acc;
            }
        for (int i = 0; i < d_mid; ++i) t2[i] = t1[s2[i]];
        /* g3 = P3^T dy:  y[i] = t3[s3[i]]  =>  g3[s3[i]] = dy[i] */
        for (int i = 0; i < d_out; ++i) g3[s3[i]] = dyv[i];
        for (int k = 0; k < nbL; ++k)
            for (int r = 0; r < l_out; ++r)
                for (int a = 0; a < l_in; ++a)
                    if (dL) dL[((size_t)k * l_out + r) * l_in + a] += g3[k * l_out + r] * t2[k * l_in + a];
        for (int k = 0; k < nbL; ++k)
            for (int a = 0; a < l_in; ++a) {
                double acc = 0.0;
                for (int r = 0; r < l_out; ++r) acc += L[((size_t)k * l_out + r) * l_in + a] * g3[k * l_out + r];
                g2[k * l_in + a] = acc;
            }
        /* g1 = P2^T g2:  t2[i] = t1[s2[i]]  =>  g1[s2[i]] = g2[i] */
        for (int i = 0; i < d_mid; ++i) g1[s2[i]] = g2[i];
        for (int k = 0; k < nbR; ++k)
            for (int r = 0; r < r_out; ++r)
                for (int c = 0; c < r_in; ++c)
                    if (dR) dR[((size_t)k * r_out + r) * r_in + c] += g1[k * r_out + r] * t0[k * r_in + c];
        if (dx) {
            for (int k = 0; k < nbR; ++k)
                for (int c = 0; c < r_in; ++c) {
                    double acc = 0.0;
                    for (int r = 0; r < r_out; ++r) acc += R[((size_t)k * r_out + r) * r_in + c] * g1[k * r_out + r];
                    g0[k * r_in + c] = acc;
                }
            /* dx = P1^T g0:  t0[i] = x[s1[i]]  =>  dx[s1[i]] = g0[i] */
            for (int i = 0; i < d_in; ++i) dx[(size_t)v * d_in + s1[i]] = g0[i];
        }
    }
    free(s1); free(s2); free(s3); free(t0); free(t1); free(t2); free(g3); free(g2); free(g1); free(g0);
    return 0;
}

/*
 * Sequence mixer with two general (learned) order-2 Monarch matrices, Sec. 3.2 Eq. 2 and its gated form:
 *   y[b,h,:] = g_out[b,h,:] o ( M2 ( K[h,:] o ( M1 ( g_in[b,h,:] o u[b,h,:] ) ) ) ),   o = elementwise product,
 * M1 = P L1 P R1 P and M2 = P L2 P R2 P square of size N = nb*nb... in general M1: d_in -> d_mid1 given by
 * its factor shapes; here both are N x N with blocks [bs][bs][bs], N = bs*bs, shared by all channels; K is
 * the kernel in the transform domain, one row per channel.  With M1 the DFT and M2 its inverse this is the
 * convolution; here the matrices are arbitrary.  u, g_in, g_out, y: rows x N with row = b*H + h; K: H x N.
 * g_in / g_out may be NULL (= 1).  Both matrices are materialised densely.
 */
int oracle_mixer(const double *u, const double *K, const double *g_in, const double *g_out,
                 const double *R1, const double *L1, const double *R2, const double *L2,
                 double *y, int64_t rows, int H, int bs)
{
    if (bs <= 0 || H <= 0) return -1;
    int N = bs * bs;
    double *M1 = (double *)malloc(sizeof(double) * (size_t)N * N);
    double *M2 = (double *)malloc(sizeof(double) * (size_t)N * N);
    int rc = oracle_monarch_dense(R1, L1, bs, bs, bs, bs, bs, bs, M1);
    if (rc == 0) rc = oracle_monarch_dense(R2, L2, bs, bs, bs, bs, bs, bs, M2);
    if (rc != 0) { free(M1); free(M2); return rc; }
#pragma omp parallel
    {
        double *a = (double *)malloc(sizeof(double) * (size_t)N);
        double *t = (double *)malloc(sizeof(double) * (size_t)N);
#pragma omp for schedule(static)
        for (int64_t r = 0; r < rows; ++r) {
            const int h = (int)(r % H);
            for (int j = 0; j < N; ++j) a[j] = u[(size_t)r * N + j] * (g_in ? g_in[(size_t)r * N + j] : 1.0);
            for (int i = 0; i < N; ++i) {
                double s = 0.0;
                for (int j = 0; j < N; ++j) s += M1[(size_t)i * N + j] * a[j];
                t[i] = s * K[(size_t)h * N + i];
            }
            for (int i = 0; i < N; ++i) {
                double s = 0.0;
                for (int j = 0; j < N; ++j) s += M2[(size_t)i * N + j] * t[j];
                y[(size_t)r * N + i] = s * (g_out ? g_out[(size_t)r * N + i] : 1.0);
            }
        }
        free(a); free(t);
    }
    free(M1); free(M2);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* DFT by its definition (Appendix: F_N[m,j] = omega_N^(m j))                */
/* ------------------------------------------------------------------------- */

/* X[r,m] = sum_j x[r,j] * omega_N^(m j), unnormalised, + sign. */
void oracle_dft(const cplx *x, cplx *X, int64_t rows, int N)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int m = 0; m < N; ++m) {
            cplx s = 0.0;
            for (int j = 0; j < N; ++j) s += x[(size_t)r * N + j] * omega_pow(N, (int64_t)m * j);
            X[(size_t)r * N + m] = s;
        }
}

/* The same definition for a chosen list of output bins only (large N):
 * Xb[r,q] = sum_j x[r,j] * omega_N^(bins[q] j). */
void oracle_dft_bins(const cplx *x, cplx *Xb, int64_t rows, int N, const int32_t *bins, int nbins)
{
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t r = 0; r < rows; ++r)
        for (int q = 0; q < nbins; ++q) {
            cplx s = 0.0;
            for (int j = 0; j < N; ++j) s += x[(size_t)r * N + j] * omega_pow(N, (int64_t)bins[q] * j);
            Xb[(size_t)r * nbins + q] = s;
        }
}

/* x[r,j] = (1/N) sum_m X[r,m] * omega_N^(-m j): the inverse of oracle_dft. */
void oracle_idft(const cplx *X, cplx *x, int64_t rows, int N)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int j = 0; j < N; ++j) {
            cplx s = 0.0;
            for (int m = 0; m < N; ++m) s += X[(size_t)r * N + m] * omega_pow(N, -(int64_t)m * j);
            x[(size_t)r * N + j] = s / (double)N;
        }
}

/*
 * Block-diagonal factors that make the order-2 Monarch product equal F_N,
 * N = N1*N2 (DFT corollary of the appendix; the rectangular split uses the
 * same argument with P_(N1,N), P_(N2,N), P_(N1,N)):
 *   R: N2 blocks, each N1 x N1:  R_a[i,c] = omega_N1^(i c)
 *   L: N1 blocks, each N2 x N2:  L_i[k,a] = omega_N2^(k a) * omega_N^(i a)
 * so that, with x[c*N2 + a] as input, output index m = k*N1 + i.
 */
void oracle_dft_factors(int N1, int N2, cplx *R, cplx *L)
{
    int64_t N = (int64_t)N1 * N2;
    for (int a = 0; a < N2; ++a)
        for (int i = 0; i < N1; ++i)
            for (int c = 0; c < N1; ++c)
                R[((size_t)a * N1 + i) * N1 + c] = omega_pow(N1, (int64_t)i * c);
    for (int i = 0; i < N1; ++i)
        for (int k = 0; k < N2; ++k)
            for (int a = 0; a < N2; ++a)
                L[((size_t)i * N2 + k) * N2 + a] =
                    omega_pow(N2, (int64_t)k * a) * omega_pow(N, (int64_t)i * a);
}

/* Dense N x N matrix of the Monarch product built from oracle_dft_factors. */
int oracle_monarch_dft_dense(int N1, int N2, cplx *M)
{
    size_t N = (size_t)N1 * N2;
    cplx *R = (cplx *)malloc(sizeof(cplx) * N * N1);
    cplx *L = (cplx *)malloc(sizeof(cplx) * N * N2);
    oracle_dft_factors(N1, N2, R, L);
    int rc = oracle_monarch_dense_c(R, L, N2, N1, N1, N1, N2, N2, M);
    free(R); free(L);
    return rc;
}

/* ------------------------------------------------------------------------- */
/* Order-3 Monarch  M = P3 * B3 * P2 * B2 * P1 * B1 * P0   (Sec. 3.1, Eq. 1;  */
/* permutations from the appendix section on p-variate Monarch matrices)      */
/* ------------------------------------------------------------------------- */

/* Dense block-diagonal permutation P_(bp,Mp,N) = diag(P_(bp,Mp), ..., N/Mp times). */
static void dense_perm3_c(int bp, int Mp, int N, cplx *P)
{
    int32_t *s = (int32_t *)malloc(sizeof(int32_t) * (size_t)Mp);
    oracle_perm(bp, Mp, s);
    for (size_t t = 0; t < (size_t)N * N; ++t) P[t] = 0.0;
    for (int blk = 0; blk < N / Mp; ++blk)
        for (int i = 0; i < Mp; ++i)
            P[((size_t)blk * Mp + i) * N + (size_t)blk * Mp + s[i]] = 1.0;
    free(s);
}

/*
 * Order-3 Monarch matrix for N = b^3 from three block-diagonal factors, each
 * [b*b blocks][b][b] complex, B1 applied first:
 *   M = P^R * B3 * P_(b,b^2,N) * B2 * P_(b^2,b^3,N) * B1 * P^R
 * P^R = P_(b,b^2,N) * P_(b^2,b^3,N) is the sub-index reversal
 * (i2,i1,i0) -> (i0,i1,i2); P_(b',M,N) = diag of N/M copies of P_(b',M).
 * With these choices the blocks of the a-th factor are numbered by the output
 * sub-indices already produced (most significant) followed by the input
 * sub-indices not yet consumed, which is the block numbering the appendix
 * lemma on p-variate Monarch matrices prescribes.
 */
int oracle_monarch3_dense_c(const cplx *B1, const cplx *B2, const cplx *B3, int b, cplx *M)
{
    if (b <= 0) return -1;
    int N = b * b * b, nb = b * b;
    size_t NN = (size_t)N * N;
    cplx *D = (cplx *)malloc(sizeof(cplx) * NN);
    cplx *Pa = (cplx *)malloc(sizeof(cplx) * NN);
    cplx *Pb = (cplx *)malloc(sizeof(cplx) * NN);
    cplx *PR = (cplx *)malloc(sizeof(cplx) * NN);
    cplx *T1 = (cplx *)malloc(sizeof(cplx) * NN);
    cplx *T2 = (cplx *)malloc(sizeof(cplx) * NN);

    dense_perm3_c(b, b * b, N, Pa);      /* P_(b,   b^2, N) */
    dense_perm3_c(b * b, N, N, Pb);      /* P_(b^2, b^3, N) */
    dense_mul_c(Pa, Pb, PR, N, N, N);    /* sub-index reversal */

    dense_blockdiag_c(B1, nb, b, b, D);
    dense_mul_c(D, PR, T1, N, N, N);                     /* B1 P0                   */
    dense_mul_c(Pb, T1, T2, N, N, N);                    /* P1 B1 P0                */
    dense_blockdiag_c(B2, nb, b, b, D);
    dense_mul_c(D, T2, T1, N, N, N);                     /* B2 P1 B1 P0             */
    dense_mul_c(Pa, T1, T2, N, N, N);                    /* P2 B2 P1 B1 P0          */
    dense_blockdiag_c(B3, nb, b, b, D);
    dense_mul_c(D, T2, T1, N, N, N);                     /* B3 P2 B2 P1 B1 P0       */
    dense_mul_c(PR, T1, M, N, N, N);                     /* P3 B3 P2 B2 P1 B1 P0    */

    free(D); free(Pa); free(Pb); free(PR); free(T1); free(T2);
    return 0;
}

/*
 * Blocks that make the order-3 product above equal F_N for N = b^3.  Write the
 * input index j = j2*b^2 + j1*b + j0 and the output index m = m2*b^2 + m1*b + m0;
 * omega_N^(m j) splits into omega_b^(m0 j2) * omega_b^(m1 j1) * omega_b^(m2 j0)
 * * omega_(b^2)^(m0 j1) * omega_(b^2)^(m1 j0) * omega_N^(m0 j0), hence
 *   B1 block (j0,j1):  [m0, j2] = omega_b^(m0 j2)
 *   B2 block (m0,j0):  [m1, j1] = omega_b^(m1 j1) * omega_(b^2)^(m0 j1)
 *   B3 block (m0,m1):  [m2, j0] = omega_b^(m2 j0) * omega_N^((m1 b + m0) j0)
 * where block (p,q) is block number p*b + q.
 */
void oracle_dft3_factors(int b, cplx *B1, cplx *B2, cplx *B3)
{
    int64_t N = (int64_t)b * b * b;
    for (int p = 0; p < b; ++p)
        for (int q = 0; q < b; ++q)
            for (int r = 0; r < b; ++r)
                for (int c = 0; c < b; ++c) {
                    size_t at = (((size_t)p * b + q) * b + r) * b + c;
                    /* B1: (p,q) = (j0,j1), r = m0, c = j2 */
                    B1[at] = omega_pow(b, (int64_t)r * c);
                    /* B2: (p,q) = (m0,j0), r = m1, c = j1 */
                    B2[at] = omega_pow(b, (int64_t)r * c) * omega_pow((int64_t)b * b, (int64_t)p * c);
                    /* B3: (p,q) = (m0,m1), r = m2, c = j0 */
                    B3[at] = omega_pow(b, (int64_t)r * c) * omega_pow(N, ((int64_t)q * b + p) * c);
                }
}

/* Dense N x N matrix of the order-3 product built from oracle_dft3_factors. */
int oracle_monarch3_dft_dense(int b, cplx *M)
{
    size_t nblk = (size_t)b * b * b * b;
    cplx *B1 = (cplx *)malloc(sizeof(cplx) * nblk);
    cplx *B2 = (cplx *)malloc(sizeof(cplx) * nblk);
    cplx *B3 = (cplx *)malloc(sizeof(cplx) * nblk);
    oracle_dft3_factors(b, B1, B2, B3);
    int rc = oracle_monarch3_dense_c(B1, B2, B3, b, M);
    free(B1); free(B2); free(B3);
    return rc;
}

/* ------------------------------------------------------------------------- */
/* Causal / circular long convolution (Sec. 2; Appendix review of Thm 3)      */
/* ------------------------------------------------------------------------- */

/*
 * causal = 1:  y[b,h,t] = g_out[b,h,t] * sum_{s=0..t, t-s<klen} k[h,t-s] * g_in[b,h,s]*u[b,h,s]
 * causal = 0:  y[b,h,t] = g_out[b,h,t] * sum_{s<n} k[h,(t-s) mod nfft] * g_in[b,h,s]*u[b,h,s],
 *              taps with (t-s) mod nfft >= klen being zero.
 * u, y, g_in, g_out: (B,H,n); k: (H,klen).  g_in / g_out may be NULL (= all ones).
 */
void oracle_causal_conv(const double *u, const double *k, const double *g_in, const double *g_out,
                        double *y, int B, int H, int n, int klen, int nfft, int causal)
{
    int64_t rows = (int64_t)B * H;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t row = 0; row < rows; ++row) {
        int h = (int)(row % H);
        const double *ur = u + (size_t)row * n;
        const double *gi = g_in ? g_in + (size_t)row * n : NULL;
        const double *go = g_out ? g_out + (size_t)row * n : NULL;
        const double *kr = k + (size_t)h * klen;
        double *yr = y + (size_t)row * n;
        for (int t = 0; t < n; ++t) {
            double s = 0.0;
            if (causal) {
                for (int q = 0; q <= t; ++q) {
                    int lag = t - q;
                    if (lag >= klen) continue;
                    double v = gi ? gi[q] * ur[q] : ur[q];
                    s += kr[lag] * v;
                }
            } else {
                for (int q = 0; q < n; ++q) {
                    int lag = (t - q) % nfft;
                    if (lag < 0) lag += nfft;
                    if (lag >= klen) continue;
                    double v = gi ? gi[q] * ur[q] : ur[q];
                    s += kr[lag] * v;
                }
            }
            yr[t] = go ? go[t] * s : s;
        }
    }
}

/*
 * Single outputs of the same sums: y_pts[i] = y[row_i, t_i] with row_i = b*H + h, for sizes at which whole
 * rows take too long (each output is one O(n) sum; same definition, same order of the additions).
 */
void oracle_causal_conv_points(const double *u, const double *k, const double *g_in, const double *g_out,
                               double *y_pts, int B, int H, int n, int klen, int nfft, int causal,
                               const int64_t *rows, const int *ts, int npts)
{
    (void)B;
#pragma omp parallel for schedule(dynamic, 16)
    for (int i = 0; i < npts; ++i) {
        int64_t row = rows[i];
        int t = ts[i];
        int h = (int)(row % H);
        const double *ur = u + (size_t)row * n;
        const double *gi = g_in ? g_in + (size_t)row * n : NULL;
        const double *kr = k + (size_t)h * klen;
        double s = 0.0;
        int last = causal ? t : n - 1;
        for (int q = 0; q <= last; ++q) {
            int lag = t - q;
            if (!causal) {
                lag %= nfft;
                if (lag < 0) lag += nfft;
            }
            if (lag >= klen) continue;
            s += kr[lag] * (gi ? gi[q] * ur[q] : ur[q]);
        }
        y_pts[i] = g_out ? g_out[(size_t)row * n + t] * s : s;
    }
}

/*
 * The same map through the convolution theorem, exactly as the paper states
 * it: y = (F^-1 ((F k') o (F u')))[0:n], k' and u' zero-padded to nfft, with
 * the DFT of this file.  One row (no gates).  Used to pin the identity on
 * small sizes, not as a reference for the GPU.
 */
void oracle_fft_conv_row(const double *u, const double *k, cplx *y_full, int n, int klen, int nfft)
{
    cplx *up = (cplx *)calloc((size_t)nfft, sizeof(cplx));
    cplx *kp = (cplx *)calloc((size_t)nfft, sizeof(cplx));
    cplx *uf = (cplx *)malloc(sizeof(cplx) * (size_t)nfft);
    cplx *kf = (cplx *)malloc(sizeof(cplx) * (size_t)nfft);
    for (int t = 0; t < n; ++t) up[t] = u[t];
    for (int t = 0; t < klen; ++t) kp[t] = k[t];
    oracle_dft(up, uf, 1, nfft);
    oracle_dft(kp, kf, 1, nfft);
    for (int m = 0; m < nfft; ++m) uf[m] *= kf[m];
    oracle_idft(uf, y_full, 1, nfft);
    free(up); free(kp); free(uf); free(kf);
}

/* ------------------------------------------------------------------------- */
/* Monarch MLP  y = W2 * act(W1 * x + b1) + b2   (Sec. 3.2, Eq. 3)            */
/* ------------------------------------------------------------------------- */

static double act_apply(double z, int act)
{
    switch (act) {
    case 1: return z > 0.0 ? z : 0.0;                       /* ReLU */
    case 2: return 0.5 * z * (1.0 + erf(z * 0.70710678118654752440)); /* exact GELU */
    default: return z;
    }
}

/*
 * Dense matrix of one linear layer of the MLP, d_in -> d_out.
 * order 1: W = diag(WR_0 .. WR_{nb-1}), WR: [nb][d_out/nb][d_in/nb], WL unused.
 * order 2: W = P3 L P2 R P1 with nb blocks per factor and width d_mid between
 *          them: R = WR: [nb][d_mid/nb][d_in/nb], L = WL: [nb][d_out/nb][d_mid/nb].
 */
static int mlp_layer_dense(const double *WR, const double *WL, int d_in, int d_out, int d_mid,
                           int nb, int order, double *W)
{
    if (d_in % nb || d_out % nb) return -1;
    if (order == 1) {
        dense_blockdiag(WR, nb, d_out / nb, d_in / nb, W);
        return 0;
    }
    if (order == 2) {
        if (d_mid % nb) return -1;
        return oracle_monarch_dense(WR, WL, nb, d_mid / nb, d_in / nb, nb, d_out / nb, d_mid / nb, W);
    }
    return -1;
}

/* x, y: tokens x d.  b1 (d_hidden) and b2 (d) may be NULL.  act: 0 none, 1 ReLU, 2 GELU(erf). */
int oracle_mlp(const double *x, double *y, int64_t tokens, int d, int d_hidden, int nb, int order,
               const double *W1_R, const double *W1_L, const double *b1,
               const double *W2_R, const double *W2_L, const double *b2,
               int mid1, int mid2, int act)
{
    double *W1 = (double *)malloc(sizeof(double) * (size_t)d_hidden * d);
    double *W2 = (double *)malloc(sizeof(double) * (size_t)d * d_hidden);
    int rc = mlp_layer_dense(W1_R, W1_L, d, d_hidden, mid1, nb, order, W1);
    if (rc == 0) rc = mlp_layer_dense(W2_R, W2_L, d_hidden, d, mid2, nb, order, W2);
    if (rc != 0) { free(W1); free(W2); return rc; }
#pragma omp parallel
    {
        double *hbuf = (double *)malloc(sizeof(double) * (size_t)d_hidden);
#pragma omp for schedule(static)
        for (int64_t t = 0; t < tokens; ++t) {
            const double *xt = x + (size_t)t * d;
            for (int i = 0; i < d_hidden; ++i) {
                double s = b1 ? b1[i] : 0.0;
                for (int j = 0; j < d; ++j) s += W1[(size_t)i * d + j] * xt[j];
                hbuf[i] = act_apply(s, act);
            }
            for (int i = 0; i < d; ++i) {
                double s = b2 ? b2[i] : 0.0;
                for (int j = 0; j < d_hidden; ++j) s += W2[(size_t)i * d_hidden + j] * hbuf[j];
                y[(size_t)t * d + i] = s;
            }
        }
        free(hbuf);
    }
    free(W1); free(W2);
    return 0;
}

/* Number of OpenMP threads the row loops above will use. */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif
