// C-ABI entry points: argument checks first (no device work until they pass), then dispatch.
#include <stdarg.h>
#include <string.h>

#include <mutex>

#include "kernels.h"

namespace monarch {

static thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}
void clear_error() { g_err[0] = 0; }

static bool misaligned(const void *p) { return ((uintptr_t)p & 15u) != 0; }

// Half-open byte ranges [a, a+na) and [b, b+nb) intersect.
static bool overlaps(const void *a, size_t na, const void *b, size_t nb)
{
    if (!a || !b || na == 0 || nb == 0) return false;
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + nb && b0 < a0 + na;
}

// fp16 I/O: the hot-path entry points (matmul, fft / ifft, causal_conv, mlp) take it; the others do not.
static int check_dtype(monarch_dtype dt, bool f16_ok = false)
{
    if (dt == MONARCH_F32 || dt == MONARCH_BF16) return MONARCH_OK;
    if (dt == MONARCH_F16) return f16_ok ? MONARCH_OK : fail(MONARCH_EDTYPE, "this entry point does not take fp16 tensors");
    return fail(MONARCH_EDTYPE, "unknown element type %d", (int)dt);
}

static int check_factors(int N, const int *factors, int nf)
{
    if (!factors) return fail(MONARCH_EINVAL, "factors is NULL");
    if (nf != 2 && nf != 3) return fail(MONARCH_ESHAPE, "nf must be 2 or 3 (got %d)", nf);
    if (N < 4 || N > (1 << 24)) return fail(MONARCH_ESHAPE, "transform length %d outside [4, 2^24]", N);
    int64_t prod = 1;
    for (int i = 0; i < nf; ++i) {
        if (factors[i] < 2) return fail(MONARCH_ESHAPE, "factor %d is %d (< 2)", i, factors[i]);
        prod *= factors[i];
    }
    if (prod != N) return fail(MONARCH_ESHAPE, "factors multiply to %lld, not %d", (long long)prod, N);
    return MONARCH_OK;
}

// Fills the digit geometry of pass q of an nf-factor transform.
static void set_pass_geometry(FftPass &p, int N, const int *factors, int nf, int q)
{
    p.N = N;
    p.nf = nf;
    for (int i = 0; i < 3; ++i) p.factors[i] = i < nf ? factors[i] : 1;
    int O = 1, S = 1;
    for (int i = 0; i < q; ++i) O *= factors[i];
    for (int i = q + 1; i < nf; ++i) S *= factors[i];
    p.O = O;
    p.f = factors[q];
    p.S = S;
}

static FftPass blank_pass()
{
    FftPass p;
    memset(&p, 0, sizeof(p));
    p.scale = 1.0f;
    p.H = 1;
    p.pair_stride = 1;
    return p;
}

}  // namespace monarch

using namespace monarch;

extern "C" {

const char *monarch_strerror(int code)
{
    switch (code) {
    case MONARCH_OK: return "ok";
    case MONARCH_EINVAL: return "invalid argument";
    case MONARCH_ESHAPE: return "unsupported or inconsistent shape";
    case MONARCH_EDTYPE: return "unsupported element type";
    case MONARCH_EWORKSPACE: return "workspace missing or too small";
    case MONARCH_EHIP: return "HIP runtime error";
    default: return "unknown error";
    }
}

const char *monarch_last_error(void) { return g_err; }

int monarch_permutation_index(int b, int N, int32_t *host_out)
{
    clear_error();
    if (!host_out) return fail(MONARCH_EINVAL, "host_out is NULL");
    if (b <= 0 || N <= 0 || N % b != 0) return fail(MONARCH_ESHAPE, "b=%d must be positive and divide N=%d", b, N);
    const int q = N / b;
    for (int i = 0; i < N; ++i) host_out[i] = (i % b) * q + i / b;
    return MONARCH_OK;
}

// ---------------------------------------------------------------------------------------------
// monarch_matmul
// ---------------------------------------------------------------------------------------------

size_t monarch_matmul_workspace_bytes(int64_t, int, int, int, int, int, int, monarch_dtype) { return 0; }

int monarch_matmul(const void *x, const void *R, const void *L, void *y, int64_t batch,
                   int nbR, int r_out, int r_in, int nbL, int l_out, int l_in,
                   monarch_dtype dt, void *ws, size_t ws_bytes, monarch_stream_t stream)
{
    (void)ws; (void)ws_bytes;
    clear_error();
    int rc = check_dtype(dt, true);
    if (rc) return rc;
    if (batch < 0) return fail(MONARCH_ESHAPE, "negative batch");
    if (nbR < 1 || r_out < 1 || r_in < 1 || nbL < 1 || l_out < 1 || l_in < 1)
        return fail(MONARCH_ESHAPE, "all block counts and block sizes must be >= 1");
    if ((int64_t)nbR * r_out != (int64_t)nbL * l_in)
        return fail(MONARCH_ESHAPE, "d_mid mismatch: nbR*r_out=%lld but nbL*l_in=%lld",
                    (long long)nbR * r_out, (long long)nbL * l_in);
    const int64_t d_in = (int64_t)nbR * r_in, d_mid = (int64_t)nbR * r_out, d_out = (int64_t)nbL * l_out;
    if (d_in > 65536 || d_mid > 65536 || d_out > 65536 || !matmul_generic_fits((int)d_in, (int)d_mid, (int)d_out))
        return fail(MONARCH_ESHAPE, "row widths %lld/%lld/%lld exceed the on-chip tile",
                    (long long)d_in, (long long)d_mid, (long long)d_out);
    if (batch == 0) return MONARCH_OK;   // nothing to read or write: empty tensors may be NULL
    if (!x || !R || !L || !y) return fail(MONARCH_EINVAL, "x, R, L and y must be non-NULL");
    if (misaligned(x) || misaligned(R) || misaligned(L) || misaligned(y))
        return fail(MONARCH_EINVAL, "pointers must be 16-byte aligned");
    const size_t es = dtype_size(dt);
    if (overlaps(y, (size_t)batch * d_out * es, x, (size_t)batch * d_in * es))
        return fail(MONARCH_EINVAL, "y overlaps x");
    if (matmul_mfma_b16_supported(nbR, r_out, r_in, nbL, l_out, l_in, dt))
        return launch_matmul_mfma_b16(x, R, L, y, batch, dt, (hipStream_t)stream);
    if (nbR == r_out && nbR == r_in && nbR == nbL && nbR == l_out && nbR == l_in && monarch_inplace_supported(nbR, dt))
        return launch_matmul_inplace(x, R, L, y, batch, nbR, dt, (hipStream_t)stream);   // square, blocks of 32 or 64
    return launch_matmul_generic(x, R, L, nullptr, y, batch, nbR, r_out, r_in, nbL, l_out, l_in, 2, 0,
                                 dt, dt, dt, (hipStream_t)stream);
}

size_t monarch_matmul_backward_workspace_bytes(int64_t, int, int, int, int, int, int, monarch_dtype) { return 0; }

int monarch_matmul_backward(const void *x, const void *R, const void *L, const void *dy,
                            void *dx, float *dR, float *dL, int64_t batch,
                            int nbR, int r_out, int r_in, int nbL, int l_out, int l_in,
                            monarch_dtype dt, void *ws, size_t ws_bytes, monarch_stream_t stream)
{
    (void)ws; (void)ws_bytes;
    clear_error();
    int rc = check_dtype(dt);
    if (rc) return rc;
    if (batch < 0) return fail(MONARCH_ESHAPE, "negative batch");
    if (nbR < 1 || r_out < 1 || r_in < 1 || nbL < 1 || l_out < 1 || l_in < 1)
        return fail(MONARCH_ESHAPE, "all block counts and block sizes must be >= 1");
    if ((int64_t)nbR * r_out != (int64_t)nbL * l_in)
        return fail(MONARCH_ESHAPE, "d_mid mismatch: nbR*r_out=%lld but nbL*l_in=%lld",
                    (long long)nbR * r_out, (long long)nbL * l_in);
    const int64_t d_in = (int64_t)nbR * r_in, d_mid = (int64_t)nbR * r_out, d_out = (int64_t)nbL * l_out;
    if (d_in > 65536 || d_mid > 65536 || d_out > 65536 || !matmul_backward_fits(nbR, r_out, r_in, nbL, l_out, l_in))
        return fail(MONARCH_ESHAPE, "row widths %lld/%lld/%lld exceed the on-chip tile",
                    (long long)d_in, (long long)d_mid, (long long)d_out);
    if (!dx && !dR && !dL) return MONARCH_OK;
    const size_t es = dtype_size(dt);
    const size_t nR = (size_t)nbR * r_out * r_in, nL = (size_t)nbL * l_out * l_in;
    if ((dR || dL) && (!R || !L)) return fail(MONARCH_EINVAL, "R and L must be non-NULL");
    if (misaligned(x) || misaligned(R) || misaligned(L) || misaligned(dy) || misaligned(dx) || misaligned(dR) || misaligned(dL))
        return fail(MONARCH_EINVAL, "pointers must be 16-byte aligned");
    if (batch > 0) {
        if (!x || !R || !L || !dy) return fail(MONARCH_EINVAL, "x, R, L and dy must be non-NULL");
        const void *ins[4] = {x, dy, R, L};
        const size_t in_bytes[4] = {(size_t)batch * d_in * es, (size_t)batch * d_out * es, nR * es, nL * es};
        const void *outs[3] = {dx, dR, dL};
        const size_t out_bytes[3] = {(size_t)batch * d_in * es, nR * sizeof(float), nL * sizeof(float)};
        for (int o = 0; o < 3; ++o) {
            if (!outs[o]) continue;
            for (int i = 0; i < 4; ++i)
                if (overlaps(outs[o], out_bytes[o], ins[i], in_bytes[i])) return fail(MONARCH_EINVAL, "an output overlaps an input");
            for (int q = o + 1; q < 3; ++q)
                if (outs[q] && overlaps(outs[o], out_bytes[o], outs[q], out_bytes[q])) return fail(MONARCH_EINVAL, "outputs overlap");
        }
    }
    // (batch == 0: the parameter gradients are zero; the launcher clears them and runs no tile)
    return launch_matmul_backward(x, R, L, dy, dx, dR, dL, batch, nbR, r_out, r_in, nbL, l_out, l_in, dt,
                                  (hipStream_t)stream);
}

// ---------------------------------------------------------------------------------------------
// monarch_matmulp / monarch_matmulp_backward
// ---------------------------------------------------------------------------------------------

static int check_matmulp(int64_t batch, int b, int p, bool backward, monarch_dtype dt, int *N)
{
    int rc = check_dtype(dt);
    if (rc) return rc;
    if (batch < 0) return fail(MONARCH_ESHAPE, "negative batch");
    *N = matmulp_length(b, p, backward);
    if (!*N)
        return fail(MONARCH_ESHAPE, "order p = %d with blocks of %d: 2 <= p <= 12, 2 <= b <= 16, b^p <= 4096 required", p, b);
    return MONARCH_OK;
}

int monarch_matmulp(const void *x, const void *B, void *y, int64_t batch, int b, int p, monarch_dtype dt, monarch_stream_t stream)
{
    clear_error();
    int N = 0;
    int rc = check_matmulp(batch, b, p, false, dt, &N);
    if (rc) return rc;
    if (batch == 0) return MONARCH_OK;
    if (!x || !B || !y) return fail(MONARCH_EINVAL, "x, B and y must be non-NULL");
    if (misaligned(x) || misaligned(B) || misaligned(y)) return fail(MONARCH_EINVAL, "pointers must be 16-byte aligned");
    const size_t es = dtype_size(dt), act = (size_t)batch * N * es, wb = (size_t)p * N * b * es;
    if (overlaps(y, act, x, act) || overlaps(y, act, B, wb)) return fail(MONARCH_EINVAL, "y overlaps an input");
    return launch_matmulp(x, B, y, batch, b, p, dt, (hipStream_t)stream);
}

int monarch_matmulp_backward(const void *x, const void *B, const void *dy, void *dx, float *dB, int64_t batch, int b, int p,
                             monarch_dtype dt, monarch_stream_t stream)
{
    clear_error();
    int N = 0;
    int rc = check_matmulp(batch, b, p, true, dt, &N);
    if (rc) return rc;
    if (!dx && !dB) return MONARCH_OK;
    if (misaligned(x) || misaligned(B) || misaligned(dy) || misaligned(dx) || misaligned(dB))
        return fail(MONARCH_EINVAL, "pointers must be 16-byte aligned");
    const size_t es = dtype_size(dt), act = (size_t)batch * N * es, wn = (size_t)p * N * b;
    if (batch > 0) {
        if (!x || !B || !dy) return fail(MONARCH_EINVAL, "x, B and dy must be non-NULL");
        const void *ins[3] = {x, dy, B};
        const size_t in_bytes[3] = {act, act, wn * es};
        const void *outs[2] = {dx, dB};
        const size_t out_bytes[2] = {act, wn * sizeof(float)};
        for (int o = 0; o < 2; ++o) {
            if (!outs[o]) continue;
            for (int i = 0; i < 3; ++i)
                if (overlaps(outs[o], out_bytes[o], ins[i], in_bytes[i])) return fail(MONARCH_EINVAL, "an output overlaps an input");
        }
        if (dx && dB && overlaps(dx, act, dB, wn * sizeof(float))) return fail(MONARCH_EINVAL, "outputs overlap");
    }
    return launch_matmulp_backward(x, B, dy, dx, dB, batch, b, p, dt, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------------------------
// monarch_matmul3 / monarch_matmul3_backward
// ---------------------------------------------------------------------------------------------

static int check_matmul3(int64_t batch, int b, monarch_dtype dt)
{
    int rc = check_dtype(dt);
    if (rc) return rc;
    if (batch < 0) return fail(MONARCH_ESHAPE, "negative batch");
    if (!matmul3_fits(b)) return fail(MONARCH_ESHAPE, "block size %d outside [1, 16] (four rows of b^3 floats must fit in LDS)", b);
    return MONARCH_OK;
}

int monarch_matmul3(const void *x, const void *B1, const void *B2, const void *B3, void *y, int64_t batch, int b,
                    monarch_dtype dt, monarch_stream_t stream)
{
    clear_error();
    int rc = check_matmul3(batch, b, dt);
    if (rc) return rc;
    if (batch == 0) return MONARCH_OK;
    if (!x || !B1 || !B2 || !B3 || !y) return fail(MONARCH_EINVAL, "x, B1, B2, B3 and y must be non-NULL");
    if (misaligned(x) || misaligned(B1) || misaligned(B2) || misaligned(B3) || misaligned(y))
        return fail(MONARCH_EINVAL, "pointers must be 16-byte aligned");
    const size_t es = dtype_size(dt), N = (size_t)b * b * b, act = (size_t)batch * N * es, wb = N * b * es;
    if (overlaps(y, act, x, act) || overlaps(y, act, B1, wb) || overlaps(y, act, B2, wb) || overlaps(y, act, B3, wb))
        return fail(MONARCH_EINVAL, "y overlaps an input");
    return launch_matmul3(x, B1, B2, B3, y, batch, b, dt, (hipStream_t)stream);
}

int monarch_matmul3_backward(const void *x, const void *B1, const void *B2, const void *B3, const void *dy, void *dx,
                             float *dB1, float *dB2, float *dB3, int64_t batch, int b, monarch_dtype dt,
                             monarch_stream_t stream)
{
    clear_error();
    int rc = check_matmul3(batch, b, dt);
    if (rc) return rc;
    if (!dx && !dB1 && !dB2 && !dB3) return MONARCH_OK;
    if (misaligned(x) || misaligned(B1) || misaligned(B2) || misaligned(B3) || misaligned(dy) || misaligned(dx) ||
        misaligned(dB1) || misaligned(dB2) || misaligned(dB3))
        return fail(MONARCH_EINVAL, "pointers must be 16-byte aligned");
    const size_t es = dtype_size(dt), N = (size_t)b * b * b, act = (size_t)batch * N * es, wn = N * b;
    if (batch > 0) {
        if (!x || !B1 || !B2 || !B3 || !dy) return fail(MONARCH_EINVAL, "x, B1, B2, B3 and dy must be non-NULL");
        const void *ins[5] = {x, dy, B1, B2, B3};
        const size_t in_bytes[5] = {act, act, wn * es, wn * es, wn * es};
        const void *outs[4] = {dx, dB1, dB2, dB3};
        const size_t out_bytes[4] = {act, wn * sizeof(float), wn * sizeof(float), wn * sizeof(float)};
        for (int o = 0; o < 4; ++o) {
            if (!outs[o]) continue;
            for (int i = 0; i < 5; ++i)
                if (overlaps(outs[o], out_bytes[o], ins[i], in_bytes[i])) return fail(MONARCH_EINVAL, "an output overlaps an input");
            for (int q = o + 1; q < 4; ++q)
                if (outs[q] && overlaps(outs[o], out_bytes[o], outs[q], out_bytes[q])) return fail(MONARCH_EINVAL, "outputs overlap");
        }
    }
    return launch_matmul3_backward(x, B1, B2, B3, dy, dx, dB1, dB2, dB3, batch, b, dt, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------------------------
// monarch_mixer
// ---------------------------------------------------------------------------------------------

size_t monarch_mixer_workspace_bytes(int64_t, int, int, monarch_dtype) { return 0; }

int monarch_mixer(const void *u, const void *K, const void *g_in, const void *g_out,
                  const void *R1, const void *L1, const void *R2, const void *L2, void *y,
                  int64_t B, int H, int bs, monarch_dtype dt, void *ws, size_t ws_bytes, monarch_stream_t stream)
{
    (void)ws; (void)ws_bytes;
    clear_error();
    int rc = check_dtype(dt);
    if (rc) return rc;
    if (B < 0 || H < 1) return fail(MONARCH_ESHAPE, "B must be >= 0 and H >= 1");
    if (bs < 1 || !mixer_fits(bs)) return fail(MONARCH_ESHAPE, "block size %d: a row of bs^2 elements must fit in LDS twice", bs);
    if (B > INT64_MAX / H) return fail(MONARCH_ESHAPE, "B * H overflows");
    const int64_t rows = B * H, N = (int64_t)bs * bs;
    if (rows == 0) return MONARCH_OK;
    if (!u || !K || !R1 || !L1 || !R2 || !L2 || !y) return fail(MONARCH_EINVAL, "u, K, R1, L1, R2, L2 and y must be non-NULL");
    if (misaligned(u) || misaligned(K) || misaligned(g_in) || misaligned(g_out) || misaligned(R1) || misaligned(L1) ||
        misaligned(R2) || misaligned(L2) || misaligned(y))
        return fail(MONARCH_EINVAL, "pointers must be 16-byte aligned");
    const size_t es = dtype_size(dt), act = (size_t)rows * N * es, wb = (size_t)N * bs * es;
    const void *ins[8] = {u, g_in, g_out, K, R1, L1, R2, L2};
    const size_t in_bytes[8] = {act, act, act, (size_t)H * N * es, wb, wb, wb, wb};
    for (int i = 0; i < 8; ++i)
        if (ins[i] && overlaps(y, act, ins[i], in_bytes[i])) return fail(MONARCH_EINVAL, "y overlaps an input");
    return launch_mixer(u, K, g_in, g_out, R1, L1, R2, L2, y, rows, H, bs, dt, MixOpt(), (hipStream_t)stream);
}

// ---------------------------------------------------------------------------------------------
// monarch_mixer_backward
// ---------------------------------------------------------------------------------------------

size_t monarch_mixer_backward_workspace_bytes(int64_t B, int H, int bs, monarch_dtype dt)
{
    if (B <= 0 || H <= 0 || bs <= 0 || (dt != MONARCH_F32 && dt != MONARCH_BF16)) return 0;
    return mixer_backward_workspace_bytes(B, H, bs, dt);
}

int monarch_mixer_backward(const void *u, const void *K, const void *g_in, const void *g_out,
                           const void *R1, const void *L1, const void *R2, const void *L2, const void *dy,
                           void *du, float *dK, void *dg_in, void *dg_out,
                           float *dR1, float *dL1, float *dR2, float *dL2,
                           int64_t B, int H, int bs, monarch_dtype dt, void *ws, size_t ws_bytes, monarch_stream_t stream)
{
    clear_error();
    int rc = check_dtype(dt);
    if (rc) return rc;
    if (B < 0 || H < 1) return fail(MONARCH_ESHAPE, "B must be >= 0 and H >= 1");
    if (bs < 1 || !mixer_fits(bs) || !matmul_backward_fits(bs, bs, bs, bs, bs, bs) || !matmul_generic_fits(bs * bs, bs * bs, bs * bs))
        return fail(MONARCH_ESHAPE, "block size %d: rows of bs^2 elements exceed the on-chip tiles", bs);
    if (B > INT64_MAX / H) return fail(MONARCH_ESHAPE, "B * H overflows");
    if ((dg_in && !g_in) || (dg_out && !g_out)) return fail(MONARCH_EINVAL, "a gate's gradient was asked for without the gate");
    const void *all[18] = {u, K, g_in, g_out, R1, L1, R2, L2, dy, du, dK, dg_in, dg_out, dR1, dL1, dR2, dL2, ws};
    for (int i = 0; i < 18; ++i)
        if (misaligned(all[i])) return fail(MONARCH_EINVAL, "pointers must be 16-byte aligned");
    const int64_t rows = B * H;
    const size_t es = dtype_size(dt), N = (size_t)bs * bs, act = (size_t)rows * N * es, wb = N * bs * es;
    const size_t need = rows > 0 ? mixer_backward_workspace_bytes(B, H, bs, dt) : 0;
    if (rows > 0) {
        if (!u || !K || !R1 || !L1 || !R2 || !L2 || !dy) return fail(MONARCH_EINVAL, "u, K, the four factors and dy must be non-NULL");
        if (!ws || ws_bytes < need) return fail(MONARCH_EWORKSPACE, "workspace of %zu bytes needed, %zu given", need, ws ? ws_bytes : (size_t)0);
    }
    const void *ins[9] = {u, g_in, g_out, dy, K, R1, L1, R2, L2};
    const size_t in_bytes[9] = {act, act, act, act, (size_t)H * N * es, wb, wb, wb, wb};
    const void *outs[9] = {du, dg_in, dg_out, dK, dR1, dL1, dR2, dL2, rows > 0 ? ws : nullptr};
    const size_t out_bytes[9] = {act, act, act, (size_t)H * N * 4, N * bs * 4, N * bs * 4, N * bs * 4, N * bs * 4, need};
    for (int o = 0; o < 9; ++o) {
        if (!outs[o]) continue;
        for (int i = 0; i < 9; ++i)
            if (ins[i] && rows > 0 && overlaps(outs[o], out_bytes[o], ins[i], in_bytes[i]))
                return fail(MONARCH_EINVAL, "an output or the workspace overlaps an input");
        for (int q = o + 1; q < 9; ++q)
            if (outs[q] && overlaps(outs[o], out_bytes[o], outs[q], out_bytes[q])) return fail(MONARCH_EINVAL, "outputs overlap");
    }
    return launch_mixer_backward(u, K, g_in, g_out, R1, L1, R2, L2, dy, du, dK, dg_in, dg_out, dR1, dL1, dR2, dL2, B, H, bs, dt,
                                 ws, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------------------------
// monarch_m2_layer
// ---------------------------------------------------------------------------------------------

size_t monarch_m2_layer_workspace_bytes(int64_t B, int n, int d, monarch_dtype dt)
{
    if (B <= 0 || n <= 0 || d <= 0 || (dt != MONARCH_F32 && dt != MONARCH_BF16)) return 0;
    return align_up((size_t)B * n * d * dtype_size(dt), 256);
}

int monarch_m2_layer(const void *x, void *y, int64_t B, int bn, int bd,
                     const void *R1, const void *L1, const void *R2, const void *L2, const void *n_kernel,
                     const void *R3, const void *L3, const void *R4, const void *L4, const void *d_kernel,
                     const void *ln_gamma, const void *ln_beta, float eps, int act,
                     monarch_dtype dt, void *ws, size_t ws_bytes, monarch_stream_t stream)
{
    clear_error();
    int rc = check_dtype(dt);
    if (rc) return rc;
    if (B < 0) return fail(MONARCH_ESHAPE, "negative batch");
    if (bn < 1 || bd < 1 || !mixer_fits(bn) || !mixer_fits(bd))
        return fail(MONARCH_ESHAPE, "block sizes %d, %d: a row of bs^2 elements must fit in LDS twice", bn, bd);
    if (act != 0 && act != 1) return fail(MONARCH_EINVAL, "activation must be 0 (none) or 1 (ReLU)");
    if (!(eps >= 0.0f)) return fail(MONARCH_EINVAL, "eps must be >= 0");
    if (B == 0) return MONARCH_OK;
    const int n = bn * bn, d = bd * bd;
    if (B > INT64_MAX / ((int64_t)n * d)) return fail(MONARCH_ESHAPE, "B * n * d overflows");
    const void *req[15] = {x, y, R1, L1, R2, L2, n_kernel, R3, L3, R4, L4, d_kernel, ln_gamma, ln_beta, ws};
    for (int i = 0; i < 15; ++i) {
        if (!req[i]) return fail(MONARCH_EINVAL, "every pointer argument must be non-NULL");
        if (misaligned(req[i])) return fail(MONARCH_EINVAL, "pointers must be 16-byte aligned");
    }
    const size_t need = monarch_m2_layer_workspace_bytes(B, n, d, dt);
    if (ws_bytes < need) return fail(MONARCH_EWORKSPACE, "workspace of %zu bytes needed, %zu given", need, ws_bytes);
    const size_t act_bytes = (size_t)B * n * d * dtype_size(dt);
    if (overlaps(y, act_bytes, x, act_bytes) || overlaps(ws, need, x, act_bytes) || overlaps(ws, need, y, act_bytes))
        return fail(MONARCH_EINVAL, "x, y and the workspace must not overlap");
    // sequence mixer: rows (b, feature), positions along the row; reads x and writes X~ in (B, n, d) order
    MixOpt seq;
    seq.act = act;
    seq.transposed = 1;
    rc = launch_mixer(x, n_kernel, nullptr, nullptr, R1, L1, R2, L2, ws, B * d, d, bn, dt, seq, (hipStream_t)stream);
    if (rc) return rc;
    // dimension mixer: rows (b, position), one kernel row for all of them; skip connection and layer norm fused
    MixOpt dim;
    dim.act = act;
    dim.layer_norm = 1;
    dim.gamma = ln_gamma;
    dim.beta = ln_beta;
    dim.eps = eps;
    return launch_mixer(ws, d_kernel, nullptr, nullptr, R3, L3, R4, L4, y, B * n, 1, bd, dt, dim, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------------------------
// monarch_hyena_layer
// ---------------------------------------------------------------------------------------------
static int conv_check(int B, int H, int n, int klen, int nfft, const int *factors, int nf, int causal, monarch_dtype dt);

static bool heads_ok(int B, int d, int head_dim)
{
    return head_dim >= 1 && head_dim <= 64 && d % head_dim == 0 && (int64_t)B * head_dim * head_dim <= INT32_MAX;
}

size_t monarch_hyena_heads_layer_workspace_bytes(int B, int n, int d, int klen, int nfft, const int *factors, int nf, int head_dim,
                                                 monarch_dtype dt)
{
    if (B <= 0 || n <= 0 || d <= 0 || !heads_ok(B, d, head_dim)) return 0;
    return hyena_layer_workspace_bytes(B, n, d, klen, nfft, factors, nf, head_dim, dt);
}

size_t monarch_hyena_layer_workspace_bytes(int B, int n, int d, int klen, int nfft, const int *factors, int nf, monarch_dtype dt)
{
    return monarch_hyena_heads_layer_workspace_bytes(B, n, d, klen, nfft, factors, nf, 1, dt);
}

int monarch_hyena_heads_layer(const void *u, const void *W_in, const void *b_in, const void *k_short, const void *k_long,
                              const void *W_out, const void *b_out, void *y, int B, int n, int d, int taps, int klen, int nfft,
                              const int *factors, int nf, int causal, int head_dim, monarch_dtype dt, void *ws, size_t ws_bytes,
                              monarch_stream_t stream)
{
    clear_error();
    int rc = check_dtype(dt);
    if (rc) return rc;
    if (B < 0 || n < 1 || d < 1) return fail(MONARCH_ESHAPE, "B >= 0, n >= 1, d >= 1 required");
    if (n % 8) return fail(MONARCH_ESHAPE, "the sequence length must be a multiple of 8");
    if (taps < 1 || taps > 8) return fail(MONARCH_ESHAPE, "short kernels of 1 to 8 taps");
    if (!heads_ok(B, d, head_dim))
        return fail(MONARCH_ESHAPE, "the head dimension must lie in [1, 64] and divide d = %d (given %d), B head_dim^2 below 2^31", d,
                    head_dim);
    if ((int64_t)B * d * n * head_dim > (int64_t)1 << 40 || (int64_t)3 * B * d > INT32_MAX) return fail(MONARCH_ESHAPE, "tensor too large");
    if (B == 0) return MONARCH_OK;
    const void *req[7] = {u, W_in, k_short, k_long, W_out, y, ws};
    for (int i = 0; i < 7; ++i)
        if (!req[i]) return fail(MONARCH_EINVAL, "u, W_in, k_short, k_long, W_out, y and ws must be non-NULL");
    const void *all[9] = {u, W_in, b_in, k_short, k_long, W_out, b_out, y, ws};
    for (int i = 0; i < 9; ++i)
        if (misaligned(all[i])) return fail(MONARCH_EINVAL, "pointers must be 16-byte aligned");
    const size_t need = monarch_hyena_heads_layer_workspace_bytes(B, n, d, klen, nfft, factors, nf, head_dim, dt);
    if (ws_bytes < need) return fail(MONARCH_EWORKSPACE, "workspace of %zu bytes needed, %zu given", need, ws_bytes);
    const size_t act = (size_t)B * n * d * dtype_size(dt);
    if (overlaps(y, act, u, act) || overlaps(ws, need, u, act) || overlaps(ws, need, y, act))
        return fail(MONARCH_EINVAL, "u, y and the workspace must not overlap");
    // the checks of the long convolution (nfft against n and klen, the factor list) before any device work
    rc = conv_check(B * head_dim * head_dim, d / head_dim, n, klen, nfft, factors, nf, causal, dt);
    if (rc) return rc;
    return launch_hyena_layer(u, W_in, b_in, k_short, k_long, W_out, b_out, y, B, n, d, taps, klen, nfft, factors, nf, causal, head_dim,
                              dt, ws, ws_bytes, (hipStream_t)stream);
}

int monarch_hyena_layer(const void *u, const void *W_in, const void *b_in, const void *k_short, const void *k_long,
                        const void *W_out, const void *b_out, void *y, int B, int n, int d, int taps, int klen, int nfft,
                        const int *factors, int nf, int causal, monarch_dtype dt, void *ws, size_t ws_bytes,
                        monarch_stream_t stream)
{
    return monarch_hyena_heads_layer(u, W_in, b_in, k_short, k_long, W_out, b_out, y, B, n, d, taps, klen, nfft, factors, nf, causal, 1,
                                     dt, ws, ws_bytes, stream);
}

// ---------------------------------------------------------------------------------------------
// monarch_blocky_prepare / monarch_blocky_conv
// ---------------------------------------------------------------------------------------------

size_t monarch_blocky_state_bytes(int H, int bs)
{
    if (H < 0 || !blocky_fits(bs)) return 0;
    return blocky_state_bytes(H, bs);
}

int monarch_blocky_state_offsets(int H, int bs, size_t *host_out)
{
    clear_error();
    if (H < 0 || !blocky_fits(bs)) return fail(MONARCH_ESHAPE, "H must be >= 0 and the block size in [2, 64]");
    if (!host_out) return fail(MONARCH_EINVAL, "host_out must be non-NULL");
    blocky_state_offsets(H, bs, host_out);
    return MONARCH_OK;
}

int monarch_blocky_prepare(const float *Lt, const float *Rt, const float *k, int H, int klen, int bs, int mask,
                           void *state, size_t state_bytes, monarch_stream_t stream)
{
    clear_error();
    if (!blocky_fits(bs)) return fail(MONARCH_ESHAPE, "block size %d outside [2, 64]", bs);
    const int N = bs * bs;
    if (H < 0 || klen < 0 || klen > N) return fail(MONARCH_ESHAPE, "H must be >= 0 and klen in [0, N = %d]", N);
    if (mask != 0 && mask != 1) return fail(MONARCH_EINVAL, "mask flag must be 0 or 1");
    if (mask && klen > bs * (bs / 2))
        return fail(MONARCH_ESHAPE, "with the causal mask the kernel may have at most bs * floor(bs / 2) = %d taps", bs * (bs / 2));
    if (!Lt || !Rt || !state || (H > 0 && klen > 0 && !k)) return fail(MONARCH_EINVAL, "Lt, Rt, k and state must be non-NULL");
    if (misaligned(Lt) || misaligned(Rt) || misaligned(k) || misaligned(state)) return fail(MONARCH_EINVAL, "pointers must be 16-byte aligned");
    const size_t need = blocky_state_bytes(H, bs);
    if (state_bytes < need) return fail(MONARCH_EWORKSPACE, "state of %zu bytes needed, %zu given", need, state_bytes);
    const size_t coeff = (size_t)N * bs * sizeof(float);
    if (overlaps(state, need, Lt, coeff) || overlaps(state, need, Rt, coeff) ||
        (k && overlaps(state, need, k, (size_t)H * klen * sizeof(float))))
        return fail(MONARCH_EINVAL, "state overlaps an input");
    return launch_blocky_prepare(Lt, Rt, k, H, klen, bs, mask, state, (hipStream_t)stream);
}

int monarch_blocky_conv(const void *u, const void *g_in, const void *g_out, const void *state, size_t state_bytes,
                        void *y, int64_t B, int H, int n, int bs, monarch_dtype dt, monarch_stream_t stream)
{
    clear_error();
    int rc = check_dtype(dt);
    if (rc) return rc;
    if (!blocky_fits(bs)) return fail(MONARCH_ESHAPE, "block size %d outside [2, 64]", bs);
    if (B < 0 || H < 1 || n < 0 || n > bs * bs) return fail(MONARCH_ESHAPE, "B >= 0, H >= 1 and n in [0, bs^2] required");
    if (B > INT64_MAX / H) return fail(MONARCH_ESHAPE, "B * H overflows");
    const int64_t rows = B * H;
    if (rows == 0 || n == 0) return MONARCH_OK;
    if (!u || !y || !state) return fail(MONARCH_EINVAL, "u, y and state must be non-NULL");
    if (misaligned(u) || misaligned(g_in) || misaligned(g_out) || misaligned(y) || misaligned(state))
        return fail(MONARCH_EINVAL, "pointers must be 16-byte aligned");
    const size_t need = blocky_state_bytes(H, bs);
    if (state_bytes < need) return fail(MONARCH_EWORKSPACE, "state of %zu bytes needed, %zu given", need, state_bytes);
    const size_t act = (size_t)rows * n * dtype_size(dt);
    if (overlaps(y, act, u, act) || (g_in && overlaps(y, act, g_in, act)) || (g_out && overlaps(y, act, g_out, act)) ||
        overlaps(y, act, state, need))
        return fail(MONARCH_EINVAL, "y overlaps an input");
    return launch_blocky_conv(u, g_in, g_out, state, y, rows, H, n, bs, dt, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------------------------
// monarch_fft / monarch_ifft
// ---------------------------------------------------------------------------------------------

size_t monarch_fft_workspace_bytes(int64_t rows, int N, const int *factors, int nf, monarch_dtype dt)
{
    if (rows <= 0 || N <= 0) return 0;
    if (nf == 2 && factors && fft2_lds_supported(factors[0], factors[1], dt)) return 0;   // one kernel, rows stay on chip
    const size_t buf = align_up((size_t)rows * N * sizeof(float2), 256);
    return nf >= 3 ? 2 * buf : buf;
}

static int fft_common(const void *src, void *dst, int64_t rows, int N, const int *factors, int nf,
                      int is_real, int inverse, monarch_dtype dt, void *ws, size_t ws_bytes,
                      hipStream_t s)
{
    int rc = check_dtype(dt, true);
    if (rc) return rc;
    rc = check_factors(N, factors, nf);
    if (rc) return rc;
    if (rows < 0) return fail(MONARCH_ESHAPE, "negative rows");
    if (is_real != 0 && is_real != 1) return fail(MONARCH_EINVAL, "real flag must be 0 or 1");
    if (rows == 0) return MONARCH_OK;
    if (!src || !dst) return fail(MONARCH_EINVAL, "input and output must be non-NULL");
    if (misaligned(src) || misaligned(dst) || misaligned(ws)) return fail(MONARCH_EINVAL, "pointers must be 16-byte aligned");
    const size_t need = monarch_fft_workspace_bytes(rows, N, factors, nf, dt);
    if (need && (!ws || ws_bytes < need))
        return fail(MONARCH_EWORKSPACE, "workspace of %zu bytes needed, %zu given", need, ws ? ws_bytes : (size_t)0);
    const size_t spec_bytes = (size_t)rows * N * sizeof(float2);
    const size_t typed_bytes = (size_t)rows * N * dtype_size(dt) * (is_real ? 1 : 2);
    if (overlaps(src, inverse ? spec_bytes : typed_bytes, dst, inverse ? typed_bytes : spec_bytes))
        return fail(MONARCH_EINVAL, "output overlaps input");

    // bf16 rows, two factors that fit an LDS-resident chunk: the whole transform in one kernel, the row read once
    // and the spectrum written once (forward) or the other way round.  (Complex bf16 rows are interleaved pairs:
    // the packed form the kernel keeps its tile in.)
    if (nf == 2 && fft2_lds_supported(factors[0], factors[1], dt)) {
        Fft2Args a;
        a.in = src;
        a.out = dst;
        a.gate = a.gate_out = a.kf = nullptr;
        a.rows = rows;
        a.N = N;
        a.O = 1;
        a.f1 = factors[0];
        a.f2 = factors[1];
        a.n_valid = N;
        a.H = 1;
        a.pair_stride = 1;
        a.real_rows = rows;
        a.scale = 1.0f / (float)N;
        a.load = inverse ? LD_C32_CONJ : is_real ? LD_REAL : LD_C16;
        a.store = !inverse ? ST_C32_NATURAL : is_real ? ST_REAL_SCALE_GATE : ST_CPLX_CONJ_SCALE;
        a.inverse = inverse;
        a.tw_outer = 0;
        return launch_fft2_lds(a, s);
    }

    const size_t buf = align_up(spec_bytes, 256);
    void *bufs[2] = {ws, (char *)ws + buf};
    const void *cur = src;
    // bf16 transforms with MFMA-sized factors run on the matrix cores and keep the rows packed as
    // bf16 pairs between passes; everything else takes the fp32 passes.
    const bool mf = fft_mfma_supported(N, factors, nf, dt);
    const bool mf32 = fft_mfma_f32_supported(N, factors, nf, dt);   // fp32 MFMA, rows stay complex fp32
    for (int q = 0; q < nf; ++q) {
        FftPass p = blank_pass();
        set_pass_geometry(p, N, factors, nf, q);
        p.rows = rows;
        p.dt = dt;
        p.n_valid = N;
        p.in = cur;
        if (q == 0)
            p.load = inverse ? LD_C32_CONJ : (is_real ? LD_REAL : LD_CPLX);
        else
            p.load = mf ? LD_C16 : LD_C32;
        if (q == nf - 1) {
            p.out = dst;
            if (!inverse) p.store = ST_C32_NATURAL;
            else {
                p.store = is_real ? ST_REAL_SCALE_GATE : ST_CPLX_CONJ_SCALE;
                p.scale = 1.0f / (float)N;
            }
        } else {
            p.out = bufs[q & 1];
            p.store = mf ? ST_C16 : ST_C32;
        }
        rc = mf ? launch_fft_pass_mfma(p, s) : mf32 ? launch_fft_pass_mfma_f32(p, s) : launch_fft_pass(p, s);
        if (rc) return rc;
        cur = p.out;
    }
    return MONARCH_OK;
}

int monarch_fft(const void *x, void *X, int64_t rows, int N, const int *factors, int nf,
                int real_input, monarch_dtype dt, void *ws, size_t ws_bytes, monarch_stream_t stream)
{
    clear_error();
    return fft_common(x, X, rows, N, factors, nf, real_input, 0, dt, ws, ws_bytes, (hipStream_t)stream);
}

int monarch_ifft(const void *X, void *x, int64_t rows, int N, const int *factors, int nf,
                 int real_output, monarch_dtype dt, void *ws, size_t ws_bytes, monarch_stream_t stream)
{
    clear_error();
    return fft_common(X, x, rows, N, factors, nf, real_output, 1, dt, ws, ws_bytes, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------------------------
// monarch_causal_conv
// ---------------------------------------------------------------------------------------------

static int conv_check(int B, int H, int n, int klen, int nfft, const int *factors, int nf, int causal,
                      monarch_dtype dt)
{
    int rc = check_dtype(dt, true);
    if (rc) return rc;
    rc = check_factors(nfft, factors, nf);
    if (rc) return rc;
    if (B < 0 || H < 0) return fail(MONARCH_ESHAPE, "negative B or H");
    if (n < 1 || klen < 1) return fail(MONARCH_ESHAPE, "n and klen must be >= 1");
    if (causal != 0 && causal != 1) return fail(MONARCH_EINVAL, "causal must be 0 or 1");
    if (n > nfft) return fail(MONARCH_ESHAPE, "n=%d exceeds nfft=%d", n, nfft);
    if (causal) {
        if (klen > n) return fail(MONARCH_ESHAPE, "causal kernel longer than the sequence (klen=%d, n=%d)", klen, n);
        if ((int64_t)n + klen - 1 > nfft)
            return fail(MONARCH_ESHAPE, "nfft=%d < n+klen-1=%d: the circular convolution would wrap", nfft, n + klen - 1);
    } else if (klen > nfft) {
        return fail(MONARCH_ESHAPE, "klen=%d exceeds nfft=%d", klen, nfft);
    }
    return MONARCH_OK;
}

// Which fused kernel serves this shape: 0 = none (multi-pass path), 1 = 64 x 32 MFMA, 2 = 16 x 16 MFMA,
// 3 = 128 x 128 MFMA, 4 = 64 x 32 fp32 MFMA.
// With n, klen <= nfft/2 the circular and the causal form coincide, so `causal` does not matter.
static int conv_fused_path(int n, int klen, const int *factors, int nf, monarch_dtype dt)
{
    if (factors && conv_mfma_2048_supported(n, klen, factors, nf, dt)) return 1;
    if (factors && conv_mfma_256_supported(n, klen, factors, nf, dt)) return 2;
    if (factors && conv_mfma_16k_supported(n, klen, factors, nf, dt)) return 3;
    if (factors && conv_f32_2048_supported(n, klen, factors, nf, dt)) return 4;
    return 0;
}

size_t monarch_causal_conv_workspace_bytes(int B, int H, int n, int klen, int nfft,
                                           const int *factors, int nf, monarch_dtype dt)
{
    if (B <= 0 || H <= 0 || nfft <= 0) return 0;
    if (conv_fused_path(n, klen, factors, nf, dt)) return 0;   // fused kernels keep everything on chip
    const size_t rows = (size_t)B * H;
    const size_t buf = align_up(rows * nfft * sizeof(float2), 256);
    const size_t kf = align_up((size_t)H * nfft * sizeof(float2), 256);
    return 2 * buf + kf;
}

// Convolution with the last two factors of every transform done in one kernel on LDS-resident chunks (bf16).
// Two factors: three launches (spectrum of k, spectrum of the paired rows, inverse), no strided pass.
// Three factors: the first factor is a strided pass before the chunk kernel (forward) and after it (inverse,
// whose factors run in the opposite order), six launches; four when the rows pair two channels (one sequence per
// channel): then one kernel does every chunk stage.  Spectra stay in the order the forward leaves them in.
static bool conv_chunks_supported(const int *factors, int nf, monarch_dtype dt)
{
    if (nf == 2) return fft2_lds_supported(factors[0], factors[1], dt);
    const int f0 = factors[0];
    return nf == 3 && (f0 == 16 || f0 == 32 || f0 == 64 || f0 == 128) && fft2_lds_supported(factors[1], factors[2], dt);
}

static int conv_chunks_lds(const void *u, const void *k, const void *g_in, const void *g_out, void *y,
                           int B, int H, int n, int klen, int nfft, const int *factors, int nf,
                           void *const bufs[2], float2 *kf, hipStream_t s)
{
    // rows that share a complex row: two batch entries of a channel, or (one sequence per channel) two
    // neighbouring channels, then with the kernels paired alike and separated again before the inverse
    const bool by_channel = B == 1 && H >= 2;
    const bool paired = B >= 2 || by_channel;
    const int pair_stride = by_channel ? 1 : H;
    const int64_t crows = by_channel ? (H + 1) / 2 : paired ? (int64_t)((B + 1) / 2) * H : (int64_t)B * H;
    const int f1 = factors[nf - 2], f2 = factors[nf - 1], O = nf == 3 ? factors[0] : 1;

    Fft2Args a;
    memset(&a, 0, sizeof(a));
    a.N = nfft;
    a.O = O;
    a.f1 = f1;
    a.f2 = f2;
    a.H = H;
    a.pair_stride = pair_stride;
    a.real_rows = (int64_t)B * H;
    a.scale = 1.0f;
    FftPass first = blank_pass();   // the strided pass of a three-factor transform
    if (nf == 3) {
        set_pass_geometry(first, nfft, factors, nf, 0);
        first.dt = MONARCH_BF16;
        first.H = H;
        first.pair_stride = pair_stride;
        first.real_rows = (int64_t)B * H;
    }
    int rc;
    // two factors, rows of a multiple of 8 elements, kernels not paired: the rows never leave the chip
    const bool one_kernel = nf == 2 && !by_channel && n % 8 == 0;
    // three factors, channels paired: four launches, the spectra never leave the chip
    const bool fused_middle = nf == 3 && by_channel && conv3_middle_supported(O, f1, f2, MONARCH_BF16);
    for (int which = 0; which < (one_kernel ? 1 : 2); ++which) {   // 0: spectrum of k (into kf), 1: spectrum of g_in o u (into bufs[1])
        const bool pair_here = which == 0 ? by_channel : paired;
        const int64_t rows = which == 0 ? (by_channel ? crows : H) : crows;
        const void *src = which == 0 ? k : u;
        const void *gate = which == 0 ? nullptr : g_in;
        const int valid = which == 0 ? klen : n;
        void *dst = which == 0 ? (void *)kf : bufs[1];
        Fft2Args p = a;
        p.rows = rows;
        p.out = dst;
        p.store = ST_C16;
        if (nf == 2) {
            p.in = src;
            p.gate = gate;
            p.n_valid = valid;
            p.load = pair_here ? LD_REAL_PAIR : LD_REAL;
        } else {
            FftPass q = first;
            q.rows = rows;
            q.in = src;
            q.gate = gate;
            q.n_valid = valid;
            q.load = pair_here ? LD_REAL_PAIR : LD_REAL;
            q.out = fused_middle ? dst : bufs[0];
            q.store = ST_C16;
            rc = launch_fft_pass_mfma(q, s);
            if (rc) return rc;
            if (fused_middle) continue;   // the chunk factors run in the middle kernel
            p.in = bufs[0];
            p.load = LD_C16;
        }
        rc = launch_fft2_lds(p, s);
        if (rc) return rc;
    }
    if (one_kernel) {
        Fft2Args p = a;
        p.rows = crows;
        p.in = u;
        p.gate = g_in;
        p.gate_out = g_out;
        p.kf = kf;
        p.out = y;
        p.n_valid = n;
        p.load = paired ? LD_REAL_PAIR : LD_REAL;
        p.store = paired ? ST_REAL_PAIR : ST_REAL_SCALE_GATE;
        p.scale = 1.0f / (float)nfft;
        return launch_fft2_lds(p, s);
    }
    // inverse: product of the spectra on load, chunk factors, then (three factors) the strided factor
    Fft2Args p = a;
    p.rows = crows;
    p.in = bufs[1];
    p.kf = kf;
    p.inverse = 1;
    p.load = by_channel ? LD_C16_HERM_MULK : LD_C16_CONJ_MULK;
    const int real_store = paired ? ST_REAL_PAIR : ST_REAL_SCALE_GATE;
    if (nf == 2) {
        p.gate = g_out;
        p.out = y;
        p.n_valid = n;
        p.store = real_store;
        p.scale = 1.0f / (float)nfft;
        return launch_fft2_lds(p, s);
    }
    p.out = bufs[0];
    p.store = ST_C16;
    p.tw_outer = 1;
    rc = fused_middle ? launch_conv3_middle(p, s) : launch_fft2_lds(p, s);
    if (rc) return rc;
    FftPass q = first;
    q.rows = crows;
    q.in = bufs[0];
    q.load = LD_C16;
    q.out = y;
    q.gate = g_out;
    q.n_valid = n;
    q.store = real_store;
    q.scale = (fused_middle ? 0.25f : 1.0f) / (float)nfft;   // the fused middle leaves the halves of its separation to this scale
    return launch_fft_pass_mfma(q, s);
}

// Multi-pass convolution on the matrix cores (bf16 or fp32, factors 16..128).  The kernel is real, so two
// real rows of the same channel are transformed as one complex row (re = batch 2 b2, im = batch
// 2 b2 + 1): conv(a + i b, k) = conv(a, k) + i conv(b, k).  Rows travel between passes as packed
// bf16 pairs; the spectrum of k is kept in fp32.
static int conv_passes_mfma(const void *u, const void *k, const void *g_in, const void *g_out, void *y,
                            int B, int H, int n, int klen, int nfft, const int *factors, int nf,
                            void *const bufs[2], float2 *kf, monarch_dtype dt, hipStream_t s)
{
    // bf16: packed bf16 pairs between passes; fp32 (16x16x4 MFMA): complex fp32 between passes
    const bool half = dt == MONARCH_BF16;
    const int ld_mid = half ? LD_C16 : LD_C32, st_mid = half ? ST_C16 : ST_C32;
    auto launch = [&](const FftPass &p) { return half ? launch_fft_pass_mfma(p, s) : launch_fft_pass_mfma_f32(p, s); };
    // B >= 2: batch entries 2 b2, 2 b2 + 1 of a channel share a complex row (same kernel, so the spectra just
    // multiply).  B = 1 (one long sequence per channel), bf16: neighbouring channels share a complex row, the
    // kernels are paired the same way and the first inverse pass separates the Hermitian halves.
    const bool by_channel = half && B == 1 && H >= 2;
    const bool paired = B >= 2 || by_channel;
    const int pair_stride = by_channel ? 1 : H;
    const int64_t crows = by_channel ? (H + 1) / 2 : paired ? (int64_t)((B + 1) / 2) * H : (int64_t)B * H;
    const void *cur = nullptr;
    int rc;
    for (int which = 0; which < 2; ++which) {   // 0: k_f = F k', 1: u_f = F (g_in o u)'
        cur = which == 0 ? k : u;
        for (int q = 0; q < nf; ++q) {
            FftPass p = blank_pass();
            set_pass_geometry(p, nfft, factors, nf, q);
            p.rows = which == 0 && !by_channel ? H : crows;
            p.dt = dt;
            p.in = cur;
            p.H = H;
            p.pair_stride = pair_stride;
            p.real_rows = (int64_t)B * H;
            if (q == 0) {
                p.load = (which == 1 && paired) || by_channel ? LD_REAL_PAIR : LD_REAL;
                p.n_valid = which == 0 ? klen : n;
                p.gate = which == 0 ? nullptr : g_in;
            } else {
                p.load = ld_mid;
            }
            if (q == nf - 1) {
                p.store = (which == 0 && !by_channel) || !half ? ST_C32_NATURAL : ST_C16_NATURAL;
                p.out = which == 0 ? (void *)kf : bufs[q & 1];
            } else {
                p.store = st_mid;
                p.out = bufs[q & 1];
            }
            rc = launch(p);
            if (rc) return rc;
            cur = p.out;
        }
    }
    // y = Re / Im of F^-1 (k_f o u_f), first n entries, times g_out:  F^-1 z = conj(F conj(z)) / N.
    const int first_out = (cur == bufs[0]) ? 1 : 0;
    for (int q = 0; q < nf; ++q) {
        FftPass p = blank_pass();
        set_pass_geometry(p, nfft, factors, nf, q);
        p.rows = crows;
        p.dt = dt;
        p.in = cur;
        p.H = H;
        p.pair_stride = pair_stride;
        p.real_rows = (int64_t)B * H;
        if (q == 0) {
            p.load = by_channel ? LD_C16_HERM_MULK : half ? LD_C16_CONJ_MULK : LD_C32_CONJ_MULK;
            p.kf = kf;
        } else {
            p.load = ld_mid;
        }
        if (q == nf - 1) {
            p.store = paired ? ST_REAL_PAIR : ST_REAL_SCALE_GATE;
            p.out = y;
            p.gate = g_out;
            p.n_valid = n;
            p.scale = 1.0f / (float)nfft;
        } else {
            p.store = st_mid;
            p.out = bufs[(first_out + q) & 1];
        }
        rc = launch(p);
        if (rc) return rc;
        cur = p.out;
    }
    return MONARCH_OK;
}

static int conv_run(const void *u, const void *k, const void *g_in, const void *g_out, void *y,
                    int B, int H, int n, int klen, int nfft, const int *factors, int nf,
                    int causal, monarch_dtype dt, void *ws, size_t ws_bytes, monarch_stream_t stream)
{
    int rc = conv_check(B, H, n, klen, nfft, factors, nf, causal, dt);
    if (rc) return rc;
    if (B == 0 || H == 0) return MONARCH_OK;
    if (!u || !k || !y) return fail(MONARCH_EINVAL, "u, k and y must be non-NULL");
    if (misaligned(u) || misaligned(k) || misaligned(y) || misaligned(g_in) || misaligned(g_out) || misaligned(ws))
        return fail(MONARCH_EINVAL, "pointers must be 16-byte aligned");
    const size_t es = dtype_size(dt);
    const size_t rows = (size_t)B * H;
    const size_t act_bytes = rows * n * es;
    if (overlaps(y, act_bytes, u, act_bytes) || overlaps(y, act_bytes, g_in, act_bytes) ||
        overlaps(y, act_bytes, g_out, act_bytes) || overlaps(y, act_bytes, k, (size_t)H * klen * es))
        return fail(MONARCH_EINVAL, "y overlaps an input");
    const size_t need = monarch_causal_conv_workspace_bytes(B, H, n, klen, nfft, factors, nf, dt);
    if (need && (!ws || ws_bytes < need))
        return fail(MONARCH_EWORKSPACE, "workspace of %zu bytes needed, %zu given", need, ws ? ws_bytes : (size_t)0);
    hipStream_t s = (hipStream_t)stream;

    const int fused = conv_fused_path(n, klen, factors, nf, dt);
    if (fused == 1) return launch_conv_mfma_2048(u, k, g_in, g_out, y, B, H, n, klen, dt, s);
    if (fused == 2) return launch_conv_mfma_256(u, k, g_in, g_out, y, B, H, n, klen, s);
    if (fused == 3) return launch_conv_mfma_16k(u, k, g_in, g_out, y, B, H, n, klen, s);
    if (fused == 4) return launch_conv_f32_2048(u, k, g_in, g_out, y, B, H, n, klen, s);

    const size_t buf = align_up(rows * nfft * sizeof(float2), 256);
    void *bufs[2] = {ws, (char *)ws + buf};
    float2 *kf = (float2 *)((char *)ws + 2 * buf);

    if (conv_chunks_supported(factors, nf, dt))
        return conv_chunks_lds(u, k, g_in, g_out, y, B, H, n, klen, nfft, factors, nf, bufs, kf, s);
    if (fft_mfma_supported(nfft, factors, nf, dt) || fft_mfma_f32_supported(nfft, factors, nf, dt))
        return conv_passes_mfma(u, k, g_in, g_out, y, B, H, n, klen, nfft, factors, nf, bufs, kf, dt, s);

    // 1. k_f = F k'  (H rows), staged through the row buffers.
    // 2. u_f = F (g_in o u)'  (B*H rows), left in natural order in one of the row buffers.
    const void *cur = nullptr;
    for (int which = 0; which < 2; ++which) {
        cur = which == 0 ? k : u;
        for (int q = 0; q < nf; ++q) {
            FftPass p = blank_pass();
            set_pass_geometry(p, nfft, factors, nf, q);
            p.rows = which == 0 ? H : (int64_t)rows;
            p.dt = dt;
            p.in = cur;
            if (q == 0) {
                p.load = LD_REAL;
                p.n_valid = which == 0 ? klen : n;
                p.gate = which == 0 ? nullptr : g_in;
            } else {
                p.load = LD_C32;
            }
            if (q == nf - 1) {
                p.store = ST_C32_NATURAL;
                p.out = which == 0 ? (void *)kf : bufs[q & 1];
            } else {
                p.store = ST_C32;
                p.out = bufs[q & 1];
            }
            rc = launch_fft_pass(p, s);
            if (rc) return rc;
            cur = p.out;
        }
    }
    // 3. y = Re F^-1 (k_f o u_f), first n entries, times g_out:  F^-1 z = conj(F conj(z)) / N.
    const int first_out = (cur == bufs[0]) ? 1 : 0;
    for (int q = 0; q < nf; ++q) {
        FftPass p = blank_pass();
        set_pass_geometry(p, nfft, factors, nf, q);
        p.rows = (int64_t)rows;
        p.dt = dt;
        p.in = cur;
        if (q == 0) {
            p.load = LD_C32_CONJ_MULK;
            p.kf = kf;
            p.H = H;
        } else {
            p.load = LD_C32;
        }
        if (q == nf - 1) {
            p.store = ST_REAL_SCALE_GATE;
            p.out = y;
            p.gate = g_out;
            p.n_valid = n;
            p.scale = 1.0f / (float)nfft;
        } else {
            p.store = ST_C32;
            p.out = bufs[(first_out + q) & 1];
        }
        rc = launch_fft_pass(p, s);
        if (rc) return rc;
        cur = p.out;
    }
    return MONARCH_OK;
}

int monarch_causal_conv(const void *u, const void *k, const void *g_in, const void *g_out, void *y,
                        int B, int H, int n, int klen, int nfft, const int *factors, int nf,
                        int causal, monarch_dtype dt, void *ws, size_t ws_bytes,
                        monarch_stream_t stream)
{
    clear_error();
    return conv_run(u, k, g_in, g_out, y, B, H, n, klen, nfft, factors, nf, causal, dt, ws, ws_bytes, stream);
}

// The same convolution for callers that cannot allocate: the row buffers and the spectrum of k live in a
// file-scope device array instead of a caller's workspace.  Every GPU the library runs on holds its own copy of
// the array at its own address; host code never uses the array's name as an address (it is only a stand-in on the
// host side) but the pointer looked up once per device below.
static __device__ __align__(256) unsigned char scratch[MONARCH_STATIC_SCRATCH_BYTES];

static const int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];          // per device: address of that device's copy, NULL until looked up
static std::mutex g_scratch_mutex;

// Address of the current device's copy of `scratch` (looked up on the first call on that device).
static int static_scratch(void **out)
{
    int dev = 0;
    MONARCH_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(MONARCH_EHIP, "device ordinal %d outside [0, %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        MONARCH_HIP_CHECK(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return fail(MONARCH_EHIP, "the static scratch array has no address on device %d", dev);
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return MONARCH_OK;
}

int monarch_causal_conv_static(const void *u, const void *k, const void *g_in, const void *g_out, void *y,
                               int B, int H, int n, int klen, int nfft, const int *factors, int nf,
                               int causal, monarch_dtype dt, monarch_stream_t stream)
{
    clear_error();
    int rc = conv_check(B, H, n, klen, nfft, factors, nf, causal, dt);
    if (rc) return rc;
    const size_t need = monarch_causal_conv_workspace_bytes(B, H, n, klen, nfft, factors, nf, dt);
    if (need > (size_t)MONARCH_STATIC_SCRATCH_BYTES)
        return fail(MONARCH_EWORKSPACE, "this shape needs %zu bytes of scratch; the static array holds %zu "
                    "(use monarch_causal_conv with a workspace)", need, (size_t)MONARCH_STATIC_SCRATCH_BYTES);
    void *ptr = nullptr;
    if (need) {
        rc = static_scratch(&ptr);
        if (rc) return rc;
    }
    return conv_run(u, k, g_in, g_out, y, B, H, n, klen, nfft, factors, nf, causal, dt, ptr, need, stream);
}

// ---------------------------------------------------------------------------------------------
// monarch_mlp
// ---------------------------------------------------------------------------------------------

static int mlp_check(int64_t tokens, int d, int d_hidden, int nb, int order, int &mid1, int &mid2,
                     int act, monarch_dtype dt)
{
    int rc = check_dtype(dt, true);
    if (rc) return rc;
    if (tokens < 0) return fail(MONARCH_ESHAPE, "negative token count");
    if (d < 1 || d_hidden < 1 || nb < 1) return fail(MONARCH_ESHAPE, "d, d_hidden and nb must be >= 1");
    if (order != 1 && order != 2) return fail(MONARCH_ESHAPE, "order must be 1 or 2 (got %d)", order);
    if (act < 0 || act > 2) return fail(MONARCH_EINVAL, "act must be 0, 1 or 2");
    if (d % nb || d_hidden % nb) return fail(MONARCH_ESHAPE, "nb=%d must divide d=%d and d_hidden=%d", nb, d, d_hidden);
    if (order == 2) {
        if (mid1 == 0) mid1 = d;
        if (mid2 == 0) mid2 = d;
        if (mid1 < 1 || mid2 < 1 || mid1 % nb || mid2 % nb)
            return fail(MONARCH_ESHAPE, "nb=%d must divide mid1=%d and mid2=%d", nb, mid1, mid2);
        if (!matmul_generic_fits(d, mid1, d_hidden) || !matmul_generic_fits(d_hidden, mid2, d))
            return fail(MONARCH_ESHAPE, "layer widths exceed the on-chip tile");
    } else {
        mid1 = mid2 = 0;
        if (!matmul_generic_fits(d, d_hidden, d_hidden) || !matmul_generic_fits(d_hidden, d, d))
            return fail(MONARCH_ESHAPE, "layer widths exceed the on-chip tile");
    }
    return MONARCH_OK;
}

// Order 2 on the matrix cores: W1 = P L1 P R1 P and W2 = P L2 P R2 P meet at the hidden vector, where
// block k of L1 feeds exactly block k of R2, so [L1, bias, activation, R2] is a block-diagonal MLP
// whose hidden vector stays on chip; R1 and L2 with the permutations around them are one launch each.
static bool mlp_order2_mfma_supported(int d, int d_hidden, int nb, int mid1, int mid2, monarch_dtype dt)
{
    if (nb < 1 || mid1 < 1 || mid1 != mid2 || d % nb || mid1 % nb || d_hidden % nb) return false;
    return factor_mfma_supported(nb, mid1 / nb, d / nb, dt) && mlp_mfma_order1_supported(mid1, d_hidden, nb, dt) &&
           factor_mfma_supported(nb, d / nb, mid2 / nb, dt);
}

size_t monarch_mlp_workspace_bytes(int64_t tokens, int d, int d_hidden, int nb, int order,
                                   int mid1, int mid2, monarch_dtype dt)
{
    if (tokens <= 0 || d_hidden <= 0) return 0;
    if (order == 1 && nb > 0 && mlp_mfma_order1_supported(d, d_hidden, nb, dt)) return 0;   // hidden stays on chip
    if (order == 2) {
        const int m1 = mid1 > 0 ? mid1 : d, m2 = mid2 > 0 ? mid2 : d;   // same defaults as the call itself
        if (mlp_order2_mfma_supported(d, d_hidden, nb, m1, m2, dt))   // the two d_mid-wide intermediates, bf16
            return 2 * align_up((size_t)tokens * m1 * sizeof(bf16_t), 256);
    }
    return align_up((size_t)tokens * d_hidden * sizeof(float), 256);   // hidden activations, fp32
}

int monarch_mlp(const void *x, void *y, int64_t tokens, int d, int d_hidden, int nb, int order,
                const void *W1_R, const void *W1_L, const void *b1,
                const void *W2_R, const void *W2_L, const void *b2,
                int mid1, int mid2, int act, monarch_dtype dt, void *ws, size_t ws_bytes,
                monarch_stream_t stream)
{
    clear_error();
    int rc = mlp_check(tokens, d, d_hidden, nb, order, mid1, mid2, act, dt);
    if (rc) return rc;
    if (tokens == 0) return MONARCH_OK;
    if (!x || !y || !W1_R || !W2_R) return fail(MONARCH_EINVAL, "x, y, W1_R and W2_R must be non-NULL");
    if (order == 2 && (!W1_L || !W2_L)) return fail(MONARCH_EINVAL, "order 2 needs W1_L and W2_L");
    if (order == 1 && (W1_L || W2_L)) return fail(MONARCH_EINVAL, "order 1 takes no W1_L / W2_L");
    if (misaligned(x) || misaligned(y) || misaligned(W1_R) || misaligned(W1_L) || misaligned(b1) ||
        misaligned(W2_R) || misaligned(W2_L) || misaligned(b2) || misaligned(ws))
        return fail(MONARCH_EINVAL, "pointers must be 16-byte aligned");
    const size_t es = dtype_size(dt);
    if (overlaps(y, (size_t)tokens * d * es, x, (size_t)tokens * d * es)) return fail(MONARCH_EINVAL, "y overlaps x");
    const size_t need = monarch_mlp_workspace_bytes(tokens, d, d_hidden, nb, order, mid1, mid2, dt);
    if (need && (!ws || ws_bytes < need))
        return fail(MONARCH_EWORKSPACE, "workspace of %zu bytes needed, %zu given", need, ws ? ws_bytes : (size_t)0);
    hipStream_t s = (hipStream_t)stream;

    if (order == 1 && mlp_mfma_order1_supported(d, d_hidden, nb, dt))
        return launch_mlp_mfma_order1(x, y, tokens, d, d_hidden, nb, W1_R, b1, W2_R, b2, act, 0, dt, s);
    if (order == 2 && mlp_order2_mfma_supported(d, d_hidden, nb, mid1, mid2, dt)) {
        void *t2 = ws, *u1 = (char *)ws + align_up((size_t)tokens * mid1 * sizeof(bf16_t), 256);
        rc = launch_factor_mfma(x, t2, tokens, nb, mid1 / nb, d / nb, W1_R, nullptr, 0, dt, s);
        if (rc) return rc;
        // hidden unit h of block k is position h nb + k of the hidden vector: that is where its bias sits
        rc = launch_mlp_mfma_order1(t2, u1, tokens, mid1, d_hidden, nb, W1_L, b1, W2_R, nullptr, act, 1, dt, s);
        if (rc) return rc;
        return launch_factor_mfma(u1, y, tokens, nb, d / nb, mid2 / nb, W2_L, b2, 2, dt, s);
    }

    // Layer 1 writes the activated hidden vector (fp32) to the workspace, layer 2 reads it.
    if (order == 1) {
        rc = launch_matmul_generic(x, W1_R, nullptr, b1, ws, tokens, nb, d_hidden / nb, d / nb, 1, 1, 1, 1, act,
                                   dt, dt, MONARCH_F32, s);
        if (rc) return rc;
        return launch_matmul_generic(ws, W2_R, nullptr, b2, y, tokens, nb, d / nb, d_hidden / nb, 1, 1, 1, 1, 0,
                                     MONARCH_F32, dt, dt, s);
    }
    rc = launch_matmul_generic(x, W1_R, W1_L, b1, ws, tokens, nb, mid1 / nb, d / nb, nb, d_hidden / nb, mid1 / nb,
                               2, act, dt, dt, MONARCH_F32, s);
    if (rc) return rc;
    return launch_matmul_generic(ws, W2_R, W2_L, b2, y, tokens, nb, mid2 / nb, d_hidden / nb, nb, d / nb, mid2 / nb,
                                 2, 0, MONARCH_F32, dt, dt, s);
}

}  // extern "C"
