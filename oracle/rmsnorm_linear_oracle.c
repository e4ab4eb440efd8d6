/*
 * CPU oracle for the RMSNorm-then-linear block.  TEST INFRASTRUCTURE ONLY.
 *
 * It exists to check the HIP library; nothing in the product path may call
 * it.  Only the test suite, the smoke check and the benchmark's CPU-baseline
 * leg load this file.  It shares no code, header, table or helper with the
 * HIP sources.
 *
 * What it computes is the plain, unfused definition, in double precision:
 *
 *   RMSNorm (case-study section, Eq. 1):
 *       Yn[i][j] = X[i][j] * G[j] / RMS(X_i),   RMS(X_i) = sqrt( (1/d) sum_j X[i][j]^2 )
 *   followed by the matrix product of the computation graph in Fig. 2a:
 *       Z[i][n] = sum_j Yn[i][j] * W[j][n]
 *
 * The fused kernel the paper discovers (Fig. 2b: the division moved behind
 * the product) reaches the same value up to rounding order, so the definition
 * itself is the reference; the rewrite is NOT used here.
 *
 * Reading taken where the paper is silent: Eq. 1 has no epsilon.  The
 * benchmark configurations carry one, and it is added to the mean square
 * under the root:  RMS_eps(X_i) = sqrt( mean_j X[i][j]^2 + eps ).
 * With eps = 0 this is Eq. 1 exactly.
 *
 * Every sum runs left to right over the reduction index, one element at a
 * time; rows are independent and are spread over OpenMP threads.  No
 * blocking, no reordering, no BLAS.
 *
 * Gated MLP (the paper's GatedMLP benchmark: two products of the same input,
 * SiLU on one, elementwise product with the other): with the block's output
 * Z [rows][2H] read as [gate | up],  Y[i][h] = SiLU(Z[i][h]) * Z[i][H + h],
 * SiLU(v) = v / (1 + exp(-v)).  oracle_silu_mul_f64 is that definition on
 * doubles, applied to the block's unrounded fp64 output.
 *
 * Normalised-Transformer chain (the paper's nTrans benchmark), y = Norm(x + alpha (Norm(h - x))),
 * x, h [M][D], alpha [D]: oracle_ntrans takes it literally, three steps per row.  Reading: the
 * paper does not say which normalisation "Norm" is; it is taken to be the only one the paper
 * defines, Eq. 1 without a gain (divide by the root of the mean square, eps under the root).
 *
 * QKNorm in front of attention (the paper's QKNorm benchmark: layer normalisation of the query and
 * key vectors before attention), decode form, one query per head: oracle_qknorm_attention takes it
 * literally -- LayerNorm of q, LayerNorm of every key, scores, softmax, weighted sum of V.
 * Readings: "layer normalization" is the usual one (subtract the mean, divide by the root of the
 * population variance plus eps, times a gain, plus a bias; gain and bias of length D, shared by the
 * heads); scores are scaled by 1/sqrt(D); the paper gives no eps.
 * Pins (tests/test_qknorm_pins.py): a D = 2 closed form, shift and scale invariance, uniform
 * attention for equal keys and for a zero key gain, library layer_norm + attention in float64.
 *
 * Parity pins (tests/test_oracle_*.py): printed-by-hand 2x3 cases, the
 * eps-placement case, exact rational brute force, scale invariance, unit-RMS
 * rows, linearity, and a library float64 product; for the gate: closed forms
 * at v = 0, +-ln 3, the identity SiLU(v) - SiLU(-v) = v, linearity in the up
 * half, library float64 sigmoids.  No function here is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F16 = 0, ORACLE_BF16 = 1, ORACLE_F32 = 2 };

/* IEEE binary16 -> double, exact.  1 sign, 5 exponent (bias 15), 10 fraction bits. */
double oracle_decode_f16(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0)
        v = ldexp((double)frac, -24);                 /* zero and subnormals */
    else if (expo == 31)
        v = frac ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)frac / 1024.0, expo - 15);
    return sign ? -v : v;
}

/* bfloat16 -> double, exact.  1 sign, 8 exponent (bias 127), 7 fraction bits. */
double oracle_decode_bf16(uint16_t b)
{
    int sign = (b >> 15) & 1;
    int expo = (b >> 7) & 0xff;
    int frac = b & 0x7f;
    double v;
    if (expo == 0)
        v = ldexp((double)frac, -133);                /* 2^-126 * frac/128 */
    else if (expo == 255)
        v = frac ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)frac / 128.0, expo - 127);
    return sign ? -v : v;
}

static inline double load_elem(const void *base, size_t idx, int dtype)
{
    switch (dtype) {
    case ORACLE_F16:  return oracle_decode_f16(((const uint16_t *)base)[idx]);
    case ORACLE_BF16: return oracle_decode_bf16(((const uint16_t *)base)[idx]);
    default:          return (double)((const float *)base)[idx];
    }
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Widen a storage array to double, element by element. */
void oracle_decode(const void *src, int dtype, size_t n, double *dst)
{
    for (size_t i = 0; i < n; ++i)
        dst[i] = load_elem(src, i, dtype);
}

/*
 * Eq. 1 on doubles: out[i][j] = x[i][j] * g[j] / sqrt(mean_j x[i][j]^2 + eps).
 * x is [M][K], g is [K], out is [M][K], all row-major.
 */
void oracle_rmsnorm_f64(const double *x, const double *g, double eps,
                        long M, long K, double *out)
{
#pragma omp parallel for schedule(static)
    for (long i = 0; i < M; ++i) {
        const double *xi = x + (size_t)i * K;
        double s = 0.0;
        for (long j = 0; j < K; ++j)
            s += xi[j] * xi[j];
        double rms = sqrt(s / (double)K + eps);
        for (long j = 0; j < K; ++j)
            out[(size_t)i * K + j] = xi[j] * g[j] / rms;
    }
}

/* Plain product on doubles: z[i][n] = sum_j a[i][j] * w[j][n]; a [M][K], w [K][N]. */
void oracle_matmul_f64(const double *a, const double *w, long M, long K, long N, double *z)
{
#pragma omp parallel for schedule(static)
    for (long i = 0; i < M; ++i) {
        double *zi = z + (size_t)i * N;
        for (long n = 0; n < N; ++n)
            zi[n] = 0.0;
        for (long j = 0; j < K; ++j) {
            double aij = a[(size_t)i * K + j];
            const double *wj = w + (size_t)j * N;
            for (long n = 0; n < N; ++n)
                zi[n] += aij * wj[n];
        }
    }
}

/*
 * The whole block on storage-typed inputs, for a list of rows.
 *
 *   X [M][K], G [K], W [K][N] in the storage type `dtype` (every element is
 *   widened exactly to double); rows[0..n_rows) are the row indices to
 *   evaluate; Z is [n_rows][N] doubles, never rounded to the storage type.
 *
 * Per row: Eq. 1 first (the normalised row is formed in full), then the
 * product with W, summing over j in increasing order for every output.
 * Returns 0, or -1 on a bad argument.
 */
int oracle_rmsnorm_linear(const void *X, const void *G, const void *W, int dtype,
                          double eps, long M, long K, long N,
                          const long *rows, long n_rows, double *Z)
{
    if (!X || !G || !W || !Z || !rows || M <= 0 || K <= 0 || N <= 0 || n_rows < 0)
        return -1;
    if (dtype != ORACLE_F16 && dtype != ORACLE_BF16 && dtype != ORACLE_F32)
        return -1;
    for (long r = 0; r < n_rows; ++r)
        if (rows[r] < 0 || rows[r] >= M)
            return -1;

    /* widen G and W to double once, so the row loops below read plain doubles */
    double *gd = (double *)malloc(sizeof(double) * (size_t)K);
    double *wd = (double *)malloc(sizeof(double) * (size_t)K * (size_t)N);
    if (!gd || !wd) {
        free(gd);
        free(wd);
        return -1;
    }
    oracle_decode(G, dtype, (size_t)K, gd);
#pragma omp parallel for schedule(static)
    for (long j = 0; j < K; ++j)
        oracle_decode((const char *)W + (size_t)j * N * (dtype == ORACLE_F32 ? 4 : 2),
                      dtype, (size_t)N, wd + (size_t)j * N);
    int failed = 0;

#pragma omp parallel
    {
        double *yn = (double *)malloc(sizeof(double) * (size_t)K);
        if (!yn) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (long r = 0; r < n_rows; ++r) {
            if (!yn)
                continue;
            size_t i = (size_t)rows[r];
            /* Eq. 1: sum of squares of the raw row, then the normalised, gained row */
            double s = 0.0;
            for (long j = 0; j < K; ++j) {
                double x = load_elem(X, i * (size_t)K + j, dtype);
                s += x * x;
            }
            double rms = sqrt(s / (double)K + eps);
            for (long j = 0; j < K; ++j) {
                double x = load_elem(X, i * (size_t)K + j, dtype);
                yn[j] = x * gd[j] / rms;
            }
            /* Fig. 2a: the product that follows the norm */
            double *zr = Z + (size_t)r * N;
            for (long n = 0; n < N; ++n)
                zr[n] = 0.0;
            for (long j = 0; j < K; ++j) {
                double a = yn[j];
                const double *wj = wd + (size_t)j * N;
                for (long n = 0; n < N; ++n)
                    zr[n] += a * wj[n];
            }
        }
        free(yn);
    }
    free(gd);
    free(wd);
    return failed ? -1 : 0;
}

/*
 * Gate of the GatedMLP block on doubles: z is [rows][2H], columns [0, H) the gate half and
 * [H, 2H) the up half; y is [rows][H]:  y[i][h] = SiLU(z[i][h]) * z[i][H + h].
 */
void oracle_silu_mul_f64(const double *z, long rows, long H, double *y)
{
#pragma omp parallel for schedule(static)
    for (long i = 0; i < rows; ++i) {
        const double *zi = z + (size_t)i * 2 * (size_t)H;
        for (long h = 0; h < H; ++h) {
            double v = zi[h];
            double silu = v / (1.0 + exp(-v));
            y[(size_t)i * H + h] = silu * zi[(size_t)H + h];
        }
    }
}

/*
 * nTrans chain on storage-typed inputs: Y[i][:] = Norm(X[i] + alpha * Norm(H[i] - X[i])), Norm(v) =
 * v / sqrt(mean(v^2) + eps).  Y is [M][D] doubles.  Returns 0, or -1 on a bad argument.
 */
int oracle_ntrans(const void *X, const void *Hh, const void *A, int dtype, double eps,
                  long M, long D, double *Y)
{
    if (!X || !Hh || !A || !Y || M <= 0 || D <= 0)
        return -1;
    if (dtype != ORACLE_F16 && dtype != ORACLE_BF16 && dtype != ORACLE_F32)
        return -1;
    int failed = 0;
#pragma omp parallel
    {
        double *d = (double *)malloc(sizeof(double) * (size_t)D);
        double *u = (double *)malloc(sizeof(double) * (size_t)D);
        if (!d || !u) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(static)
        for (long i = 0; i < M; ++i) {
            if (!d || !u)
                continue;
            /* inner Norm(h - x) */
            double s = 0.0;
            for (long j = 0; j < D; ++j) {
                d[j] = load_elem(Hh, (size_t)i * D + j, dtype) - load_elem(X, (size_t)i * D + j, dtype);
                s += d[j] * d[j];
            }
            double r1 = sqrt(s / (double)D + eps);
            /* x + alpha * (that) */
            double t = 0.0;
            for (long j = 0; j < D; ++j) {
                u[j] = load_elem(X, (size_t)i * D + j, dtype) + load_elem(A, (size_t)j, dtype) * (d[j] / r1);
                t += u[j] * u[j];
            }
            /* outer Norm */
            double r2 = sqrt(t / (double)D + eps);
            for (long j = 0; j < D; ++j)
                Y[(size_t)i * D + j] = u[j] / r2;
        }
        free(d);
        free(u);
    }
    return failed ? -1 : 0;
}

/* v[0..D) -> (v - mean) / sqrt(var + eps) * gain + bias, population variance. */
static void layer_norm_row(const double *v, const void *gain, const void *bias, int dtype, double eps,
                           long D, double *out)
{
    double mean = 0.0;
    for (long j = 0; j < D; ++j)
        mean += v[j];
    mean /= (double)D;
    double var = 0.0;
    for (long j = 0; j < D; ++j)
        var += (v[j] - mean) * (v[j] - mean);
    var /= (double)D;
    double r = sqrt(var + eps);
    for (long j = 0; j < D; ++j)
        out[j] = (v[j] - mean) / r * load_elem(gain, (size_t)j, dtype) + load_elem(bias, (size_t)j, dtype);
}

/*
 * QKNorm + attention, one query per (sample, head): Q [B][H][D], K and V [B][H][S][D], gains and
 * biases [D], O [B][H][D] doubles:
 *   qn = LayerNorm(q; gq, bq), kn_t = LayerNorm(k_t; gk, bk), s_t = qn . kn_t / sqrt(D),
 *   p = softmax_t(s), o = sum_t p_t v_t.
 * Returns 0, or -1 on a bad argument.
 */
int oracle_qknorm_attention(const void *Q, const void *K, const void *V, const void *gq, const void *bq,
                            const void *gk, const void *bk, int dtype, double eps,
                            long B, long H, long S, long D, double *O)
{
    if (!Q || !K || !V || !gq || !bq || !gk || !bk || !O || B <= 0 || H <= 0 || S <= 0 || D <= 0)
        return -1;
    if (dtype != ORACLE_F16 && dtype != ORACLE_BF16 && dtype != ORACLE_F32)
        return -1;
    int failed = 0;
#pragma omp parallel
    {
        double *raw = (double *)malloc(sizeof(double) * (size_t)D);
        double *qn = (double *)malloc(sizeof(double) * (size_t)D);
        double *kn = (double *)malloc(sizeof(double) * (size_t)D);
        double *sc = (double *)malloc(sizeof(double) * (size_t)S);
        if (!raw || !qn || !kn || !sc) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(static)
        for (long bh = 0; bh < B * H; ++bh) {
            if (!raw || !qn || !kn || !sc)
                continue;
            for (long j = 0; j < D; ++j)
                raw[j] = load_elem(Q, (size_t)bh * D + j, dtype);
            layer_norm_row(raw, gq, bq, dtype, eps, D, qn);
            double top = -INFINITY;
            for (long t = 0; t < S; ++t) {
                for (long j = 0; j < D; ++j)
                    raw[j] = load_elem(K, ((size_t)bh * S + t) * D + j, dtype);
                layer_norm_row(raw, gk, bk, dtype, eps, D, kn);
                double dot = 0.0;
                for (long j = 0; j < D; ++j)
                    dot += qn[j] * kn[j];
                sc[t] = dot / sqrt((double)D);
                if (sc[t] > top)
                    top = sc[t];
            }
            double denom = 0.0;
            for (long t = 0; t < S; ++t) {
                sc[t] = exp(sc[t] - top);
                denom += sc[t];
            }
            for (long j = 0; j < D; ++j) {
                double acc = 0.0;
                for (long t = 0; t < S; ++t)
                    acc += sc[t] / denom * load_elem(V, ((size_t)bh * S + t) * D + j, dtype);
                O[(size_t)bh * D + j] = acc;
            }
        }
        free(raw);
        free(qn);
        free(kn);
        free(sc);
    }
    return failed ? -1 : 0;
}
