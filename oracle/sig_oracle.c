/*
 * fp64 CPU oracle for the truncated signature transform.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the yardstick the HIP library is checked against; it is not part of the
 * product.  Only the tests, the smoke check and the benchmark's cpu_baseline leg may
 * call it.  It shares no code, header, table or helper with the HIP path.
 *
 * What it computes is the plain definition, by the "conventional" route the paper
 * describes (section 2.2, eq. "computation"; appendix A.1.1): the signature of a
 * piecewise-linear path is the group product of the tensor exponentials of its
 * increments,
 *     Sig(x_1..x_L) = exp(x_2 - x_1) [x] exp(x_3 - x_2) [x] ... [x] exp(x_L - x_{L-1}),
 * with   exp(v) = (v, v^{(x)2}/2!, ..., v^{(x)N}/N!)                    (section 2.2)
 * and    (A [x] B)_k = sum_{j=0..k} A_j (x) B_{k-j},  A_0 = B_0 = 1      (section 2.2,
 *                                                                 appendix eq. "tensorproduct").
 * Every exponential is formed separately and every product follows the definition term
 * by term: no Horner scheme, no fusion, no in-place update, no blocking.  The only
 * parallelism is an OpenMP loop over the batch.
 *
 * Layout of one truncated tensor-algebra element (section 2.4 gives only its size,
 * sum_{k=1..N} d^k; the order is this build's reading): levels k = 1..N concatenated,
 * the k = 0 term (identically 1, footnote in section 2.1) omitted; inside level k the
 * coefficient of e_{i_1} (x) ... (x) e_{i_k} sits at row-major offset
 * sum_m i_m d^{k-m} (0-based letters, i_1 slowest), i.e. lexicographic word order under
 * the identification of appendix A.2.2.
 *
 * Pinned by tests/test_oracle_pins.py against closed forms, invariants, brute force from
 * the integral definition and a hand-computed example; the gradient (second half of the file)
 * by tests/test_oracle_backward_pins.py against finite differences of the pinned forward and
 * closed forms; the logarithm and its gradient (third part) by tests/test_oracle_log_pins.py.
 * Nothing here is "parity unpinned".
 *
 * The entry points are declared, each with the passage it follows, in sig_oracle.h.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include "sig_oracle.h"

#ifdef _OPENMP
#include <omp.h>
#endif

/* d^k as int64; the callers keep d^N small enough (checked in sig_oracle_channels). */
static int64_t ipow64(int d, int k)
{
    int64_t r = 1;
    for (int i = 0; i < k; ++i) r *= d;
    return r;
}

/* Number of scalars in a depth-N element over R^d: sum_{k=1..N} d^k (section 2.4).
 * Returns -1 for d < 1, N < 1 or a size that does not fit 2^40 scalars. */
int64_t sig_oracle_channels(int d, int N)
{
    if (d < 1 || N < 1) return -1;
    const int64_t cap = (int64_t)1 << 40;
    int64_t total = 0, p = 1;
    for (int k = 1; k <= N; ++k) {
        if (p > cap / d) return -1;
        p *= d;
        total += p;
        if (total > cap) return -1;
    }
    return total;
}

/* Offset of level k (1-based) inside an element. */
static int64_t level_offset(int d, int k)
{
    int64_t off = 0;
    for (int j = 1; j < k; ++j) off += ipow64(d, j);
    return off;
}

/* Tensor exponential (section 2.2): E_k = z^{(x)k} / k!.
 * Built level by level as E_k = (E_{k-1} (x) z) / k, a true division each time. */
void sig_oracle_exp(const double *z, int d, int N, double *E)
{
    for (int i = 0; i < d; ++i) E[i] = z[i];
    for (int k = 2; k <= N; ++k) {
        const double *prev = E + level_offset(d, k - 1);
        double *cur = E + level_offset(d, k);
        const int64_t n_prev = ipow64(d, k - 1);
        for (int64_t w = 0; w < n_prev; ++w)
            for (int j = 0; j < d; ++j)
                cur[w * d + j] = prev[w] * z[j] / (double)k;
    }
}

/* Group product (section 2.2): C_k = sum_{j=0..k} A_j (x) B_{k-j} with A_0 = B_0 = 1,
 * i.e. C_k = B_k + A_k + sum_{j=1..k-1} A_j (x) B_{k-j}.  C must not alias A or B.
 * (A_j (x) B_m)[u, v] = A_j[u] * B_m[v]: the indices of B are appended on the right
 * (definition 1). */
void sig_oracle_mul(const double *A, const double *B, int d, int N, double *C)
{
    for (int k = 1; k <= N; ++k) {
        const int64_t off_k = level_offset(d, k);
        const int64_t n_k = ipow64(d, k);
        double *Ck = C + off_k;
        for (int64_t w = 0; w < n_k; ++w)
            Ck[w] = B[off_k + w] + A[off_k + w];
        for (int j = 1; j <= k - 1; ++j) {
            const int m = k - j;
            const double *Aj = A + level_offset(d, j);
            const double *Bm = B + level_offset(d, m);
            const int64_t n_j = ipow64(d, j);
            const int64_t n_m = ipow64(d, m);
            for (int64_t u = 0; u < n_j; ++u)
                for (int64_t v = 0; v < n_m; ++v)
                    Ck[u * n_m + v] += Aj[u] * Bm[v];
        }
    }
}

/* Signature of one path of L points in R^d (row-major [L][d]), per eq. "computation".
 * basepoint != 0 prepends the origin as an extra first point (this build's reading of the
 * `basepoint` argument named in section 5.5), giving L increments instead of L - 1.
 * stream != 0 writes the signature of every prefix (section 5.5, "expanding intervals"):
 * entry j is the signature after the (j+1)-th increment.  Otherwise only the last. */
static int one_path(const double *x, int64_t L, int d, int N, int stream, int basepoint,
                    double *out, int64_t S)
{
    const int64_t n_inc = basepoint ? L : L - 1;
    double *z = (double *)malloc(sizeof(double) * (size_t)d);
    double *cur = (double *)malloc(sizeof(double) * (size_t)S);
    double *E = (double *)malloc(sizeof(double) * (size_t)S);
    double *nxt = (double *)malloc(sizeof(double) * (size_t)S);
    if (!z || !cur || !E || !nxt) {
        free(z); free(cur); free(E); free(nxt);
        return 1;
    }
    for (int64_t s = 0; s < n_inc; ++s) {
        /* increment number s: between consecutive points of the (possibly extended) path */
        for (int c = 0; c < d; ++c) {
            double hi, lo;
            if (basepoint) {
                hi = x[s * d + c];
                lo = (s == 0) ? 0.0 : x[(s - 1) * d + c];
            } else {
                hi = x[(s + 1) * d + c];
                lo = x[s * d + c];
            }
            z[c] = hi - lo;
        }
        if (s == 0) {
            sig_oracle_exp(z, d, N, cur);
        } else {
            sig_oracle_exp(z, d, N, E);
            sig_oracle_mul(cur, E, d, N, nxt);
            double *t = cur; cur = nxt; nxt = t;
        }
        if (stream) memcpy(out + s * S, cur, sizeof(double) * (size_t)S);
    }
    if (!stream) memcpy(out, cur, sizeof(double) * (size_t)S);
    free(z); free(cur); free(E); free(nxt);
    return 0;
}

/* Batched forward signature, host pointers, fp64.
 *   path: [B][L][d] row-major.   out: [B][S] (stream == 0) or [B][n_inc][S] (stream != 0),
 *   S = sig_oracle_channels(d, N), n_inc = L - 1 (L with basepoint).
 * num_threads <= 0 lets OpenMP choose.  Returns 0 on success, 1 on bad arguments
 * (d < 1, N < 1, B < 0, fewer than two points once the basepoint is counted, null
 * pointers), 2 if memory ran out. */
int sig_oracle_forward_f64(const double *path, int64_t B, int64_t L, int d, int N,
                           int stream, int basepoint, double *out, int num_threads)
{
    const int64_t S = sig_oracle_channels(d, N);
    if (S < 0 || B < 0) return 1;
    if (basepoint ? (L < 1) : (L < 2)) return 1;
    if (B == 0) return 0;
    if (!path || !out) return 1;
    const int64_t n_inc = basepoint ? L : L - 1;
    const int64_t out_stride = stream ? n_inc * S : S;
    int failed = 0;
#ifdef _OPENMP
    if (num_threads > 0) omp_set_num_threads(num_threads);
#else
    (void)num_threads;
#endif
#pragma omp parallel for schedule(dynamic, 1) reduction(| : failed)
    for (int64_t b = 0; b < B; ++b)
        failed |= one_path(path + b * L * d, L, d, N, stream, basepoint, out + b * out_stride, S);
    return failed ? 2 : 0;
}

/* ------------------------------------------------------------------------------------------
 * Gradient of a scalar loss with respect to the path, given the gradient with respect to the
 * signature (section 5.3, appendix C).  The paper obtains it by treating the transform as a
 * composition of differentiable primitives (appendix C, first paragraph); this is that chain
 * rule written out over the oracle's own forward computation: every intermediate signature and
 * every exponential is kept in memory, and each primitive's adjoint is the transpose of the
 * loops above.  No reversibility, no recomputation, no Horner scheme.
 * ------------------------------------------------------------------------------------------ */

/* Adjoint of sig_oracle_mul: C = A [x] B, gC given; ADDS the gradients into gA and gB.
 * C_k = B_k + A_k + sum_{j=1..k-1} A_j (x) B_{k-j}. */
static void mul_adjoint(const double *A, const double *B, const double *gC, int d, int N, double *gA, double *gB)
{
    for (int k = 1; k <= N; ++k) {
        const int64_t off_k = level_offset(d, k);
        const int64_t n_k = ipow64(d, k);
        const double *gk = gC + off_k;
        for (int64_t w = 0; w < n_k; ++w) {
            gB[off_k + w] += gk[w];
            gA[off_k + w] += gk[w];
        }
        for (int j = 1; j <= k - 1; ++j) {
            const int m = k - j;
            const int64_t off_j = level_offset(d, j), off_m = level_offset(d, m);
            const int64_t n_j = ipow64(d, j), n_m = ipow64(d, m);
            for (int64_t u = 0; u < n_j; ++u)
                for (int64_t v = 0; v < n_m; ++v) {
                    const double g = gk[u * n_m + v];
                    gA[off_j + u] += g * B[off_m + v];
                    gB[off_m + v] += A[off_j + u] * g;
                }
        }
    }
}

/* Gradient of one group product C = A [x] B: WRITES gA and gB given gC (the transpose of sig_oracle_mul). */
void sig_oracle_mul_backward(const double *A, const double *B, const double *gC, int d, int N, double *gA, double *gB)
{
    const int64_t S = sig_oracle_channels(d, N);
    for (int64_t i = 0; i < S; ++i) gA[i] = gB[i] = 0.0;
    mul_adjoint(A, B, gC, d, N, gA, gB);
}

/* Adjoint of sig_oracle_exp: E_1 = z, E_k[w j] = E_{k-1}[w] z[j] / k.  gE is consumed (its lower
 * levels are used as accumulators); the gradient with respect to z is WRITTEN to gz. */
static void exp_adjoint(const double *z, const double *E, double *gE, int d, int N, double *gz)
{
    for (int j = 0; j < d; ++j) gz[j] = 0.0;
    for (int k = N; k >= 2; --k) {
        const double *prev = E + level_offset(d, k - 1);
        double *g_prev = gE + level_offset(d, k - 1);
        const double *g_cur = gE + level_offset(d, k);
        const int64_t n_prev = ipow64(d, k - 1);
        const double div = (double)k;
        for (int64_t w = 0; w < n_prev; ++w)
            for (int j = 0; j < d; ++j) {
                const double g = g_cur[w * d + j];
                g_prev[w] += g * z[j] / div;
                gz[j] += g * prev[w] / div;
            }
    }
    for (int j = 0; j < d; ++j) gz[j] += gE[j];
}

static int one_path_backward(const double *x, const double *gout, int64_t L, int d, int N, int stream, int basepoint,
                             double *gx, int64_t S)
{
    const int64_t n_inc = basepoint ? L : L - 1;
    double *z = (double *)malloc(sizeof(double) * (size_t)(n_inc * d));
    double *A = (double *)calloc((size_t)((n_inc + 1) * S), sizeof(double)); /* A[s] = signature after s increments; A[0] = identity = 0 */
    double *E = (double *)malloc(sizeof(double) * (size_t)(n_inc * S));
    double *gA = (double *)calloc((size_t)S, sizeof(double));
    double *gA_prev = (double *)malloc(sizeof(double) * (size_t)S);
    double *gE = (double *)malloc(sizeof(double) * (size_t)S);
    double *gz = (double *)malloc(sizeof(double) * (size_t)d);
    if (!z || !A || !E || !gA || !gA_prev || !gE || !gz) {
        free(z); free(A); free(E); free(gA); free(gA_prev); free(gE); free(gz);
        return 1;
    }
    /* forward, everything kept */
    for (int64_t s = 0; s < n_inc; ++s) {
        for (int c = 0; c < d; ++c) {
            double hi, lo;
            if (basepoint) {
                hi = x[s * d + c];
                lo = (s == 0) ? 0.0 : x[(s - 1) * d + c];
            } else {
                hi = x[(s + 1) * d + c];
                lo = x[s * d + c];
            }
            z[s * d + c] = hi - lo;
        }
        sig_oracle_exp(z + s * d, d, N, E + s * S);
        sig_oracle_mul(A + s * S, E + s * S, d, N, A + (s + 1) * S);
    }
    /* backward */
    for (int64_t i = 0; i < L * d; ++i) gx[i] = 0.0;
    if (!stream) memcpy(gA, gout, sizeof(double) * (size_t)S);
    for (int64_t s = n_inc - 1; s >= 0; --s) {
        if (stream) { /* entry s of the output is A[s+1] */
            const double *g = gout + s * S;
            for (int64_t w = 0; w < S; ++w) gA[w] += g[w];
        }
        memset(gA_prev, 0, sizeof(double) * (size_t)S);
        memset(gE, 0, sizeof(double) * (size_t)S);
        mul_adjoint(A + s * S, E + s * S, gA, d, N, gA_prev, gE);
        exp_adjoint(z + s * d, E + s * S, gE, d, N, gz);
        for (int c = 0; c < d; ++c) {
            if (basepoint) {
                gx[s * d + c] += gz[c];
                if (s > 0) gx[(s - 1) * d + c] -= gz[c];
            } else {
                gx[(s + 1) * d + c] += gz[c];
                gx[s * d + c] -= gz[c];
            }
        }
        double *t = gA; gA = gA_prev; gA_prev = t;
    }
    free(z); free(A); free(E); free(gA); free(gA_prev); free(gE); free(gz);
    return 0;
}

/* Batched gradient, host pointers, fp64.
 *   path: [B][L][d];  grad_out: same shape as the forward output ([B][S] or [B][n_inc][S]);
 *   grad_path: [B][L][d], overwritten with d(loss)/d(path) where d(loss)/d(output) = grad_out.
 * Same argument checks and return codes as sig_oracle_forward_f64. */
int sig_oracle_backward_f64(const double *path, const double *grad_out, int64_t B, int64_t L, int d, int N,
                            int stream, int basepoint, double *grad_path, int num_threads)
{
    const int64_t S = sig_oracle_channels(d, N);
    if (S < 0 || B < 0) return 1;
    if (basepoint ? (L < 1) : (L < 2)) return 1;
    if (B == 0) return 0;
    if (!path || !grad_out || !grad_path) return 1;
    const int64_t n_inc = basepoint ? L : L - 1;
    const int64_t out_stride = stream ? n_inc * S : S;
    int failed = 0;
#ifdef _OPENMP
    if (num_threads > 0) omp_set_num_threads(num_threads);
#else
    (void)num_threads;
#endif
#pragma omp parallel for schedule(dynamic, 1) reduction(| : failed)
    for (int64_t b = 0; b < B; ++b)
        failed |= one_path_backward(path + b * L * d, grad_out + b * out_stride, L, d, N, stream, basepoint,
                                    grad_path + b * L * d, S);
    return failed ? 2 : 0;
}

/* ------------------------------------------------------------------------------------------
 * Logarithm in the truncated tensor algebra (section 2.3, eq. "logarithm"): the inverse of the
 * tensor exponential, given by the power series  log(1 + x) = sum_{m=1..N} (-1)^{m+1} x^{[x] m} / m,
 * where x is the element without its constant term 1 (powers beyond N vanish in the truncation).
 * Written out literally: every power by one more product with x, every term added in turn.
 * ------------------------------------------------------------------------------------------ */

/* Product of two elements WITHOUT constant terms: C_k = sum_{j=1..k-1} A_j (x) B_{k-j}. */
static void mul_no_unit(const double *A, const double *B, int d, int N, double *C)
{
    const int64_t S = sig_oracle_channels(d, N);
    for (int64_t i = 0; i < S; ++i) C[i] = 0.0;
    for (int k = 2; k <= N; ++k)
        for (int j = 1; j <= k - 1; ++j) {
            const int m = k - j;
            const double *Aj = A + level_offset(d, j);
            const double *Bm = B + level_offset(d, m);
            double *Ck = C + level_offset(d, k);
            const int64_t n_j = ipow64(d, j), n_m = ipow64(d, m);
            for (int64_t u = 0; u < n_j; ++u)
                for (int64_t v = 0; v < n_m; ++v) Ck[u * n_m + v] += Aj[u] * Bm[v];
        }
}

/* out = log(1 + x) for one element x (S scalars, constant term implicit).  Returns 0, or 2 if memory ran out. */
int sig_oracle_log(const double *x, int d, int N, double *out)
{
    const int64_t S = sig_oracle_channels(d, N);
    if (S < 0) return 1;
    double *power = (double *)malloc(sizeof(double) * (size_t)S);
    double *next = (double *)malloc(sizeof(double) * (size_t)S);
    if (!power || !next) {
        free(power); free(next);
        return 2;
    }
    memcpy(power, x, sizeof(double) * (size_t)S);   /* x^1 */
    for (int64_t i = 0; i < S; ++i) out[i] = x[i];
    for (int m = 2; m <= N; ++m) {
        mul_no_unit(power, x, d, N, next);           /* x^m = x^{m-1} [x] x */
        double *t = power; power = next; next = t;
        const double sign = (m % 2 == 0) ? -1.0 : 1.0;
        const double div = (double)m;
        for (int64_t i = 0; i < S; ++i) out[i] += sign * power[i] / div;
    }
    free(power); free(next);
    return 0;
}

/* Adjoint of mul_no_unit: C = A * B (no constant terms), gC given; ADDS into gA and gB. */
static void mul_no_unit_adjoint(const double *A, const double *B, const double *gC, int d, int N, double *gA, double *gB)
{
    for (int k = 2; k <= N; ++k)
        for (int j = 1; j <= k - 1; ++j) {
            const int m = k - j;
            const double *gk = gC + level_offset(d, k);
            const int64_t off_j = level_offset(d, j), off_m = level_offset(d, m);
            const int64_t n_j = ipow64(d, j), n_m = ipow64(d, m);
            for (int64_t u = 0; u < n_j; ++u)
                for (int64_t v = 0; v < n_m; ++v) {
                    const double g = gk[u * n_m + v];
                    gA[off_j + u] += g * B[off_m + v];
                    gB[off_m + v] += A[off_j + u] * g;
                }
        }
}

/* Gradient through sig_oracle_log (the chain rule over its own steps; section 5.3 treats the logarithm as one more
 * differentiable primitive): given g = dLoss/d log(1 + x), WRITES gx = dLoss/dx.  Every power x^m is kept, then the
 * loop of sig_oracle_log is walked backwards.  Returns 0, or 2 if memory ran out. */
int sig_oracle_log_backward(const double *x, const double *g, int d, int N, double *gx)
{
    const int64_t S = sig_oracle_channels(d, N);
    if (S < 0) return 1;
    double *powers = (double *)malloc(sizeof(double) * (size_t)S * (size_t)N);   /* powers[m-1] = x^m */
    double *g_pow = (double *)calloc((size_t)S, sizeof(double));                 /* cotangent of the current power */
    double *g_prev = (double *)calloc((size_t)S, sizeof(double));
    if (!powers || !g_pow || !g_prev) {
        free(powers); free(g_pow); free(g_prev);
        return 2;
    }
    memcpy(powers, x, sizeof(double) * (size_t)S);
    for (int m = 2; m <= N; ++m) mul_no_unit(powers + (size_t)(m - 2) * S, x, d, N, powers + (size_t)(m - 1) * S);
    for (int64_t i = 0; i < S; ++i) gx[i] = 0.0;
    /* out = sum_m sign_m x^m / m: the cotangent of x^m is sign_m g / m plus what x^{m+1} = x^m * x sends back */
    for (int m = N; m >= 1; --m) {
        const double sign = (m % 2 == 0) ? -1.0 : 1.0;
        const double div = (double)m;
        for (int64_t i = 0; i < S; ++i) g_pow[i] += sign * g[i] / div;
        if (m == 1) break;
        for (int64_t i = 0; i < S; ++i) g_prev[i] = 0.0;
        mul_no_unit_adjoint(powers + (size_t)(m - 2) * S, x, g_pow, d, N, g_prev, gx);
        double *t = g_pow; g_pow = g_prev; g_prev = t;
    }
    for (int64_t i = 0; i < S; ++i) gx[i] += g_pow[i];   /* x^1 = x */
    free(powers); free(g_pow); free(g_prev);
    return 0;
}

/* Threads an OpenMP region would use right now (1 when built without OpenMP). */
int sig_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
