/*
 * fp64 CPU oracle for the truncated signature transform: the entry points of libsig_oracle.so.
 * TEST INFRASTRUCTURE ONLY: the yardstick the HIP library is checked against, in a library of its own so that
 * the product cannot reach it.  Only the tests, the smoke check and the benchmark's cpu_baseline leg call it.
 *
 * All pointers are HOST pointers to fp64 data owned by the caller.  One truncated tensor-algebra element is
 * S = sum_{k=1..N} d^k scalars (section 2.4): levels k = 1..N concatenated, the constant k = 0 term omitted
 * (footnote of section 2.1), inside level k the coefficient of e_{i_1} (x) ... (x) e_{i_k} at row-major offset
 * sum_m i_m d^{k-m} (0-based letters, first letter slowest).
 */
#ifndef SIG_ORACLE_H_
#define SIG_ORACLE_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* S(d, N) = sum_{k=1..N} d^k (section 2.4); -1 for d < 1, N < 1 or more than 2^40 scalars. */
int64_t sig_oracle_channels(int d, int N);

/* Tensor exponential of z in R^d (section 2.2): E_k = z^{(x)k} / k!, built as E_k = (E_{k-1} (x) z) / k with a
 * true division.   z: [d];  E: [S], written. */
void sig_oracle_exp(const double *z, int d, int N, double *E);

/* Group product (section 2.2, appendix eq. "tensorproduct"): C_k = sum_{j=0..k} A_j (x) B_{k-j}, A_0 = B_0 = 1,
 * term by term.   A, B: [S];  C: [S], written, must not alias A or B. */
void sig_oracle_mul(const double *A, const double *B, int d, int N, double *C);

/* Transpose of sig_oracle_mul (section 5.3): given gC = dLoss/dC, WRITES gA = dLoss/dA and gB = dLoss/dB. */
void sig_oracle_mul_backward(const double *A, const double *B, const double *gC, int d, int N, double *gA, double *gB);

/* Batched forward signature (section 2.1 definitions 2 and 4; section 2.2 eq. "computation"):
 *   Sig(x_1..x_L) = exp(x_2 - x_1) [x] ... [x] exp(x_L - x_{L-1}), every exponential formed by sig_oracle_exp and
 *   every product by sig_oracle_mul (the "conventional" route of appendix A.1.1).
 *   path  [B][L][d] row-major.
 *   stream != 0: out is [B][n_inc][S], entry j = the signature after the (j+1)-th increment (section 5.5,
 *          "expanding intervals"); otherwise out is [B][S].
 *   basepoint != 0: the origin is prepended as an extra first point, n_inc = L instead of L - 1 (this build's
 *          reading of the `basepoint` argument named in section 5.5).
 *   num_threads <= 0 lets OpenMP choose (the only parallelism is a loop over the batch).
 * Returns 0, 1 on bad arguments (d < 1, N < 1, B < 0, fewer than two points once the basepoint is counted, null
 * pointers), 2 if memory ran out.
 * The host-side fp64 counterpart of the library's sig_forward (its "host oracle" entry point, sig_forward_host_oracle_f64
 * under another name). */
int sig_oracle_forward_f64(const double *path, int64_t B, int64_t L, int d, int N, int stream, int basepoint,
                           double *out, int num_threads);

/* Gradient of a scalar loss with respect to the path given its gradient with respect to the output of
 * sig_oracle_forward_f64 (section 5.3; appendix C, first paragraph: the chain rule over differentiable primitives).
 * Every intermediate signature and exponential of the forward pass is kept and each primitive's adjoint applied in
 * reverse; no reversibility, no recomputation.
 *   grad_out  shaped like the forward output;  grad_path  [B][L][d], overwritten.
 * Return codes as sig_oracle_forward_f64. */
int sig_oracle_backward_f64(const double *path, const double *grad_out, int64_t B, int64_t L, int d, int N,
                            int stream, int basepoint, double *grad_path, int num_threads);

/* Logarithm in the truncated tensor algebra (section 2.3, eq. "logarithm"):
 * log(1 + x) = sum_{m=1..N} (-1)^{m+1} x^{[x] m} / m, every power by one more literal product.
 *   x, out: [S] (one element; out must not alias x).   Returns 0, 1 on bad d or N, 2 if memory ran out. */
int sig_oracle_log(const double *x, int d, int N, double *out);

/* Gradient through sig_oracle_log (section 5.3): given g = dLoss/d log(1 + x), WRITES gx = dLoss/dx, walking the
 * loop of sig_oracle_log backwards over the stored powers.   Return codes as sig_oracle_log. */
int sig_oracle_log_backward(const double *x, const double *g, int d, int N, double *gx);

/* Threads an OpenMP region would use right now (1 when built without OpenMP). */
int sig_oracle_max_threads(void);

#ifdef __cplusplus
}
#endif

#endif /* SIG_ORACLE_H_ */
