/*
 * libsig — truncated signature transform of batched piecewise-linear paths on one
 * AMD MI355X (gfx950).  C ABI: plain pointers and sizes, no C++ or framework types.
 *
 * The transform (paper, section 2.1 definitions 2 and 4, and section 2.2): a sequence
 * x_1..x_L in R^d is read as the continuous piecewise-affine path through its points, and
 *     Sig^N(x) = exp(x_2 - x_1) [x] exp(x_3 - x_2) [x] ... [x] exp(x_L - x_{L-1}),
 * an element of prod_{k=1..N} (R^d)^{(x)k}.  The library folds the increments in one at a
 * time with the fused multiply-exponentiate A <- A [x] exp(z) of section 4.1 (appendix
 * A.1.2, eq. "fusedterm"), levels updated highest first so the update is in place.
 *
 * Layout of one signature: S = sum_{k=1..N} d^k scalars (section 2.4); levels k = 1..N
 * concatenated (the constant k = 0 term is omitted, footnote of section 2.1); inside level
 * k the coefficient of e_{i_1} (x) ... (x) e_{i_k} is at row-major offset
 * sum_m i_m d^{k-m} (0-based letters, first letter slowest) — lexicographic word order
 * under the identification of appendix A.2.2.
 *
 * All functions but one are thread-safe and keep no state between calls.  Nothing here allocates
 * or frees device memory: the calls that need scratch memory (sig_backward, sig_backward_chunked, sig_forward_chunked,
 * sig_combine_many, sig_combine_backward, sig_combine_grouped_backward, sig_log_backward) take a workspace
 * from the caller, sized by their *_workspace_bytes companions; the exception is
 * sig_forward_chunked_static, whose scratch is an array inside the library that all its calls on a GPU
 * share.  Nothing synchronises the device.
 */
#ifndef SIG_H_
#define SIG_H_

#include <stdint.h>
#include <hip/hip_runtime_api.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SIG_OK = 0,
    SIG_ERR_INVALID_ARG = 1,  /* null pointer, negative size, d < 1, N < 1, too few points, bad enum */
    SIG_ERR_UNSUPPORTED = 2,  /* valid request that no kernel variant can serve */
    SIG_ERR_OVERFLOW = 3,     /* a size does not fit the library's 64-bit index budget */
    SIG_ERR_HIP = 4,          /* the HIP runtime refused the launch */
    SIG_ERR_TOO_LARGE = 5     /* sig_forward_chunked_static only: the request needs more than SIG_STATIC_SCRATCH_BYTES */
} sig_status;

typedef enum {
    SIG_F32 = 0,  /* path and out are float; arithmetic in fp32 */
    SIG_F64 = 1   /* path and out are double; arithmetic in fp64 */
} sig_dtype;

/* Which kernel family serves a call.  SIG_VARIANT_AUTO picks the fastest one that
 * supports the shape; the others force one family (SIG_ERR_UNSUPPORTED if it cannot
 * serve the shape) and exist so that every family can be tested on every shape. */
typedef enum {
    SIG_VARIANT_AUTO = 0,
    SIG_VARIANT_GENERIC = 1,  /* any d, N, dtype: one workgroup per path, state in LDS or in `out` */
    SIG_VARIANT_MFMA = 2,     /* fp32, final mode, state in registers, outer products on the matrix cores:
                                 d = 4, N = 4..6 (one wavefront per path); d = 8, N = 4..6 (64 wavefronts per
                                 path); d = 16, N = 4 (8 wavefronts per path) */
    SIG_VARIANT_MFMA_SHARD = 3,/* fp32, d = 4, N = 4..7, final and stream mode: four independent wavefronts
                                 per path, one per first letter */
    SIG_VARIANT_SMALL = 4,    /* any dtype and mode, S <= 512, N <= 8, d <= 64: one wavefront per path, state in LDS */
    SIG_VARIANT_TREE = 5,     /* any dtype and mode; d = 2..8 at N = 2..9: a thread per word of N-2 letters; d = 9..16 at
                                 N = 2..6: a thread per word of N-1 letters; state in registers, any number of
                                 workgroups per path (large signatures, few paths) */
    SIG_VARIANT_MFMA_STREAM = 6,/* fp32, d = 4, N = 4..6, stream mode only: the four first-letter wavefronts of a path in
                                 one workgroup; prefix signatures are assembled in LDS and written out in whole runs
                                 cut at 128-byte boundaries (what sig_forward picks for outputs beyond ~300 MB) */
    SIG_VARIANT_WIDE = 8,     /* any dtype and mode, any d >= 2 at N = 2..9 up to 2^28 words of N-1 letters (what serves
                                 d > 16, and d = 9..16 beyond depth 6): a thread per word of
                                 N-1 letters and block of 16 last letters, channel count a run-time value */
    SIG_VARIANT_DEPTH2 = 9,   /* any dtype, final mode, N = 2, d <= 1024: level 2 as a contraction over the increments,
                                 a thread per 4 x 4 block of coefficients, no scan (what serves N = 2 in final mode) */
    SIG_VARIANT_ROW_STREAM = 7 /* any dtype and mode, d = 2..16 where a lane per word of P letters (d^P <= 64)
                                 leaves one level below it, or two up to d = 8 (d = 8: N = 2..4; d = 3: N = 3..5;
                                 d = 2: N = 4..8; d = 9..16: N = 2): a wavefront per row or few rows, state in registers,
                                 prefix signatures assembled in LDS and written as whole rows */
} sig_variant;

/* Largest depth the kernels accept. */
#define SIG_MAX_DEPTH 32

/* Number of scalars in one depth-N signature over R^d: S(d, N) = sum_{k=1..N} d^k
 * (section 2.4).  Returns -1 if d < 1, N < 1, N > SIG_MAX_DEPTH or S exceeds 2^40. */
int64_t sig_signature_channels(int d, int N);

/* Number of scalars `sig_forward` writes: B*S (stream == 0) or B*n_inc*S (stream != 0),
 * n_inc = L - 1, or L with basepoint.  Returns -1 on invalid arguments (as sig_forward)
 * or if the count exceeds 2^60. */
int64_t sig_output_elems(int64_t B, int64_t L, int d, int N, int stream, int basepoint);

/* Multiply-adds in one fused multiply-exponentiate, M(d, N) = sum_{i=2..N} (N-i+1) d^i:
 * eq. "fusedterm" spends d^2 + ... + d^k of them on level k (appendix A.1.2).  The paper's
 * multiplication count is F(d, N) = M(d, N) + d(N-1) (eq. "fusedresult").  -1 on bad args. */
int64_t sig_fused_fmas(int d, int N);

/* Batched forward signature.
 *
 *   path       DEVICE pointer, [B][L][d] contiguous row-major, element type `dtype`; read only.
 *   B, L, d, N batch, points per path, channels, depth.
 *   stream     0: out is [B][S], the signature of each whole path.
 *              1: out is [B][n_inc][S]; entry j is the signature of the first j+2 points
 *                 (first j+1 points after the basepoint, if basepoint != 0): the expanding
 *                 intervals of section 5.5, all by-products of the same scan (eq. "iterative").
 *   basepoint  0: n_inc = L - 1 increments x_{l+1} - x_l.
 *              1: the origin of R^d is prepended as an extra first point, n_inc = L
 *                 (this library's reading of the `basepoint` argument of section 5.5).
 *   dtype      SIG_F32 or SIG_F64.
 *   out        DEVICE pointer, caller-allocated, sig_output_elems(...) elements of `dtype`,
 *              fully overwritten; must not overlap `path`.
 *              For `path` and `out` any alignment natural for `dtype` is accepted; 16-byte
 *              alignment of both lets the fastest kernels serve the call.
 *   hip_stream the work is enqueued on this stream; the call returns without waiting.
 *
 * The caller owns both buffers and must keep them alive until the stream has passed the
 * enqueued work.  Returns SIG_OK, or an error code with nothing enqueued and `out`
 * untouched: SIG_ERR_INVALID_ARG for null pointers (with B > 0), B < 0, d < 1, N < 1 or
 * N > SIG_MAX_DEPTH, L < 2 (L < 1 with basepoint), an unknown dtype; SIG_ERR_OVERFLOW if a
 * size overflows; SIG_ERR_HIP if the launch failed.  B == 0 is SIG_OK and enqueues nothing.
 * Results are deterministic: the same inputs give bit-identical outputs on every call.
 * In final mode sig_forward scans every path (or every word-prefix shard of it) from end to end and never splits a
 * path over its length, since it has no workspace for partial results: a few very long paths (B * shards far below
 * the number of compute units, L in the tens of thousands) are served many times faster by sig_forward_chunked
 * (sig_forward_chunks_hint says when, and into how many chunks).  In stream mode the output itself has room for
 * partial results, and up to 512 paths of at least 128 increments are cut into chunks internally where the kernel
 * family gains from it (everything but the d = 4 matrix-core kernels); the values then differ from an end-to-end
 * scan by rounding only, and `out` is read as well as written while the call runs. */
sig_status sig_forward(const void *path, int64_t B, int64_t L, int d, int N,
                       int stream, int basepoint, sig_dtype dtype,
                       void *out, hipStream_t hip_stream);

/* As sig_forward, with the kernel family chosen by the caller (see sig_variant). */
sig_status sig_forward_variant(const void *path, int64_t B, int64_t L, int d, int N,
                               int stream, int basepoint, sig_dtype dtype,
                               void *out, hipStream_t hip_stream, sig_variant variant);

/* sig_forward (final mode) as a parallel reduction over the length of the path (section 5.1: the scan is a
 * reduction with respect to an associative operation, so it may be split into chunks): every path is cut into
 * `chunks` stretches of ceil(n_inc / chunks) increments, all B * chunks stretches are scanned at once by the
 * kernels of sig_forward, and neighbouring results are joined pairwise by sig_combine's product (Chen's identity,
 * eq. "grouplike") in log2(chunks) rounds.  Worth it when B alone cannot fill the device and L is long.
 * At depth 2 nothing is multiplied: level 2 is a plain sum over the increments of (midpoint - first point) (x)
 * increment (sections 2.1, 2.2), so every stretch adds up its own terms and a second launch adds the stretches.
 *   chunks     a power of two, 2 .. 65536 (stretches past the end of a short path are empty and count as the
 *              identity).
 *   basepoint_value  as for sig_signature.
 *   workspace  DEVICE pointer, 16-byte aligned, at least sig_forward_chunked_workspace_bytes(...) bytes
 *              (1.5 * B * chunks signatures); contents undefined on return; calls that overlap in time must not
 *              share it.
 * Same result as sig_forward up to rounding.  Errors as for sig_forward; SIG_ERR_INVALID_ARG for a bad `chunks` or a
 * missing, short or misaligned workspace; SIG_ERR_UNSUPPORTED if S >= 2^31. */
sig_status sig_forward_chunked(const void *path, int64_t B, int64_t L, int d, int N, int basepoint,
                               const void *basepoint_value, int chunks, sig_dtype dtype, void *out,
                               void *workspace, int64_t workspace_bytes, hipStream_t hip_stream);

/* Bytes of workspace sig_forward_chunked needs; -1 on invalid arguments. */
int64_t sig_forward_chunked_workspace_bytes(int64_t B, int64_t L, int d, int N, int basepoint, int chunks, sig_dtype dtype);

/* How many chunks sig_forward_chunked should be given for this call, or 1 where plain sig_forward is the faster
 * one (host arithmetic only, nothing is launched).  Chunking pays for few, long paths: at most 64 paths of at least
 * 512 increments (4096 at d = 8, N = 4..6 in fp32, whose kernels already spread a path over 64 wavefronts); measured:
 * B = 1, L = 65536, d = 4, N = 6 takes 6.5 ms plain and 0.09 ms in 512 chunks.  The hint is the largest power of two
 * that leaves every stretch at least 64 increments, keeps B * chunks within 1024 stretches and their signatures
 * within 256 MiB (the products that join them move every one of them).  At depth 2 (a sum, two launches of about
 * 22 us in all): up to 1024 paths, from 24 staged tiles of increments on (3072 increments up to 28 channels, 1512 at
 * 64), stretches of at least 128 increments, 2048 at most; B = 1, L = 131073, d = 64 takes 7.8 ms plain and 0.03 to
 * 0.07 ms cut into 256 to 1024 stretches.  0 on invalid arguments. */
int sig_forward_chunks_hint(int64_t B, int64_t L, int d, int N, int basepoint, sig_dtype dtype);

/* Size of the scratch array built into the library for sig_forward_chunked_static: 32 MiB of device memory that
 * every GPU the library runs on holds from the moment the library is loaded until the process ends. */
#define SIG_STATIC_SCRATCH_BYTES (32 * 1024 * 1024)

/* sig_forward_chunked for callers that can neither allocate device memory nor hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical
 * results; the chunk signatures and the partial products live in the library's own fixed scratch array instead of a
 * caller's workspace.  The call allocates and frees nothing and calls no allocating routine.
 *   Limit: sig_forward_chunked_workspace_bytes(...) for the same arguments must not exceed
 *          SIG_STATIC_SCRATCH_BYTES (= sig_forward_chunked_static_max_bytes()), else SIG_ERR_TOO_LARGE with nothing
 *          enqueued and `out` untouched.
 *   Device: the scratch array used is the one of the device that is current at the call, which must be the device
 *          of `path`, `out` and `hip_stream`.  Its address is looked up once per device, on the first call made with
 *          that device current (that first call is therefore not a call to make under graph capture).
 *   Sharing: all calls on one GPU use the same array, which keeps the previous call's contents (every scalar a call
 *          reads it has written first, so nothing needs clearing).  Calls that overlap in time on one GPU (two
 *          streams, two threads) race on it: serialise them, or use sig_forward_chunked with separate workspaces.
 * Other errors as for sig_forward_chunked; SIG_ERR_HIP also if the array's address cannot be obtained. */
sig_status sig_forward_chunked_static(const void *path, int64_t B, int64_t L, int d, int N, int basepoint,
                                      const void *basepoint_value, int chunks, sig_dtype dtype, void *out,
                                      hipStream_t hip_stream);

/* SIG_STATIC_SCRATCH_BYTES as the library was built. */
int64_t sig_forward_chunked_static_max_bytes(void);

/* Group product of two batches of signatures: out[b] = a[b] [x] b[b], with
 * (A [x] B)_k = sum_{j=0..k} A_j (x) B_{k-j}, A_0 = B_0 = 1 (section 2.2).  By Chen's identity
 * (eq. "grouplike") this joins the signatures of two adjacent intervals that share their
 * boundary point, Sig(x_1..x_L) = Sig(x_1..x_j) [x] Sig(x_j..x_L), without going back to the data
 * (section 5.5, "combining adjacent intervals").
 *
 *   a, b, out  DEVICE pointers, [B][S] contiguous, S = sig_signature_channels(d, N), element type
 *              `dtype`; `out` is fully overwritten and must not overlap `a` or `b`.
 * Enqueued on `hip_stream`, no wait.  Errors as for sig_forward (SIG_ERR_UNSUPPORTED if S >= 2^31). */
sig_status sig_combine(const void *a, const void *b, int64_t B, int d, int N, sig_dtype dtype,
                       void *out, hipStream_t hip_stream);

/* As sig_combine, for signatures that are not packed: signature p of `a` starts at a + p * a_stride scalars
 * (likewise b, out; a stride of 0 repeats one signature for every p).  out_stride >= S; `out` must not overlap
 * the inputs.  With a = the inverted signatures of the prefixes x_1..x_i of a path and b = the signatures of its
 * prefixes x_1..x_j, both rows of stream-mode outputs, this answers Sig(x_i..x_j) in one product, independent of
 * the length of the path (section 4.2). */
sig_status sig_combine_strided(const void *a, int64_t a_stride, const void *b, int64_t b_stride, int64_t B, int d, int N,
                               sig_dtype dtype, void *out, int64_t out_stride, hipStream_t hip_stream);

/* Group product of n signatures per batch row, in order: out[b] = sigs[b][0] [x] sigs[b][1] [x] ... [x] sigs[b][n-1]
 * (section 5.5, "combining adjacent intervals": the signatures of n consecutive intervals, each starting at the
 * point where the one before ends, joined without going back to the data).  Neighbours are multiplied pairwise in
 * ceil(log2 n) rounds.
 *   sigs       DEVICE pointer [B][n][S]; read only.   out  DEVICE pointer [B][S]; must not overlap `sigs`.
 *   workspace  DEVICE pointer, 16-byte aligned, at least sig_combine_many_workspace_bytes(...) bytes (0 for n <= 2,
 *              then it may be NULL); contents undefined on return.
 * Errors as for sig_combine; n < 1 and a missing or short workspace are SIG_ERR_INVALID_ARG. */
sig_status sig_combine_many(const void *sigs, int64_t B, int64_t n, int d, int N, sig_dtype dtype, void *out,
                            void *workspace, int64_t workspace_bytes, hipStream_t hip_stream);

/* Bytes of workspace sig_combine_many needs; -1 on invalid arguments. */
int64_t sig_combine_many_workspace_bytes(int64_t B, int64_t n, int d, int N, sig_dtype dtype);

/* Gradient through sig_combine (section 5.3: every operation is differentiable): given
 * grad_out = dLoss/d(a [x] b), writes grad_a = dLoss/da and grad_b = dLoss/db,
 *   grad_a[u] = grad_out[u] + sum_v grad_out[u v] b[v],   grad_b[v] = grad_out[v] + sum_u a[u] grad_out[u v]
 * (u v: a word cut into a non-empty prefix and a non-empty suffix).  Deterministic (no atomics).
 *   a, b, grad_out  DEVICE pointers [B][S], read only.   grad_a, grad_b  DEVICE pointers [B][S], overwritten; they
 *              must differ from each other and from the inputs.
 *   workspace  DEVICE pointer, 16-byte aligned, at least sig_combine_backward_workspace_bytes(...) bytes (0 for
 *              N = 1, then it may be NULL); contents undefined on return.
 * Errors as for sig_combine; a missing, short or misaligned workspace is SIG_ERR_INVALID_ARG. */
sig_status sig_combine_backward(const void *a, const void *b, const void *grad_out, int64_t B, int d, int N, sig_dtype dtype,
                                void *grad_a, void *grad_b, void *workspace, int64_t workspace_bytes, hipStream_t hip_stream);

/* Bytes of workspace sig_combine_backward needs; -1 on invalid arguments or S >= 2^31. */
int64_t sig_combine_backward_workspace_bytes(int64_t B, int d, int N, sig_dtype dtype);

/* One left factor for a group of right factors: out[b][s] = a[b] [x] sigs[b][s], s < group.  This is what `initial`
 * does to a stream-mode output (section 5.5, "keeping the signature up-to-date": a[b] the signature of what came
 * before, sigs[b][s] the signatures of the prefixes of path b), offered on its own so that the prefix signatures
 * themselves remain available, which the gradient below needs.
 *   a          DEVICE pointer [B][S]; read only.
 *   sigs, out  DEVICE pointers [B][group][S]; `out` may be `sigs` itself (in place) but must not overlap it otherwise.
 * Errors as for sig_combine; group < 1 is SIG_ERR_INVALID_ARG. */
sig_status sig_combine_grouped(const void *a, const void *sigs, int64_t B, int64_t group, int d, int N, sig_dtype dtype,
                               void *out, hipStream_t hip_stream);

/* Gradient through sig_combine_grouped (section 5.3; with it `initial` is differentiable in stream mode as well):
 *   grad_sigs[b][s] as grad_b of sig_combine_backward for the product a[b] [x] sigs[b][s];
 *   grad_a[b] = the sum over s, in the order of s, of what sig_combine_backward gives as grad_a for those products.
 *   a  DEVICE [B][S];  sigs, grad_out  DEVICE [B][group][S]; read only.
 *   grad_a  DEVICE [B][S], grad_sigs  DEVICE [B][group][S]: overwritten; must differ from each other and the inputs.
 *   workspace  DEVICE pointer, 16-byte aligned, at least sig_combine_grouped_backward_workspace_bytes(...) bytes (it
 *              holds one signature per product besides the partial sums); contents undefined on return.
 * Errors as for sig_combine_backward. */
sig_status sig_combine_grouped_backward(const void *a, const void *sigs, const void *grad_out, int64_t B, int64_t group, int d,
                                        int N, sig_dtype dtype, void *grad_a, void *grad_sigs, void *workspace,
                                        int64_t workspace_bytes, hipStream_t hip_stream);

/* Bytes of workspace sig_combine_grouped_backward needs; -1 on invalid arguments or S >= 2^31. */
int64_t sig_combine_grouped_backward_workspace_bytes(int64_t B, int64_t group, int d, int N, sig_dtype dtype);

/* Group inverse of `rows` signatures: out[r] = sig[r]^{-1}, which is the signature of the same path traversed
 * backwards (section 5.4).  It is a signed permutation of the scalars: level k of the inverse holds
 * (-1)^k times the coefficient of the reversed word.
 *   sig, out   DEVICE pointers, [rows][S]; `out` may be `sig` itself (in place) but must not overlap it otherwise.
 * Errors as for sig_combine. */
sig_status sig_invert(const void *sig, int64_t rows, int d, int N, sig_dtype dtype, void *out, hipStream_t hip_stream);

/* The signature with every option of section 5.5: sig_forward, then
 *   basepoint_value  DEVICE pointer [B][d] or NULL.  With basepoint != 0 the point prepended to path b is
 *              basepoint_value[b] (the origin if NULL); must be NULL when basepoint == 0.  16-byte alignment lets
 *              the fastest kernels serve the call.
 *   initial    DEVICE pointer [B][S] or NULL: the signature of the data that came before this path (whose last
 *              point is this path's first point, or its basepoint).  The result is initial [x] Sig(path), in stream
 *              mode for every prefix: the signature of everything so far (section 5.5, "keeping the signature
 *              up-to-date").  Applied by one product per output signature, in place, after the scan.
 *   inverse    != 0: every signature written is replaced by its group inverse (section 5.4), after `initial` has
 *              been applied; `initial` itself is always a plain (not inverted) signature.
 * Everything else, and the errors, as for sig_forward; with `initial` or `inverse`, S must be below 2^31. */
sig_status sig_signature(const void *path, int64_t B, int64_t L, int d, int N, int stream, int basepoint,
                         const void *basepoint_value, const void *initial, int inverse, sig_dtype dtype,
                         void *out, hipStream_t hip_stream);

/* Logarithm in the truncated tensor algebra of `rows` signatures (section 2.3, eq. "logarithm"): with x the
 * signature without its constant term, log(1 + x) = sum_{m=1..N} (-1)^{m+1} x^{[x] m} / m.  The result has the
 * same layout as a signature (every word kept).
 *   sig, out   DEVICE pointers, [rows][S]; must not overlap (and must differ).
 * Errors as for sig_combine. */
sig_status sig_log(const void *sig, int64_t rows, int d, int N, sig_dtype dtype, void *out, hipStream_t hip_stream);

/* Number of Lyndon words of length 1..N over d letters = the dimension w(d, N) of the logsignature (Witt's formula,
 * section 2.3).  -1 on bad arguments or if S >= 2^31. */
int64_t sig_logsignature_channels(int d, int N);

/* Offsets, inside a flat depth-N element, of the coefficients of the Lyndon words (appendix A.2.1: the words that
 * come strictly before all of their rotations), ordered by length and lexicographically inside a length.
 *   indices    HOST pointer to `capacity` >= sig_logsignature_channels(d, N) entries, filled on return.
 * A host function: nothing is enqueued.  SIG_ERR_INVALID_ARG if the capacity is too small. */
sig_status sig_lyndon_indices(int d, int N, int64_t *indices, int64_t capacity);

/* Logsignature in the basis of appendix A.2.4, psi(log(Sig)): from the logarithms computed by sig_log, keep the
 * coefficients of the Lyndon words.  out[r][i] = log_sig[r][indices[i]].
 *   log_sig    DEVICE pointer [rows][S];  indices  DEVICE pointer to n offsets in [0, S) (sig_lyndon_indices, copied
 *              to the device by the caller);  out  DEVICE pointer [rows][n].
 * Errors as for sig_combine. */
sig_status sig_lyndon_gather(const void *log_sig, int64_t rows, int d, int N, const int64_t *indices, int64_t n,
                             sig_dtype dtype, void *out, hipStream_t hip_stream);

/* Gradient through sig_log (section 5.3 treats every operation as a differentiable primitive; the paper's
 * benchmarks time the logsignature backwards as well): given grad_log = dLoss/d sig_log(sig), writes
 * grad_sig = dLoss/d sig.  Deterministic: partial sums are added in a fixed order, no atomics.
 *   sig, grad_log  DEVICE pointers [rows][S], read only.   grad_sig  DEVICE pointer [rows][S], overwritten; must
 *              not overlap the other two.
 *   workspace  DEVICE pointer, 16-byte aligned, at least sig_log_backward_workspace_bytes(...) bytes (0 for N = 1
 *              and for signatures small enough for the single-launch kernel; then it may be NULL); contents
 *              undefined on return.
 * Errors as for sig_combine; a missing, short or misaligned workspace is SIG_ERR_INVALID_ARG. */
sig_status sig_log_backward(const void *sig, const void *grad_log, int64_t rows, int d, int N, sig_dtype dtype,
                            void *grad_sig, void *workspace, int64_t workspace_bytes, hipStream_t hip_stream);

/* Bytes of workspace sig_log_backward needs; -1 on invalid arguments or S >= 2^31. */
int64_t sig_log_backward_workspace_bytes(int64_t rows, int d, int N, sig_dtype dtype);

/* Transpose of sig_lyndon_gather: grad_log[r][indices[i]] = grad_logsig[r][i], every other scalar of grad_log 0
 * (the words that are not Lyndon words do not reach the logsignature, appendix A.2.4).
 *   grad_logsig  DEVICE pointer [rows][n];  indices  DEVICE pointer to n distinct offsets in [0, S);
 *   grad_log     DEVICE pointer [rows][S], overwritten.
 * Errors as for sig_lyndon_gather. */
sig_status sig_lyndon_scatter(const void *grad_logsig, int64_t rows, int d, int N, const int64_t *indices, int64_t n,
                              sig_dtype dtype, void *grad_log, hipStream_t hip_stream);

/* Gradient of a scalar loss with respect to the path, given its gradient with respect to the output of
 * sig_forward (or sig_signature without `initial` and `inverse`) called with the same arguments (section 5.3;
 * appendix C).  Nothing from the forward pass is kept but its output: each earlier signature is recovered from the
 * next one by undoing the increment between them (appendix C.1, reversibility, eq. "reverse"), and the increment's
 * gradient comes from the transpose of the fused multiply-exponentiate (section 4.1, eq. "fusedterm").
 *
 *   path       DEVICE pointer, [B][L][d], as given to the forward call; read only.
 *   sig        DEVICE pointer, the forward output for (path, N, stream, basepoint): [B][S], or [B][n_inc][S] in
 *              stream mode; read only.
 *   grad_out   DEVICE pointer, same shape as `sig`: d(loss)/d(output); read only.
 *   basepoint_value  DEVICE pointer [B][d] or NULL: as for sig_signature; only with basepoint != 0.
 *   grad_path  DEVICE pointer, [B][L][d], fully overwritten with d(loss)/d(path); must not overlap the inputs.
 *   grad_basepoint  DEVICE pointer [B][d] or NULL: if given (only with basepoint != 0), receives the gradient with
 *              respect to the basepoint.
 *   workspace  DEVICE pointer to at least sig_backward_workspace_bytes(...) bytes, 16-byte aligned, contents
 *              irrelevant on entry and undefined on return; may be NULL when that size is 0.  Calls that overlap
 *              in time must not share a workspace.
 * Enqueued on `hip_stream`, no wait.  Served: d <= 16 at the depths of the register-resident and prefix-tree
 * kernels; any d at N = 2..9 (up to 204 channels, 102 in fp64; depth 2 in final mode by a closed form up to d = 122,
 * 85 in fp64); everything else with d <= 64 and S < 2^30 on a generic kernel that is two to three orders of
 * magnitude slower per increment; otherwise SIG_ERR_UNSUPPORTED.  Other errors as for sig_forward; a missing or
 * short workspace is SIG_ERR_INVALID_ARG.  Deterministic. */
sig_status sig_backward(const void *path, const void *sig, const void *grad_out, int64_t B, int64_t L, int d, int N,
                        int stream, int basepoint, const void *basepoint_value, sig_dtype dtype, void *grad_path,
                        void *grad_basepoint, void *workspace, int64_t workspace_bytes, hipStream_t hip_stream);

/* Bytes of device workspace sig_backward needs for these arguments on the current device: 0 when the per-path
 * working set (the signature, its cotangent and the Horner terms, about 2.7 S scalars) fits on chip.
 * -1 on invalid or unsupported arguments. */
int64_t sig_backward_workspace_bytes(int64_t B, int64_t L, int d, int N, int stream, int basepoint, sig_dtype dtype);

/* sig_backward in final mode for few long paths (sections 5.1 and 5.3): the walk back along a path, one increment
 * after the other, is cut into at most `chunks` stretches of ceil(n_inc / chunks) increments that are walked at the
 * same time.  The stretches' signatures are computed first; their running products (Chen's identity, section 2.2) are
 * the signatures at the ends of the stretches, and the gradient with respect to each of those follows from the one
 * after it, because a product is linear in its left factor.  The result is that of sig_backward up to rounding; the
 * forward output is not an argument (it is the last of the running products).
 *   path, grad_out, basepoint_value, grad_path, grad_basepoint: as for sig_backward with stream = 0.
 *   chunks     2 .. 65536 (any number; more stretches than increments are not made).
 *   workspace  DEVICE pointer, 16-byte aligned, at least sig_backward_chunked_workspace_bytes(...) bytes, contents
 *              irrelevant on entry and undefined on return; overlapping calls must not share one.
 * Enqueued on `hip_stream` (chunks + 6 launches or so), no wait.  Needs B <= 65535, the stretches' shape served by
 * sig_forward and sig_backward, S < 2^31: otherwise SIG_ERR_UNSUPPORTED; other errors as for sig_backward.
 * Deterministic. */
sig_status sig_backward_chunked(const void *path, const void *grad_out, int64_t B, int64_t L, int d, int N, int basepoint,
                                const void *basepoint_value, int chunks, sig_dtype dtype, void *grad_path, void *grad_basepoint,
                                void *workspace, int64_t workspace_bytes, hipStream_t hip_stream);

/* Bytes of workspace sig_backward_chunked needs (the stretches' points and point gradients, three signatures per
 * stretch, and what sig_backward needs for the stretches); -1 on invalid or unsupported arguments. */
int64_t sig_backward_chunked_workspace_bytes(int64_t B, int64_t L, int d, int N, int basepoint, int chunks, sig_dtype dtype);

/* The number of stretches to give sig_backward_chunked for this shape, a power of two; 1 where sig_backward is the
 * faster call (short paths, many paths, depth below 3); 0 on invalid arguments. */
int sig_backward_chunks_hint(int64_t B, int64_t L, int d, int N, int basepoint, sig_dtype dtype);

/* Name of the kernel family that `variant` resolves to for this shape ("generic",
 * "mfma_d4", ...), or "unsupported" / "invalid".  The string is static. */
const char *sig_variant_name(int64_t B, int64_t L, int d, int N, int stream, int basepoint,
                             sig_dtype dtype, sig_variant variant);

/* Static English text for a status code. */
const char *sig_status_string(sig_status status);

#ifdef __cplusplus
}
#endif

#endif /* SIG_H_ */
