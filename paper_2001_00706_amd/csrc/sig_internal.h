// Internal declarations shared by the translation units of libsig (not part of the C ABI).
#ifndef SIG_INTERNAL_H_
#define SIG_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sig.h"

namespace sig {

// A validated call: sizes, level sizes d^k and level offsets, passed by value to kernels.
struct Shape {
    int64_t B;       // paths
    int64_t L;       // points per path
    int64_t S;       // scalars per signature, sum_{k=1..N} d^k
    int64_t n_inc;   // increments folded in: L - 1, or L with basepoint
    int d, N;
    int stream, basepoint;
    const void *basepoint_value;     // DEVICE [B][d]: the point prepended when basepoint != 0; null = the origin
    // Chunked scans (final mode only): B counts chunks, `chunks` consecutive ones belong to one path of L points
    // and n_inc increments; chunk c folds in the increments c*chunk_len .. min((c+1)*chunk_len, n_inc) - 1 and
    // basepoint_value is indexed by path.  chunks == 1: B counts paths.
    int chunks;
    int64_t chunk_len;
    // Chunked scans whose rows live inside a stream-mode output [paths][n_inc][S] (served by the small-state, prefix-tree,
    // row and many-channel families): with stream == 0 a chunk that has increments writes its signature to the row of its
    // last increment; with stream != 0 a chunk starts from the row before its first increment (the empty signature
    // at the start of a path) and writes the row of every increment of its own but the last.  0: rows are packed.
    int rows_in_stream;
    // Gradient calls: 0 when the signature handed in belongs to a longer path of which the rows are stretches (the
    // walk back then starts from that signature and must not assume that a row's own increments make it up).
    int from_identity;
    int64_t pw[SIG_MAX_DEPTH + 1];   // pw[k] = d^k, k = 0..N
    int64_t off[SIG_MAX_DEPTH + 2];  // off[k] = offset of level k (1-based) in a signature; off[N+1] = S
};

// Which stretch of which path the scan of output row `row` folds in.
struct ChunkView {
    int64_t path;   // index of the path (for the path pointer and the basepoint value)
    int64_t inc0;   // number of its first increment inside that path
    int64_t n;      // increments to fold in (0 for a chunk past the end: its result is the identity)
};

__host__ __device__ inline ChunkView chunk_view(int64_t row, int chunks, int64_t chunk_len, int64_t n_inc_total)
{
    if (chunks <= 1) return {row, 0, n_inc_total};
    const int64_t p = row / chunks;
    const int64_t inc0 = (row - p * chunks) * chunk_len;
    const int64_t left = n_inc_total - inc0;
    return {p, inc0, left < 0 ? 0 : left < chunk_len ? left : chunk_len};
}

// Generic family: any d, N; one workgroup per path.  `generic_supported` is false only when
// the per-step scalings z/1..z/N (N*d scalars) do not fit the workgroup's LDS.
bool generic_supported(const Shape &sh, sig_dtype dtype);
hipError_t launch_generic_f32(const Shape &sh, const float *path, float *out, hipStream_t st);
hipError_t launch_generic_f64(const Shape &sh, const double *path, double *out, hipStream_t st);

// Group product of two batches of signatures (any d, N with S < 2^31).
bool combine_supported(const Shape &sh);
// `strides`: null = packed (S each), else 7 entries {a, b, out, n_inner, a_outer, b_outer, out_outer}: product
// p = q * n_inner + i reads a + q * a_outer + i * a (likewise b, out); n_inner = 0 means no outer level.
hipError_t launch_combine_f32(const Shape &sh, const float *a, const float *b, float *out, hipStream_t st,
                              const int64_t *strides = nullptr);
hipError_t launch_combine_f64(const Shape &sh, const double *a, const double *b, double *out, hipStream_t st,
                              const int64_t *strides = nullptr);

// Inverse of each of sh.B signatures (a signed permutation; `out` may be `in`), and multiplication on the
// left in place: out[r] <- a[r / group] [x] out[r] for sh.B rows.  Both need S < 2^31.
hipError_t launch_invert_f32(const Shape &sh, const float *in, float *out, hipStream_t st);
hipError_t launch_invert_f64(const Shape &sh, const double *in, double *out, hipStream_t st);
// Running product along the chunk ends of a stream-mode output [paths][n_inc][S], in place (sh: d, N and the level
// tables): the last row of every chunk of chunk_len rows is multiplied on the left by the last row of the chunk before.
hipError_t launch_chunk_prefix_f32(const Shape &sh, int64_t paths, int64_t n_inc, int64_t chunk_len, float *out, hipStream_t st);
hipError_t launch_chunk_prefix_f64(const Shape &sh, int64_t paths, int64_t n_inc, int64_t chunk_len, double *out, hipStream_t st);
hipError_t launch_left_mul_f32(const Shape &sh, const float *a, int64_t group, float *out, hipStream_t st);
hipError_t launch_left_mul_f64(const Shape &sh, const double *a, int64_t group, double *out, hipStream_t st);

// Gradient with respect to the path (any N, d <= 64, S < 2^30).  `backward_workspace_bytes` is what the launch
// needs in `workspace` (0 when everything fits LDS, -1 if unsupported).
bool backward_supported(const Shape &sh);
int64_t backward_workspace_bytes(const Shape &sh, sig_dtype dtype);
// `gbase` (may be null): [B][d] gradient of the basepoint, written when sh.basepoint != 0.
hipError_t launch_backward_f32(const Shape &sh, const float *path, const float *sig, const float *gout, float *gpath,
                               float *gbase, void *workspace, int64_t workspace_bytes, hipStream_t st);
hipError_t launch_backward_f64(const Shape &sh, const double *path, const double *sig, const double *gout, double *gpath,
                               double *gbase, void *workspace, int64_t workspace_bytes, hipStream_t st);

// Logarithm of sh.B signatures in the tensor algebra (out != in), the gather of n coefficients per signature by a
// device index table, and that table for the Lyndon words, built on the host (returns the count; `indices` may be
// null to count only; -1 if `cap` is too small).
hipError_t launch_log_f32(const Shape &sh, const float *in, float *out, hipStream_t st);
hipError_t launch_log_f64(const Shape &sh, const double *in, double *out, hipStream_t st);
hipError_t launch_gather_f32(const Shape &sh, const float *in, const int64_t *index, int64_t n, float *out, hipStream_t st);
hipError_t launch_gather_f64(const Shape &sh, const double *in, const int64_t *index, int64_t n, double *out, hipStream_t st);
int64_t lyndon_indices_host(const Shape &sh, int64_t *indices, int64_t cap);

// Plumbing of the gradient computed stretch by stretch (sig_backward_chunked.hip); `sh` is the whole call's shape
// except for the chain, which takes the shape of the B K stretches.  K stretches of m increments per path.
hipError_t launch_stretch_gather(const Shape &sh, sig_dtype dtype, int64_t K, int64_t m, const void *path, void *rows, hipStream_t st);
hipError_t launch_copy_rows(sig_dtype dtype, const void *src, int64_t src_stride, void *dst, int64_t dst_stride, int64_t len,
                            int64_t rows, hipStream_t st);
hipError_t launch_stretch_adjoint_chain(const Shape &sh, sig_dtype dtype, int64_t K, const void *C, void *g, hipStream_t st);
hipError_t launch_stretch_scatter(const Shape &sh, sig_dtype dtype, int64_t K, int64_t m, const void *grows, void *gpath, void *gbase,
                                  hipStream_t st);

// Gradient through the logarithm (sh.B rows; S < 2^31) and through the selection of the Lyndon words.
int64_t log_backward_workspace_bytes(const Shape &sh, sig_dtype dtype);
int64_t combine_backward_workspace_bytes(const Shape &sh, sig_dtype dtype);
hipError_t launch_log_backward_f32(const Shape &sh, const float *sig, const float *grad_log, float *grad_sig, void *workspace,
                                   hipStream_t st);
hipError_t launch_log_backward_f64(const Shape &sh, const double *sig, const double *grad_log, double *grad_sig, void *workspace,
                                   hipStream_t st);
// Gradient of the group product out = a [x] b; workspace: combine_backward_workspace_bytes.
hipError_t launch_combine_backward_f32(const Shape &sh, const float *a, const float *b, const float *g, float *ga, float *gb,
                                       void *workspace, hipStream_t st);
hipError_t launch_combine_backward_f64(const Shape &sh, const double *a, const double *b, const double *g, double *ga, double *gb,
                                       void *workspace, hipStream_t st);
// The same for rows that share their left factor in groups: row r is a[r / group] [x] b[r] (sh.B rows, a multiple of
// `group`); ga has sh.B / group rows, each the sum over its group in row order.  The workspace is that of the plain
// product's gradient, rounded up to 256 bytes, followed by one signature per row.
int64_t combine_grouped_backward_workspace_bytes(const Shape &sh, sig_dtype dtype);
hipError_t launch_combine_grouped_backward_f32(const Shape &sh, int64_t group, const float *a, const float *b, const float *g,
                                               float *ga, float *gb, void *workspace, hipStream_t st);
hipError_t launch_combine_grouped_backward_f64(const Shape &sh, int64_t group, const double *a, const double *b, const double *g,
                                               double *ga, double *gb, void *workspace, hipStream_t st);
hipError_t launch_scatter_f32(const Shape &sh, const float *in, const int64_t *index, int64_t n, float *out, hipStream_t st);
hipError_t launch_scatter_f64(const Shape &sh, const double *in, const int64_t *index, int64_t n, double *out, hipStream_t st);

// Register-resident gradient kernel: fp32, d = 4, N = 4..6, 16-byte aligned buffers; needs no workspace.
bool backward_d4_supported(const Shape &sh);
hipError_t launch_backward_d4_f32(const Shape &sh, const float *path, const float *sig, const float *gout, float *gpath,
                                  float *gbase, hipStream_t st);

// Gradient kernel for d = 16, N = 4, final mode, fp32, 16-byte aligned buffers: one workgroup of 512 threads per path
// with the top level's cotangent in registers; workspace: one gradient per increment, [B][n_inc][16] floats.
bool backward_d16_supported(const Shape &sh);
int64_t backward_d16_workspace_bytes(const Shape &sh);
hipError_t launch_backward_d16_f32(const Shape &sh, const float *path, const float *sig, const float *gout, float *gpath,
                                   float *gbase, void *workspace, int64_t workspace_bytes, hipStream_t st);

// Gradient kernel for d = 4, N = 6, final mode, fp32, 16-byte aligned buffers: one workgroup of 128 threads per path,
// a thread per word of three letters and half of the letters below it, the top level's cotangent in registers;
// workspace: one gradient per increment, [B][n_inc][4] floats.
bool backward_d4n6_supported(const Shape &sh);
int64_t backward_d4n6_workspace_bytes(const Shape &sh);
hipError_t launch_backward_d4n6_f32(const Shape &sh, const float *path, const float *sig, const float *gout, float *gpath,
                                    float *gbase, void *workspace, int64_t workspace_bytes, hipStream_t st);

// The same scheme for d = 2 (N = 2..9) and d = 8 (N = 2..5); buffers aligned to min(d, 4) floats.
bool backward_pow2_supported(const Shape &sh);
hipError_t launch_backward_pow2_f32(const Shape &sh, const float *path, const float *sig, const float *gout, float *gpath,
                                    float *gbase, hipStream_t st);

// Prefix-tree family (d = 2..8 at N = 2..9, d = 9..16 at N = 2..6): a thread per word of N-2 letters carries the word's
// prefixes and the two levels below it; no communication, any number of workgroups per path.
bool tree_supported(const Shape &sh);
hipError_t launch_tree_wide(const Shape &sh, const float *path, float *out, hipStream_t st);    // d = 9..16
hipError_t launch_tree_wide(const Shape &sh, const double *path, double *out, hipStream_t st);
hipError_t launch_tree_f32(const Shape &sh, const float *path, float *out, hipStream_t st);
hipError_t launch_tree_f64(const Shape &sh, const double *path, double *out, hipStream_t st);

// Row-stream family (d = 2..16 with one or two levels below a word of at most 64 per row; see sig_row_stream.hip): stream
// mode, both passes of a stream scan cut into chunks (Shape::rows_in_stream), and final mode.
bool row_stream_supported(const Shape &sh, sig_dtype dtype);
bool row_stream_one_level(const Shape &sh);   // one level below a lane's word (N - 1 letters fit a wavefront)
hipError_t launch_row_stream_f32(const Shape &sh, const float *path, float *out, hipStream_t st);
hipError_t launch_row_stream_f64(const Shape &sh, const double *path, double *out, hipStream_t st);

// Many channels (any d >= 2 at N = 2..9; see sig_wide.hip): what serves d > 16, and 9 to 16 channels beyond depth 6; chunked
// scans in final mode only.
bool wide_supported(const Shape &sh, sig_dtype dtype);
hipError_t launch_wide_f32(const Shape &sh, const float *path, float *out, hipStream_t st);
hipError_t launch_wide_f64(const Shape &sh, const double *path, double *out, hipStream_t st);

// Depth-2 signature in final mode as a contraction over the increments (no scan; see sig_forward_n2.hip): any d.
bool forward_n2_supported(const Shape &sh, sig_dtype dtype);
hipError_t launch_forward_n2_f32(const Shape &sh, const float *path, float *out, hipStream_t st);
hipError_t launch_forward_n2_f64(const Shape &sh, const double *path, double *out, hipStream_t st);
// A chunked scan at depth 2 (Shape::chunks > 1, B counting stretches): the stretches' sums, [B][S] scalars in `partial`,
// then their sum per path in `out`.
bool forward_n2_chunked_supported(const Shape &sh, sig_dtype dtype);
hipError_t launch_forward_n2_chunked_f32(const Shape &sh, const float *path, float *partial, float *out, hipStream_t st);
hipError_t launch_forward_n2_chunked_f64(const Shape &sh, const double *path, double *partial, double *out, hipStream_t st);
// The same on the matrix cores (fp32, 17 to 256 channels; see sig_forward_n2_mfma.hip).  The launch returns
// hipErrorNotSupported, with nothing enqueued, where unaligned buffers leave no room for a tile of four increments.
bool forward_n2_mfma_supported(const Shape &sh);
bool forward_n2_mfma_preferred(const Shape &sh);   // ... and measured faster than the vector kernel
hipError_t launch_forward_n2_mfma_f32(const Shape &sh, const float *path, float *out, hipStream_t st);

// Gradient for many channels (any d at N = 2..9, both modes; see sig_wide_backward.hip); the workspace
// holds one partial gradient per workgroup of a path.
bool wide_backward_supported(const Shape &sh, sig_dtype dtype);
int64_t wide_backward_workspace_bytes(const Shape &sh, sig_dtype dtype);
hipError_t launch_wide_backward_f32(const Shape &sh, const float *path, const float *sig, const float *gout, float *gpath,
                                    float *gbase, void *workspace, int64_t workspace_bytes, hipStream_t st);
hipError_t launch_wide_backward_f64(const Shape &sh, const double *path, const double *sig, const double *gout, double *gpath,
                                    double *gbase, void *workspace, int64_t workspace_bytes, hipStream_t st);

// Gradient of the depth-2 signature in final mode by its closed form (no scan, no workspace; see sig_backward_n2.hip):
// any channel count whose d x (d + 1) output gradient fits the LDS (d <= 122 in fp32, 85 in fp64).
bool backward_n2_supported(const Shape &sh, sig_dtype dtype);
// ... and on the matrix cores (fp32, 8 to 112 channels; see sig_backward_n2_mfma.hip)
bool backward_n2_mfma_supported(const Shape &sh);
hipError_t launch_backward_n2_mfma_f32(const Shape &sh, const float *path, const float *gout, float *gpath, float *gbase,
                                       hipStream_t st);
hipError_t launch_backward_n2_f32(const Shape &sh, const float *path, const float *gout, float *gpath, float *gbase, hipStream_t st);
hipError_t launch_backward_n2_f64(const Shape &sh, const double *path, const double *gout, double *gpath, double *gbase,
                                  hipStream_t st);

// Prefix-tree gradient kernels (d = 2..8 at N = 2..9, d = 9..16 at N = 2..6, any alignment): no communication between threads; the
// per-increment partial gradients go to a workspace of `tree_backward_workspace_bytes` and are summed by a second
// kernel.
hipError_t launch_tree_backward_wide(const Shape &sh, const float *path, const float *sig, const float *gout, float *gpath,
                                     float *gbase, void *workspace, int64_t workspace_bytes, hipStream_t st);   // d = 9..16
hipError_t launch_tree_backward_wide(const Shape &sh, const double *path, const double *sig, const double *gout,
                                     double *gpath, double *gbase, void *workspace, int64_t workspace_bytes, hipStream_t st);
bool tree_backward_supported(const Shape &sh);
int64_t tree_backward_workspace_bytes(const Shape &sh, sig_dtype dtype);
hipError_t launch_tree_backward_f32(const Shape &sh, const float *path, const float *sig, const float *gout, float *gpath,
                                    float *gbase, void *workspace, int64_t workspace_bytes, hipStream_t st);
hipError_t launch_tree_backward_f64(const Shape &sh, const double *path, const double *sig, const double *gout,
                                    double *gpath, double *gbase, void *workspace, int64_t workspace_bytes, hipStream_t st);

// Small-state family: S <= 512 scalars, one wavefront per path, state in LDS, words decoded once.
bool small_supported(const Shape &sh);
hipError_t launch_small_f32(const Shape &sh, const float *path, float *out, hipStream_t st);
hipError_t launch_small_f64(const Shape &sh, const double *path, double *out, hipStream_t st);

// Matrix-core family for d = 4, N = 4..6, final mode (fp32): one wavefront per path.
// `mfma_kernel_name` returns nullptr for shapes the family cannot serve.
const char *mfma_kernel_name(const Shape &sh);
hipError_t launch_mfma_f32(const Shape &sh, const float *path, float *out, hipStream_t st);

// Matrix-core family with four wavefronts per path, one per first letter (fp32, d = 4, N = 4..7,
// final and stream mode).
const char *mfma_shard_kernel_name(const Shape &sh);
hipError_t launch_mfma_shard_f32(const Shape &sh, const float *path, float *out, hipStream_t st);

// Stream mode of that family for N = 4..6 with the four wavefronts of a path in one workgroup: prefix signatures are
// assembled in LDS and written in whole runs.  `mfma_stream_preferred`: the output is too large for the last-level
// cache, which is when this store pattern pays.
const char *mfma_stream_kernel_name(const Shape &sh);
bool mfma_stream_preferred(const Shape &sh);
hipError_t launch_mfma_stream_f32(const Shape &sh, const float *path, float *out, hipStream_t st);

// Matrix-core kernel for d = 16, N = 4, final mode: one workgroup of 8 wavefronts per path.
const char *mfma_d16_kernel_name(const Shape &sh);
hipError_t launch_mfma_d16_f32(const Shape &sh, const float *path, float *out, hipStream_t st);

// Matrix-core kernel for d = 8, N = 4..6, final mode: 64 independent wavefronts per path.
const char *mfma_d8_kernel_name(const Shape &sh);
hipError_t launch_mfma_d8_f32(const Shape &sh, const float *path, float *out, hipStream_t st);

}  // namespace sig

#endif  // SIG_INTERNAL_H_
