// C ABI of libsig: argument validation, size helpers and kernel-family dispatch.
// The operations are those declared in sig.h; nothing here dereferences a device pointer.
#include "sig_internal.h"

#include <atomic>

// Scratch memory of sig_forward_chunked_static, the one entry point for callers that cannot allocate: every GPU the
// library runs on holds its own copy of this array, at its own address, until the process ends.  In host code the
// name is only a handle for hipGetSymbolAddress: kernels and copies are given the address that call returns.
static __device__ __align__(256) unsigned char scratch[SIG_STATIC_SCRATCH_BYTES];

namespace {

constexpr int64_t kMaxChannels = int64_t(1) << 40;
constexpr int64_t kMaxElems = int64_t(1) << 60;

constexpr int kMaxDevices = 64;
std::atomic<void *> scratch_address[kMaxDevices];   // per device, filled on the first call made with that device current

// Device address of `scratch` on the current device; nullptr if the runtime refuses.  The look-up is done once per
// device (threads that race to it obtain the same address, so the race is harmless).
void *scratch_on_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void *ptr = scratch_address[dev].load(std::memory_order_acquire);
    if (ptr == nullptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return nullptr;
        scratch_address[dev].store(ptr, std::memory_order_release);
    }
    return ptr;
}

// Fills pw/off/S; false if d, N are invalid or S exceeds kMaxChannels.
bool fill_levels(int d, int N, sig::Shape &sh)
{
    if (d < 1 || N < 1 || N > SIG_MAX_DEPTH) return false;
    sh.d = d;
    sh.N = N;
    sh.pw[0] = 1;
    sh.off[1] = 0;
    int64_t total = 0;
    for (int k = 1; k <= N; ++k) {
        if (sh.pw[k - 1] > kMaxChannels / d) return false;
        sh.pw[k] = sh.pw[k - 1] * d;
        total += sh.pw[k];
        if (total > kMaxChannels) return false;
        sh.off[k + 1] = total;
    }
    sh.off[0] = 0;
    sh.S = total;
    return true;
}

// Validates a whole call.  On SIG_OK `sh` is complete.
sig_status make_shape(int64_t B, int64_t L, int d, int N, int stream, int basepoint, sig::Shape &sh)
{
    if (B < 0 || d < 1 || N < 1 || N > SIG_MAX_DEPTH) return SIG_ERR_INVALID_ARG;
    if (basepoint ? (L < 1) : (L < 2)) return SIG_ERR_INVALID_ARG;
    if (!fill_levels(d, N, sh)) return SIG_ERR_OVERFLOW;
    sh.B = B;
    sh.L = L;
    sh.stream = stream ? 1 : 0;
    sh.basepoint = basepoint ? 1 : 0;
    sh.basepoint_value = nullptr;
    sh.chunks = 1;
    sh.rows_in_stream = 0;
    sh.from_identity = 1;
    sh.chunk_len = 0;
    sh.n_inc = basepoint ? L : L - 1;
    // path elements B*L*d and output elements B*[n_inc*]S must stay below kMaxElems
    if (L > kMaxElems / d) return SIG_ERR_OVERFLOW;
    const int64_t per_path_in = L * d;
    if (B > 0 && per_path_in > kMaxElems / B) return SIG_ERR_OVERFLOW;
    int64_t per_path_out = sh.S;
    if (sh.stream) {
        if (sh.n_inc > kMaxElems / sh.S) return SIG_ERR_OVERFLOW;
        per_path_out = sh.n_inc * sh.S;
    }
    if (B > 0 && per_path_out > kMaxElems / B) return SIG_ERR_OVERFLOW;
    return SIG_OK;
}

// Shape of a batch of `rows` signatures with no path attached.
sig_status make_rows_shape(int64_t rows, int d, int N, sig::Shape &sh)
{
    if (rows < 0 || d < 1 || N < 1 || N > SIG_MAX_DEPTH) return SIG_ERR_INVALID_ARG;
    if (!fill_levels(d, N, sh)) return SIG_ERR_OVERFLOW;
    if (rows > 0 && sh.S > kMaxElems / rows) return SIG_ERR_OVERFLOW;
    sh.B = rows;
    sh.L = 0;
    sh.n_inc = 0;
    sh.stream = sh.basepoint = 0;
    sh.basepoint_value = nullptr;
    sh.chunks = 1;
    sh.rows_in_stream = 0;
    sh.from_identity = 1;
    sh.chunk_len = 0;
    return SIG_OK;
}

enum class Family { Generic, Mfma, MfmaShard, MfmaStream, MfmaD16, MfmaD8, Small, Tree, RowStream, Wide, Depth2, None };

// The pointers decide only alignment: the matrix-core family loads and stores 16 bytes per lane.
Family resolve(const sig::Shape &sh, sig_dtype dtype, sig_variant variant, const void *path, const void *out)
{
    const bool aligned = reinterpret_cast<uintptr_t>(out) % 16 == 0 && reinterpret_cast<uintptr_t>(path) % 16 == 0 &&
                         reinterpret_cast<uintptr_t>(sh.basepoint_value) % 16 == 0;
    const bool mfma_ok = dtype == SIG_F32 && aligned && sig::mfma_kernel_name(sh) != nullptr;
    const bool shard_ok = dtype == SIG_F32 && aligned && sig::mfma_shard_kernel_name(sh) != nullptr;
    const bool stream_ok = dtype == SIG_F32 && aligned && sig::mfma_stream_kernel_name(sh) != nullptr;
    const bool d16_ok = dtype == SIG_F32 && aligned && sig::mfma_d16_kernel_name(sh) != nullptr;
    const bool d8_ok = dtype == SIG_F32 && aligned && sig::mfma_d8_kernel_name(sh) != nullptr;
    const bool generic_ok = sig::generic_supported(sh, dtype);
    const bool small_ok = sig::small_supported(sh);
    const bool tree_ok = sig::tree_supported(sh);
    const bool wide_ok = sig::wide_supported(sh, dtype);
    const bool depth2_ok = sig::forward_n2_supported(sh, dtype);
    const bool rows_any = sig::row_stream_supported(sh, dtype);
    const bool rows_ok = sh.stream && rows_any;
    switch (variant) {
        case SIG_VARIANT_AUTO:
            if (depth2_ok) return Family::Depth2;   // depth 2 in final mode needs no scan
            // four wavefronts per path when one per path would leave most of the chip idle, when every
            // prefix is stored (stream mode) or when the state does not fit one wavefront (N = 7)
            if (stream_ok && sig::mfma_stream_preferred(sh)) return Family::MfmaStream;
            if (shard_ok && (!mfma_ok || sh.B < 512)) return Family::MfmaShard;
            if (mfma_ok) return Family::Mfma;
            // one workgroup per path leaves the chip idle below ~48 paths (B = 8: 45 us against 25 for the prefix-tree
            // kernel, which spreads a path over 16 workgroups)
            if (d16_ok && !(sh.B < 48 && tree_ok)) return Family::MfmaD16;
            // 64 wavefronts per path pay off while paths are few; from 512 paths on each shard's own prefix sums
            // are pure overhead (N = 4 at B = 2048: 170 us against 62 for the prefix-tree kernel); N = 6 stays
            if (d8_ok && !(sh.N <= 5 && sh.B >= 512 && tree_ok)) return Family::MfmaD8;
            // every prefix stored: a wavefront per row with whole-row stores, wherever it applies; in final mode where
            // one level lies below a lane's word and the state is more than a wavefront's worth of scalars (measured
            // at 128 points: d = 8, N = 3: 19 us against 47 at 32 paths, 30 against 56 at 4096; d = 3, N = 4: 17 against
            // 23 and 23 against 47; with two levels below the word the prefix-tree kernel is as fast or faster)
            if (rows_ok || (rows_any && sh.S > 64 && sig::row_stream_one_level(sh))) return Family::RowStream;
            // up to 128 scalars (two words per lane) the one-wavefront kernel wins; beyond, its lanes carry 4 or 8
            // words each and the prefix-tree kernel is up to 6 times faster (d = 2, N = 8: 38 us against 194)
            // (in stream mode up to depth 3 as well: its lanes store 64 consecutive scalars per instruction, the
            // prefix-tree kernel's lanes store d^2 scalars apart: d = 16, N = 2: 52 us against 75, d = 7, N = 3: 67 against 85
            // at 128 paths of 256 points)
            if (wide_ok && sh.d > 16 && sh.S > 128) return Family::Wide;   // d = 20, N = 2: 52 us against 57 on `small`
            if (small_ok && (sh.S <= 128 || !tree_ok || (sh.stream && sh.N <= 3))) return Family::Small;
            if (tree_ok) return Family::Tree;
            // beyond 16 channels at depths 2..4: the run-time-d kernel (d = 32, N = 2 at 32 paths of 128 points: 0.72 ms
            // on the generic kernel)
            if (wide_ok) return Family::Wide;
            return generic_ok ? Family::Generic : Family::None;
        case SIG_VARIANT_GENERIC: return generic_ok ? Family::Generic : Family::None;
        case SIG_VARIANT_MFMA:
            return mfma_ok ? Family::Mfma : d16_ok ? Family::MfmaD16 : d8_ok ? Family::MfmaD8 : Family::None;
        case SIG_VARIANT_MFMA_SHARD: return shard_ok ? Family::MfmaShard : Family::None;
        case SIG_VARIANT_MFMA_STREAM: return stream_ok ? Family::MfmaStream : Family::None;
        case SIG_VARIANT_SMALL: return small_ok ? Family::Small : Family::None;
        case SIG_VARIANT_TREE: return tree_ok ? Family::Tree : Family::None;
        case SIG_VARIANT_ROW_STREAM: return rows_any ? Family::RowStream : Family::None;
        case SIG_VARIANT_WIDE: return wide_ok ? Family::Wide : Family::None;
        case SIG_VARIANT_DEPTH2: return depth2_ok ? Family::Depth2 : Family::None;
    }
    return Family::None;
}

// Launches the scan of one kernel family (not Family::None) as the shape stands.
hipError_t launch_scan(Family family, const sig::Shape &sh, sig_dtype dtype, const void *path, void *out,
                       hipStream_t hip_stream)
{
    switch (family) {
        case Family::Mfma:
            return sig::launch_mfma_f32(sh, static_cast<const float *>(path), static_cast<float *>(out), hip_stream);
        case Family::MfmaShard:
            return sig::launch_mfma_shard_f32(sh, static_cast<const float *>(path), static_cast<float *>(out), hip_stream);
        case Family::MfmaStream:
            return sig::launch_mfma_stream_f32(sh, static_cast<const float *>(path), static_cast<float *>(out), hip_stream);
        case Family::MfmaD16:
            return sig::launch_mfma_d16_f32(sh, static_cast<const float *>(path), static_cast<float *>(out), hip_stream);
        case Family::MfmaD8:
            return sig::launch_mfma_d8_f32(sh, static_cast<const float *>(path), static_cast<float *>(out), hip_stream);
        case Family::Tree:
            return dtype == SIG_F32
                       ? sig::launch_tree_f32(sh, static_cast<const float *>(path), static_cast<float *>(out), hip_stream)
                       : sig::launch_tree_f64(sh, static_cast<const double *>(path), static_cast<double *>(out), hip_stream);
        case Family::RowStream:
            return dtype == SIG_F32
                       ? sig::launch_row_stream_f32(sh, static_cast<const float *>(path), static_cast<float *>(out), hip_stream)
                       : sig::launch_row_stream_f64(sh, static_cast<const double *>(path), static_cast<double *>(out), hip_stream);
        case Family::Depth2:
            // From 49 channels on, where padding to whole 16 x 16 tiles adds at most 30 % of work, the contraction runs
            // on the matrix cores (fp32; d = 64: 1.2 to 1.6 times the vector kernel from 32 to 16 384 paths).
            if (dtype == SIG_F32 && sig::forward_n2_mfma_preferred(sh)) {
                const hipError_t err = sig::launch_forward_n2_mfma_f32(sh, static_cast<const float *>(path), static_cast<float *>(out), hip_stream);
                if (err != hipErrorNotSupported) return err;
            }
            return dtype == SIG_F32
                       ? sig::launch_forward_n2_f32(sh, static_cast<const float *>(path), static_cast<float *>(out), hip_stream)
                       : sig::launch_forward_n2_f64(sh, static_cast<const double *>(path), static_cast<double *>(out), hip_stream);
        case Family::Wide:
            return dtype == SIG_F32
                       ? sig::launch_wide_f32(sh, static_cast<const float *>(path), static_cast<float *>(out), hip_stream)
                       : sig::launch_wide_f64(sh, static_cast<const double *>(path), static_cast<double *>(out), hip_stream);
        case Family::Small:
            return dtype == SIG_F32
                       ? sig::launch_small_f32(sh, static_cast<const float *>(path), static_cast<float *>(out), hip_stream)
                       : sig::launch_small_f64(sh, static_cast<const double *>(path), static_cast<double *>(out), hip_stream);
        case Family::Generic:
            return dtype == SIG_F32
                       ? sig::launch_generic_f32(sh, static_cast<const float *>(path), static_cast<float *>(out), hip_stream)
                       : sig::launch_generic_f64(sh, static_cast<const double *>(path), static_cast<double *>(out), hip_stream);
        case Family::None: break;
    }
    return hipErrorNotSupported;
}

// Stream mode of the small-state and prefix-tree families, into how many chunks a path is cut (1: not at all).  These
// kernels scan a path in one wavefront or a few threads, so with few paths the chain of increments is all there is to
// wait for (128 paths of 256 points, d = 8, N = 3: 357 us, 0.2 TB/s).  The scan is a reduction (section 5.1), in stream
// mode as well: the prefix signatures of a chunk are those of the chunk alone multiplied on the left by the
// signature of everything before it.
int stream_chunks(Family family, const sig::Shape &sh)
{
    if (!sh.stream || sh.chunks != 1 ||
        (family != Family::Small && family != Family::Tree && family != Family::RowStream && family != Family::Wide))
        return 1;
    // the kernel for many channels: at depth 2 up to 64 channels only (32 below 192 increments; beyond, a path has
    // workgroups enough, and from depth 3 on the chain of products along the chunk ends costs more than it saves: 32 paths of 128 points at d = 20, N = 3
    // take 283 us in chunks against 103)
    if (family == Family::Wide && (sh.N != 2 || sh.d > 64 || (sh.d > 32 && sh.n_inc < 192))) return 1;
    if (sh.S >= (int64_t(1) << 31)) return 1;
    // Two scans of n_inc / chunks increments each and a chain of chunks - 1 products (about the cost of an increment
    // each) are shortest near sqrt(n_inc) chunks; more than ~2048 rows at a time add no parallelism.  Measured at
    // L = 256, B = 128: 8 chunks take 97 us against 359 at d = 8, N = 3 (4, 16: 146, 94), 57 against 89 at d = 3, N = 5,
    // 78 against 195 at d = 16, N = 2; at B = 1024 nothing is gained, and below ~128 increments the two extra launches
    // cost more than the shorter chain saves.
    // ... for the prefix-tree and one-wavefront kernels; the row kernel gains from 96 increments on (32 paths of 128
    // points: d = 16, N = 2: 35 us against 79, d = 3, N = 4: 25 against 41; 65 points: no gain)
    if (sh.n_inc < (family == Family::RowStream || family == Family::Wide ? 96 : 128)) return 1;
    int chunks = 1;
    while (int64_t(chunks) * 2 * chunks * 2 <= sh.n_inc && int64_t(chunks) * 2 * sh.B <= 2048) chunks *= 2;
    return chunks >= 4 ? chunks : 1;
}

// Launches the scan of one kernel family (not Family::None); few long paths in stream mode are cut into chunks:
// every chunk's own signature goes to the row of its last increment, a running product along those rows turns them
// into the path's prefix signatures there (final values), and every chunk is scanned again from the row before it,
// writing the rows in between.  The output is written once and nothing else is needed for scratch.
hipError_t launch_family(Family family, const sig::Shape &sh, sig_dtype dtype, const void *path, void *out,
                         hipStream_t hip_stream)
{
    const int chunks = stream_chunks(family, sh);
    if (chunks <= 1) return launch_scan(family, sh, dtype, path, out, hip_stream);
    sig::Shape ch = sh;
    ch.chunks = chunks;
    ch.chunk_len = (sh.n_inc + chunks - 1) / chunks;
    ch.B = sh.B * chunks;
    ch.rows_in_stream = 1;
    ch.stream = 0;
    hipError_t err = launch_scan(family, ch, dtype, path, out, hip_stream);
    if (err != hipSuccess) return err;
    err = dtype == SIG_F32 ? sig::launch_chunk_prefix_f32(sh, sh.B, sh.n_inc, ch.chunk_len, static_cast<float *>(out), hip_stream)
                           : sig::launch_chunk_prefix_f64(sh, sh.B, sh.n_inc, ch.chunk_len, static_cast<double *>(out), hip_stream);
    if (err != hipSuccess) return err;
    ch.stream = 1;
    return launch_scan(family, ch, dtype, path, out, hip_stream);
}

bool valid_enums(sig_dtype dtype, sig_variant variant)
{
    return (dtype == SIG_F32 || dtype == SIG_F64) &&
           (variant == SIG_VARIANT_AUTO || variant == SIG_VARIANT_GENERIC || variant == SIG_VARIANT_MFMA ||
            variant == SIG_VARIANT_MFMA_SHARD || variant == SIG_VARIANT_SMALL || variant == SIG_VARIANT_TREE ||
            variant == SIG_VARIANT_MFMA_STREAM || variant == SIG_VARIANT_ROW_STREAM || variant == SIG_VARIANT_WIDE || variant == SIG_VARIANT_DEPTH2);
}

}  // namespace

extern "C" {

int64_t sig_signature_channels(int d, int N)
{
    sig::Shape sh;
    return fill_levels(d, N, sh) ? sh.S : -1;
}

int64_t sig_output_elems(int64_t B, int64_t L, int d, int N, int stream, int basepoint)
{
    sig::Shape sh;
    if (make_shape(B, L, d, N, stream, basepoint, sh) != SIG_OK) return -1;
    return B * (sh.stream ? sh.n_inc * sh.S : sh.S);
}

int64_t sig_fused_fmas(int d, int N)
{
    sig::Shape sh;
    if (!fill_levels(d, N, sh)) return -1;
    int64_t m = 0;
    for (int i = 2; i <= N; ++i) m += int64_t(N - i + 1) * sh.pw[i];
    return m;
}

sig_status sig_forward_variant(const void *path, int64_t B, int64_t L, int d, int N,
                               int stream, int basepoint, sig_dtype dtype,
                               void *out, hipStream_t hip_stream, sig_variant variant)
{
    if (!valid_enums(dtype, variant)) return SIG_ERR_INVALID_ARG;
    sig::Shape sh;
    const sig_status st = make_shape(B, L, d, N, stream, basepoint, sh);
    if (st != SIG_OK) return st;
    if (B == 0) return SIG_OK;
    if (path == nullptr || out == nullptr) return SIG_ERR_INVALID_ARG;
    const Family family = resolve(sh, dtype, variant, path, out);
    if (family == Family::None) return SIG_ERR_UNSUPPORTED;
    const hipError_t err = launch_family(family, sh, dtype, path, out, hip_stream);
    return err == hipSuccess ? SIG_OK : SIG_ERR_HIP;
}

sig_status sig_combine(const void *a, const void *b, int64_t B, int d, int N, sig_dtype dtype,
                       void *out, hipStream_t hip_stream)
{
    if (dtype != SIG_F32 && dtype != SIG_F64) return SIG_ERR_INVALID_ARG;
    sig::Shape sh;
    const sig_status st = make_rows_shape(B, d, N, sh);
    if (st != SIG_OK) return st;
    if (B == 0) return SIG_OK;
    if (a == nullptr || b == nullptr || out == nullptr) return SIG_ERR_INVALID_ARG;
    if (!sig::combine_supported(sh)) return SIG_ERR_UNSUPPORTED;
    const hipError_t err =
        dtype == SIG_F32
            ? sig::launch_combine_f32(sh, static_cast<const float *>(a), static_cast<const float *>(b),
                                      static_cast<float *>(out), hip_stream)
            : sig::launch_combine_f64(sh, static_cast<const double *>(a), static_cast<const double *>(b),
                                      static_cast<double *>(out), hip_stream);
    return err == hipSuccess ? SIG_OK : SIG_ERR_HIP;
}

int64_t sig_backward_workspace_bytes(int64_t B, int64_t L, int d, int N, int stream, int basepoint, sig_dtype dtype)
{
    if (dtype != SIG_F32 && dtype != SIG_F64) return -1;
    sig::Shape sh;
    if (make_shape(B, L, d, N, stream, basepoint, sh) != SIG_OK) return -1;
    if (B == 0) return 0;
    return sig::backward_workspace_bytes(sh, dtype);
}

sig_status sig_backward(const void *path, const void *sig, const void *grad_out, int64_t B, int64_t L, int d, int N,
                        int stream, int basepoint, const void *basepoint_value, sig_dtype dtype, void *grad_path,
                        void *grad_basepoint, void *workspace, int64_t workspace_bytes, hipStream_t hip_stream)
{
    if (dtype != SIG_F32 && dtype != SIG_F64) return SIG_ERR_INVALID_ARG;
    sig::Shape sh;
    const sig_status st = make_shape(B, L, d, N, stream, basepoint, sh);
    if (st != SIG_OK) return st;
    if (B == 0) return SIG_OK;
    if (path == nullptr || sig == nullptr || grad_out == nullptr || grad_path == nullptr) return SIG_ERR_INVALID_ARG;
    if (!sh.basepoint && (basepoint_value != nullptr || grad_basepoint != nullptr)) return SIG_ERR_INVALID_ARG;
    sh.basepoint_value = basepoint_value;
    const int64_t need = sig::backward_workspace_bytes(sh, dtype);
    if (need < 0) return SIG_ERR_UNSUPPORTED;
    if (need > 0 && (workspace == nullptr || workspace_bytes < need)) return SIG_ERR_INVALID_ARG;
    const hipError_t err =
        dtype == SIG_F32
            ? sig::launch_backward_f32(sh, static_cast<const float *>(path), static_cast<const float *>(sig),
                                       static_cast<const float *>(grad_out), static_cast<float *>(grad_path),
                                       static_cast<float *>(grad_basepoint), workspace, workspace_bytes, hip_stream)
            : sig::launch_backward_f64(sh, static_cast<const double *>(path), static_cast<const double *>(sig),
                                       static_cast<const double *>(grad_out), static_cast<double *>(grad_path),
                                       static_cast<double *>(grad_basepoint), workspace, workspace_bytes, hip_stream);
    return err == hipSuccess ? SIG_OK : SIG_ERR_HIP;
}

// Layout of a gradient computed stretch by stretch: K stretches of m increments per path, served as the B K short paths
// of `rows`; the workspace holds, each 256-byte aligned, the stretches' points, their signatures, the running products,
// the gradients with respect to those, the stretches' point gradients and the workspace of the gradient kernels.
struct StretchPlan {
    int64_t K, m;
    sig::Shape rows;
    int64_t at_points, at_sigs, at_prefix, at_grads, at_point_grads, at_inner, inner_bytes, total;
};

static sig_status plan_backward_chunked(int64_t B, int64_t L, int d, int N, int basepoint, int chunks, sig_dtype dtype, sig::Shape &sh,
                                        StretchPlan &pl)
{
    if (dtype != SIG_F32 && dtype != SIG_F64) return SIG_ERR_INVALID_ARG;
    const sig_status st = make_shape(B, L, d, N, 0, basepoint, sh);
    if (st != SIG_OK) return st;
    if (chunks < 2 || chunks > 65536) return SIG_ERR_INVALID_ARG;
    if (B > 65535) return SIG_ERR_UNSUPPORTED;
    pl.m = (sh.n_inc + chunks - 1) / chunks;
    pl.K = (sh.n_inc + pl.m - 1) / pl.m;
    if (B > 0 && pl.K > kMaxElems / B) return SIG_ERR_OVERFLOW;
    const sig_status rs = make_shape(B * pl.K, pl.m + 1, d, N, 0, 0, pl.rows);
    if (rs != SIG_OK) return rs;
    if (B == 0) {
        pl.total = 0;
        return SIG_OK;
    }
    if (!sig::combine_supported(pl.rows)) return SIG_ERR_UNSUPPORTED;
    pl.rows.from_identity = 0;   // a stretch is walked back from the signature of the path up to its end
    pl.inner_bytes = sig::backward_workspace_bytes(pl.rows, dtype);
    if (pl.inner_bytes < 0) return SIG_ERR_UNSUPPORTED;
    const int64_t elem = dtype == SIG_F32 ? int64_t(sizeof(float)) : int64_t(sizeof(double));
    const auto round_up = [](int64_t bytes) { return (bytes + 255) / 256 * 256; };
    const int64_t points = round_up(pl.rows.B * (pl.m + 1) * d * elem), sigs = round_up(pl.rows.B * sh.S * elem);
    if (sigs > kMaxElems || points > kMaxElems) return SIG_ERR_OVERFLOW;
    pl.at_points = 0;
    pl.at_sigs = pl.at_points + points;
    pl.at_prefix = pl.at_sigs + sigs;
    pl.at_grads = pl.at_prefix + sigs;
    pl.at_point_grads = pl.at_grads + sigs;
    pl.at_inner = pl.at_point_grads + points;
    pl.total = pl.at_inner + round_up(pl.inner_bytes);
    return SIG_OK;
}

int64_t sig_backward_chunked_workspace_bytes(int64_t B, int64_t L, int d, int N, int basepoint, int chunks, sig_dtype dtype)
{
    sig::Shape sh;
    StretchPlan pl;
    if (plan_backward_chunked(B, L, d, N, basepoint, chunks, dtype, sh, pl) != SIG_OK) return -1;
    if (B > 0 && resolve(pl.rows, dtype, SIG_VARIANT_AUTO, nullptr, nullptr) == Family::None) return -1;
    return pl.total;
}

sig_status sig_backward_chunked(const void *path, const void *grad_out, int64_t B, int64_t L, int d, int N, int basepoint,
                                const void *basepoint_value, int chunks, sig_dtype dtype, void *grad_path, void *grad_basepoint,
                                void *workspace, int64_t workspace_bytes, hipStream_t hip_stream)
{
    sig::Shape sh;
    StretchPlan pl;
    const sig_status st = plan_backward_chunked(B, L, d, N, basepoint, chunks, dtype, sh, pl);
    if (st != SIG_OK) return st;
    if (B == 0) return SIG_OK;
    if (path == nullptr || grad_out == nullptr || grad_path == nullptr) return SIG_ERR_INVALID_ARG;
    if (!sh.basepoint && (basepoint_value != nullptr || grad_basepoint != nullptr)) return SIG_ERR_INVALID_ARG;
    if (workspace == nullptr || workspace_bytes < pl.total || reinterpret_cast<uintptr_t>(workspace) % 16 != 0) return SIG_ERR_INVALID_ARG;
    sh.basepoint_value = basepoint_value;
    char *ws = static_cast<char *>(workspace);
    void *points = ws + pl.at_points, *sigs = ws + pl.at_sigs, *prefix = ws + pl.at_prefix, *grads = ws + pl.at_grads,
         *point_grads = ws + pl.at_point_grads, *inner = ws + pl.at_inner;
    const Family family = resolve(pl.rows, dtype, SIG_VARIANT_AUTO, points, sigs);
    if (family == Family::None) return SIG_ERR_UNSUPPORTED;
    // the stretches as paths of their own, and their signatures
    if (sig::launch_stretch_gather(sh, dtype, pl.K, pl.m, path, points, hip_stream) != hipSuccess) return SIG_ERR_HIP;
    if (launch_family(family, pl.rows, dtype, points, sigs, hip_stream) != hipSuccess) return SIG_ERR_HIP;
    // the signature of the path up to the end of every stretch: a running product along each path's stretches, by one
    // workgroup per path while a signature fits its LDS three times over, else a launch per product
    const int64_t elem = dtype == SIG_F32 ? int64_t(sizeof(float)) : int64_t(sizeof(double));
    if (3 * sh.S * elem <= 64 * 1024 || pl.K == 1) {
        if (sig::launch_copy_rows(dtype, sigs, sh.S, prefix, sh.S, sh.S, pl.rows.B, hip_stream) != hipSuccess) return SIG_ERR_HIP;
        if (pl.K > 1) {
            const hipError_t err = dtype == SIG_F32
                                       ? sig::launch_chunk_prefix_f32(pl.rows, B, pl.K, 1, static_cast<float *>(prefix), hip_stream)
                                       : sig::launch_chunk_prefix_f64(pl.rows, B, pl.K, 1, static_cast<double *>(prefix), hip_stream);
            if (err != hipSuccess) return SIG_ERR_HIP;
        }
    } else {
        const int64_t per_path = pl.K * sh.S;
        if (sig::launch_copy_rows(dtype, sigs, per_path, prefix, per_path, sh.S, B, hip_stream) != hipSuccess) return SIG_ERR_HIP;
        sig::Shape paths = pl.rows;
        paths.B = B;
        const int64_t strides[7] = {per_path, per_path, per_path, 0, 0, 0, 0};
        for (int64_t c = 1; c < pl.K; ++c) {
            const char *left = static_cast<const char *>(prefix) + (c - 1) * sh.S * elem;
            const char *right = static_cast<const char *>(sigs) + c * sh.S * elem;
            char *product = static_cast<char *>(prefix) + c * sh.S * elem;
            const hipError_t err =
                dtype == SIG_F32 ? sig::launch_combine_f32(paths, reinterpret_cast<const float *>(left), reinterpret_cast<const float *>(right),
                                                           reinterpret_cast<float *>(product), hip_stream, strides)
                                 : sig::launch_combine_f64(paths, reinterpret_cast<const double *>(left), reinterpret_cast<const double *>(right),
                                                           reinterpret_cast<double *>(product), hip_stream, strides);
            if (err != hipSuccess) return SIG_ERR_HIP;
        }
    }
    // the gradient with respect to each of them, from the last stretch back
    if (sig::launch_copy_rows(dtype, grad_out, sh.S, static_cast<char *>(grads) + (pl.K - 1) * sh.S * elem, pl.K * sh.S, sh.S, B,
                              hip_stream) != hipSuccess)
        return SIG_ERR_HIP;
    if (sig::launch_stretch_adjoint_chain(pl.rows, dtype, pl.K, sigs, grads, hip_stream) != hipSuccess) return SIG_ERR_HIP;
    // every stretch walked backwards on its own, then the point gradients added up
    const hipError_t err =
        dtype == SIG_F32
            ? sig::launch_backward_f32(pl.rows, static_cast<const float *>(points), static_cast<const float *>(prefix),
                                       static_cast<const float *>(grads), static_cast<float *>(point_grads), nullptr, inner,
                                       pl.inner_bytes, hip_stream)
            : sig::launch_backward_f64(pl.rows, static_cast<const double *>(points), static_cast<const double *>(prefix),
                                       static_cast<const double *>(grads), static_cast<double *>(point_grads), nullptr, inner,
                                       pl.inner_bytes, hip_stream);
    if (err != hipSuccess) return SIG_ERR_HIP;
    if (sig::launch_stretch_scatter(sh, dtype, pl.K, pl.m, point_grads, grad_path, grad_basepoint, hip_stream) != hipSuccess)
        return SIG_ERR_HIP;
    return SIG_OK;
}

int sig_backward_chunks_hint(int64_t B, int64_t L, int d, int N, int basepoint, sig_dtype dtype)
{
    if (dtype != SIG_F32 && dtype != SIG_F64) return 0;
    sig::Shape sh;
    if (make_shape(B, L, d, N, 0, basepoint, sh) != SIG_OK) return 0;
    // Depth 2 has a closed form with no walk at all.  Otherwise the walk is one increment after the other, and cutting
    // it pays once the stretches' walks are shorter by more than the two chains between them cost (the running
    // products and the gradients with respect to them, a few microseconds per stretch each): measured from 512
    // increments on, best near sqrt(n_inc) / 2 stretches for signatures up to 2048 scalars, fewer for larger ones
    // (a quarter of sqrt(n_inc) once the chains take a launch per stretch).
    if (N < 3 || B < 1 || B > 128 || sh.n_inc < 512) return 1;
    const int64_t elem = dtype == SIG_F32 ? int64_t(sizeof(float)) : int64_t(sizeof(double));
    const int64_t per_stretch = sh.S <= 2048 ? 4 : 3 * sh.S * elem <= 64 * 1024 ? 8 : 16;
    int chunks = 1;
    for (;;) {
        const int64_t next = int64_t(chunks) * 2;
        if (next * B > 1024 || sh.n_inc / next < 32 || next * next * per_stretch > sh.n_inc) break;
        const int64_t bytes = sig_backward_chunked_workspace_bytes(B, L, d, N, basepoint, int(next), dtype);
        if (bytes < 0 || bytes > (int64_t(2) << 30)) break;
        chunks = int(next);
    }
    return chunks;
}

sig_status sig_invert(const void *sig, int64_t rows, int d, int N, sig_dtype dtype, void *out, hipStream_t hip_stream)
{
    if (dtype != SIG_F32 && dtype != SIG_F64) return SIG_ERR_INVALID_ARG;
    sig::Shape sh;
    const sig_status st = make_rows_shape(rows, d, N, sh);
    if (st != SIG_OK) return st;
    if (rows == 0) return SIG_OK;
    if (sig == nullptr || out == nullptr) return SIG_ERR_INVALID_ARG;
    if (!sig::combine_supported(sh)) return SIG_ERR_UNSUPPORTED;
    const hipError_t err =
        dtype == SIG_F32 ? sig::launch_invert_f32(sh, static_cast<const float *>(sig), static_cast<float *>(out), hip_stream)
                         : sig::launch_invert_f64(sh, static_cast<const double *>(sig), static_cast<double *>(out), hip_stream);
    return err == hipSuccess ? SIG_OK : SIG_ERR_HIP;
}

sig_status sig_combine_strided(const void *a, int64_t a_stride, const void *b, int64_t b_stride, int64_t B, int d, int N,
                               sig_dtype dtype, void *out, int64_t out_stride, hipStream_t hip_stream)
{
    if (dtype != SIG_F32 && dtype != SIG_F64) return SIG_ERR_INVALID_ARG;
    sig::Shape sh;
    const sig_status st = make_rows_shape(B, d, N, sh);
    if (st != SIG_OK) return st;
    if (a_stride < 0 || b_stride < 0 || out_stride < sh.S) return SIG_ERR_INVALID_ARG;
    if (B > 0 && (a_stride > kMaxElems / B || b_stride > kMaxElems / B || out_stride > kMaxElems / B)) return SIG_ERR_OVERFLOW;
    if (B == 0) return SIG_OK;
    if (a == nullptr || b == nullptr || out == nullptr) return SIG_ERR_INVALID_ARG;
    if (!sig::combine_supported(sh)) return SIG_ERR_UNSUPPORTED;
    const int64_t strides[7] = {a_stride, b_stride, out_stride, 0, 0, 0, 0};
    const hipError_t err =
        dtype == SIG_F32
            ? sig::launch_combine_f32(sh, static_cast<const float *>(a), static_cast<const float *>(b),
                                      static_cast<float *>(out), hip_stream, strides)
            : sig::launch_combine_f64(sh, static_cast<const double *>(a), static_cast<const double *>(b),
                                      static_cast<double *>(out), hip_stream, strides);
    return err == hipSuccess ? SIG_OK : SIG_ERR_HIP;
}

// Shape of a chunked scan: B * chunks rows, each a stretch of chunk_len increments.  SIG_OK or why not.
static sig_status make_chunked_shape(int64_t B, int64_t L, int d, int N, int basepoint, int chunks, sig::Shape &sh)
{
    const sig_status st = make_shape(B, L, d, N, 0, basepoint, sh);
    if (st != SIG_OK) return st;
    if (chunks < 2 || chunks > 65536 || (chunks & (chunks - 1)) != 0) return SIG_ERR_INVALID_ARG;
    if (B > 0 && sh.S > kMaxElems / 2 / chunks / B) return SIG_ERR_OVERFLOW;
    sh.chunks = chunks;
    sh.chunk_len = (sh.n_inc + chunks - 1) / chunks;
    sh.B = B * chunks;
    return SIG_OK;
}

int64_t sig_forward_chunked_workspace_bytes(int64_t B, int64_t L, int d, int N, int basepoint, int chunks, sig_dtype dtype)
{
    if (dtype != SIG_F32 && dtype != SIG_F64) return -1;
    sig::Shape sh;
    if (make_chunked_shape(B, L, d, N, basepoint, chunks, sh) != SIG_OK) return -1;
    // the chunk signatures, and half as much again for the first round of products
    return (sh.B + sh.B / 2) * sh.S * int64_t(dtype == SIG_F32 ? sizeof(float) : sizeof(double));
}

int sig_forward_chunks_hint(int64_t B, int64_t L, int d, int N, int basepoint, sig_dtype dtype)
{
    if (dtype != SIG_F32 && dtype != SIG_F64) return 0;
    sig::Shape sh;
    if (make_shape(B, L, d, N, 0, basepoint, sh) != SIG_OK) return 0;
    // the d = 8 matrix family already spreads a path over 64 wavefronts; everything else scans a path in one
    // workgroup and gains from 512 increments on
    if (N == 2) {
        // Depth 2 is one sum over the increments: a path alone takes about 1.5 us per staged tile (128 increments up to
        // 28 channels, 63 at 64, 39 at 100), cut into stretches two launches of about 22 us in all: from 24 tiles on;
        // stretches of at least 128 increments, at most 2048 of them.
        const int64_t padded = (d + 3) / 4 * 4;
        const int64_t tile = 4096 / padded - 1 < 128 ? (4096 / padded - 1 < 1 ? 1 : 4096 / padded - 1) : 128;
        if (B < 1 || B > 1024 || sh.n_inc < 24 * tile) return 1;
        int chunks = 1;
        const int64_t elem2 = dtype == SIG_F32 ? int64_t(sizeof(float)) : int64_t(sizeof(double));
        while (int64_t(chunks) * 2 * B <= 2048 && sh.n_inc / (int64_t(chunks) * 2) >= 128 &&
               int64_t(chunks) * 2 * B * sh.S * elem2 <= (int64_t(256) << 20) &&
               sig_forward_chunked_workspace_bytes(B, L, d, N, basepoint, chunks * 2, dtype) >= 0)
            chunks *= 2;
        return chunks;
    }
    const int64_t shortest = (d == 8 && N >= 4 && N <= 6 && dtype == SIG_F32) ? 4096 : 512;
    if (B < 1 || B > 64 || sh.n_inc < shortest) return 1;
    const int64_t elem = dtype == SIG_F32 ? int64_t(sizeof(float)) : int64_t(sizeof(double));
    int chunks = 1;
    for (;;) {
        const int64_t next = int64_t(chunks) * 2;
        if (next > 65536 || next * B > 1024 || sh.n_inc / next < 64) break;
        if (next * B > (int64_t(256) << 20) / (sh.S * elem)) break;   // the products move every stretch's signature
        if (sig_forward_chunked_workspace_bytes(B, L, d, N, basepoint, int(next), dtype) < 0) break;
        chunks = int(next);
    }
    return chunks;
}

// The chunked scan itself; `use_static_scratch` selects the library's own scratch array instead of `workspace`.
static sig_status forward_chunked(const void *path, int64_t B, int64_t L, int d, int N, int basepoint,
                                  const void *basepoint_value, int chunks, sig_dtype dtype, void *out,
                                  void *workspace, int64_t workspace_bytes, bool use_static_scratch, hipStream_t hip_stream)
{
    if (dtype != SIG_F32 && dtype != SIG_F64) return SIG_ERR_INVALID_ARG;
    sig::Shape sh;
    const sig_status st = make_chunked_shape(B, L, d, N, basepoint, chunks, sh);
    if (st != SIG_OK) return st;
    if (!sh.basepoint && basepoint_value != nullptr) return SIG_ERR_INVALID_ARG;
    if (B == 0) return SIG_OK;
    const int64_t elem = dtype == SIG_F32 ? int64_t(sizeof(float)) : int64_t(sizeof(double));
    if (use_static_scratch) {
        if (path == nullptr || out == nullptr) return SIG_ERR_INVALID_ARG;
        if ((sh.B + sh.B / 2) * sh.S * elem > int64_t(SIG_STATIC_SCRATCH_BYTES)) return SIG_ERR_TOO_LARGE;
        workspace = scratch_on_current_device();
        if (workspace == nullptr) return SIG_ERR_HIP;
        workspace_bytes = int64_t(SIG_STATIC_SCRATCH_BYTES);
    }
    if (path == nullptr || out == nullptr || workspace == nullptr) return SIG_ERR_INVALID_ARG;
    if (workspace_bytes < (sh.B + sh.B / 2) * sh.S * elem || reinterpret_cast<uintptr_t>(workspace) % 16 != 0)
        return SIG_ERR_INVALID_ARG;
    sh.basepoint_value = basepoint_value;
    // Depth 2 is a plain sum over the increments (see sig_forward_n2.hip): the stretches' sums are added, not multiplied
    if (sig::forward_n2_chunked_supported(sh, dtype)) {
        const hipError_t err =
            dtype == SIG_F32 ? sig::launch_forward_n2_chunked_f32(sh, static_cast<const float *>(path), static_cast<float *>(workspace),
                                                                  static_cast<float *>(out), hip_stream)
                             : sig::launch_forward_n2_chunked_f64(sh, static_cast<const double *>(path), static_cast<double *>(workspace),
                                                                  static_cast<double *>(out), hip_stream);
        return err == hipSuccess ? SIG_OK : SIG_ERR_HIP;
    }
    if (!sig::combine_supported(sh)) return SIG_ERR_UNSUPPORTED;
    const Family family = resolve(sh, dtype, SIG_VARIANT_AUTO, path, workspace);
    if (family == Family::None) return SIG_ERR_UNSUPPORTED;
    // every chunk scanned on its own ...
    char *ws0 = static_cast<char *>(workspace);
    char *ws1 = ws0 + sh.B * sh.S * elem;
    if (launch_family(family, sh, dtype, path, ws0, hip_stream) != hipSuccess) return SIG_ERR_HIP;
    // ... then neighbours joined pairwise (Chen's identity), halving the count each round
    sig::Shape rows = sh;
    rows.chunks = 1;
    const char *src = ws0;
    char *spare = ws1;
    for (int64_t count = sh.B / 2; count >= B; count /= 2) {
        rows.B = count;
        char *dst = count == B ? static_cast<char *>(out) : spare;
        const int64_t strides[7] = {2 * sh.S, 2 * sh.S, sh.S, 0, 0, 0, 0};
        const hipError_t err =
            dtype == SIG_F32
                ? sig::launch_combine_f32(rows, reinterpret_cast<const float *>(src), reinterpret_cast<const float *>(src) + sh.S,
                                          reinterpret_cast<float *>(dst), hip_stream, strides)
                : sig::launch_combine_f64(rows, reinterpret_cast<const double *>(src), reinterpret_cast<const double *>(src) + sh.S,
                                          reinterpret_cast<double *>(dst), hip_stream, strides);
        if (err != hipSuccess) return SIG_ERR_HIP;
        spare = const_cast<char *>(src);
        src = dst;
    }
    return SIG_OK;
}

sig_status sig_forward_chunked(const void *path, int64_t B, int64_t L, int d, int N, int basepoint,
                               const void *basepoint_value, int chunks, sig_dtype dtype, void *out,
                               void *workspace, int64_t workspace_bytes, hipStream_t hip_stream)
{
    return forward_chunked(path, B, L, d, N, basepoint, basepoint_value, chunks, dtype, out, workspace, workspace_bytes,
                           false, hip_stream);
}

sig_status sig_forward_chunked_static(const void *path, int64_t B, int64_t L, int d, int N, int basepoint,
                                      const void *basepoint_value, int chunks, sig_dtype dtype, void *out,
                                      hipStream_t hip_stream)
{
    return forward_chunked(path, B, L, d, N, basepoint, basepoint_value, chunks, dtype, out, nullptr, 0, true, hip_stream);
}

int64_t sig_forward_chunked_static_max_bytes(void) { return int64_t(SIG_STATIC_SCRATCH_BYTES); }

int64_t sig_combine_many_workspace_bytes(int64_t B, int64_t n, int d, int N, sig_dtype dtype)
{
    if (dtype != SIG_F32 && dtype != SIG_F64) return -1;
    sig::Shape sh;
    if (n < 1 || make_rows_shape(B, d, N, sh) != SIG_OK) return -1;
    if (B > 0 && n > kMaxElems / sh.S / B) return -1;
    // two buffers: the results of the first round and of the second, reused alternately afterwards
    const int64_t first = (n + 1) / 2, second = (first + 1) / 2;
    return n <= 2 ? 0 : B * (first + (first > 2 ? second : 0)) * sh.S * int64_t(dtype == SIG_F32 ? sizeof(float) : sizeof(double));
}

sig_status sig_combine_many(const void *sigs, int64_t B, int64_t n, int d, int N, sig_dtype dtype, void *out,
                            void *workspace, int64_t workspace_bytes, hipStream_t hip_stream)
{
    if (dtype != SIG_F32 && dtype != SIG_F64) return SIG_ERR_INVALID_ARG;
    if (n < 1) return SIG_ERR_INVALID_ARG;
    sig::Shape sh;
    const sig_status st = make_rows_shape(B, d, N, sh);
    if (st != SIG_OK) return st;
    if (B > 0 && n > kMaxElems / sh.S / B) return SIG_ERR_OVERFLOW;
    if (B == 0) return SIG_OK;
    if (sigs == nullptr || out == nullptr) return SIG_ERR_INVALID_ARG;
    if (!sig::combine_supported(sh)) return SIG_ERR_UNSUPPORTED;
    const int64_t need = sig_combine_many_workspace_bytes(B, n, d, N, dtype);
    if (need > 0 && (workspace == nullptr || workspace_bytes < need || reinterpret_cast<uintptr_t>(workspace) % 16 != 0))
        return SIG_ERR_INVALID_ARG;
    const int64_t elem = dtype == SIG_F32 ? int64_t(sizeof(float)) : int64_t(sizeof(double));
    const int64_t S = sh.S;
    // rounds of pairwise products in order (the product is associative, not commutative); an odd one out is carried
    const char *src = static_cast<const char *>(sigs);
    int64_t count = n;
    const int64_t first = (n + 1) / 2;
    char *bufs[2] = {static_cast<char *>(workspace), static_cast<char *>(workspace) + B * first * S * elem};
    int which = 0;
    if (count == 1) {
        return hipMemcpyAsync(out, sigs, size_t(B * S * elem), hipMemcpyDeviceToDevice, hip_stream) == hipSuccess ? SIG_OK
                                                                                                             : SIG_ERR_HIP;
    }
    while (count > 1) {
        const int64_t pairs = count / 2, next = (count + 1) / 2;
        char *dst = next == 1 ? static_cast<char *>(out) : bufs[which];
        sig::Shape rows = sh;
        rows.B = B * pairs;
        const int64_t strides[7] = {2 * S, 2 * S, S, pairs, count * S, count * S, next * S};
        const hipError_t err =
            dtype == SIG_F32
                ? sig::launch_combine_f32(rows, reinterpret_cast<const float *>(src), reinterpret_cast<const float *>(src) + S,
                                          reinterpret_cast<float *>(dst), hip_stream, strides)
                : sig::launch_combine_f64(rows, reinterpret_cast<const double *>(src), reinterpret_cast<const double *>(src) + S,
                                          reinterpret_cast<double *>(dst), hip_stream, strides);
        if (err != hipSuccess) return SIG_ERR_HIP;
        if (count % 2 == 1) {
            // the last signature of every row moves on unchanged
            if (hipMemcpy2DAsync(dst + pairs * S * elem, size_t(next * S * elem), src + (count - 1) * S * elem,
                                 size_t(count * S * elem), size_t(S * elem), size_t(B), hipMemcpyDeviceToDevice,
                                 hip_stream) != hipSuccess)
                return SIG_ERR_HIP;
        }
        src = dst;
        count = next;
        which ^= 1;
    }
    return SIG_OK;
}

int64_t sig_logsignature_channels(int d, int N)
{
    sig::Shape sh;
    if (make_rows_shape(0, d, N, sh) != SIG_OK || sh.S >= (int64_t(1) << 31)) return -1;
    return sig::lyndon_indices_host(sh, nullptr, 0);
}

sig_status sig_lyndon_indices(int d, int N, int64_t *indices, int64_t capacity)
{
    sig::Shape sh;
    const sig_status st = make_rows_shape(0, d, N, sh);
    if (st != SIG_OK) return st;
    if (sh.S >= (int64_t(1) << 31)) return SIG_ERR_UNSUPPORTED;
    if (indices == nullptr || capacity < 0) return SIG_ERR_INVALID_ARG;
    return sig::lyndon_indices_host(sh, indices, capacity) < 0 ? SIG_ERR_INVALID_ARG : SIG_OK;
}

sig_status sig_log(const void *sig, int64_t rows, int d, int N, sig_dtype dtype, void *out, hipStream_t hip_stream)
{
    if (dtype != SIG_F32 && dtype != SIG_F64) return SIG_ERR_INVALID_ARG;
    sig::Shape sh;
    const sig_status st = make_rows_shape(rows, d, N, sh);
    if (st != SIG_OK) return st;
    if (rows == 0) return SIG_OK;
    if (sig == nullptr || out == nullptr || sig == out) return SIG_ERR_INVALID_ARG;
    if (!sig::combine_supported(sh)) return SIG_ERR_UNSUPPORTED;
    const hipError_t err =
        dtype == SIG_F32 ? sig::launch_log_f32(sh, static_cast<const float *>(sig), static_cast<float *>(out), hip_stream)
                         : sig::launch_log_f64(sh, static_cast<const double *>(sig), static_cast<double *>(out), hip_stream);
    return err == hipSuccess ? SIG_OK : SIG_ERR_HIP;
}

sig_status sig_lyndon_gather(const void *log_sig, int64_t rows, int d, int N, const int64_t *indices, int64_t n,
                             sig_dtype dtype, void *out, hipStream_t hip_stream)
{
    if (dtype != SIG_F32 && dtype != SIG_F64) return SIG_ERR_INVALID_ARG;
    sig::Shape sh;
    const sig_status st = make_rows_shape(rows, d, N, sh);
    if (st != SIG_OK) return st;
    if (n < 0 || n > sh.S) return SIG_ERR_INVALID_ARG;
    if (rows == 0 || n == 0) return SIG_OK;
    if (log_sig == nullptr || indices == nullptr || out == nullptr) return SIG_ERR_INVALID_ARG;
    const hipError_t err =
        dtype == SIG_F32
            ? sig::launch_gather_f32(sh, static_cast<const float *>(log_sig), indices, n, static_cast<float *>(out), hip_stream)
            : sig::launch_gather_f64(sh, static_cast<const double *>(log_sig), indices, n, static_cast<double *>(out), hip_stream);
    return err == hipSuccess ? SIG_OK : SIG_ERR_HIP;
}

int64_t sig_log_backward_workspace_bytes(int64_t rows, int d, int N, sig_dtype dtype)
{
    if (dtype != SIG_F32 && dtype != SIG_F64) return -1;
    sig::Shape sh;
    if (make_rows_shape(rows, d, N, sh) != SIG_OK || !sig::combine_supported(sh)) return -1;
    return sig::log_backward_workspace_bytes(sh, dtype);
}

sig_status sig_log_backward(const void *sig, const void *grad_log, int64_t rows, int d, int N, sig_dtype dtype,
                            void *grad_sig, void *workspace, int64_t workspace_bytes, hipStream_t hip_stream)
{
    if (dtype != SIG_F32 && dtype != SIG_F64) return SIG_ERR_INVALID_ARG;
    sig::Shape sh;
    const sig_status st = make_rows_shape(rows, d, N, sh);
    if (st != SIG_OK) return st;
    if (rows == 0) return SIG_OK;
    if (sig == nullptr || grad_log == nullptr || grad_sig == nullptr || grad_sig == sig || grad_sig == grad_log)
        return SIG_ERR_INVALID_ARG;
    if (!sig::combine_supported(sh)) return SIG_ERR_UNSUPPORTED;
    const int64_t need = sig::log_backward_workspace_bytes(sh, dtype);
    if (need > 0 && (workspace == nullptr || workspace_bytes < need || reinterpret_cast<uintptr_t>(workspace) % 16 != 0))
        return SIG_ERR_INVALID_ARG;
    const hipError_t err =
        dtype == SIG_F32 ? sig::launch_log_backward_f32(sh, static_cast<const float *>(sig), static_cast<const float *>(grad_log),
                                                        static_cast<float *>(grad_sig), workspace, hip_stream)
                         : sig::launch_log_backward_f64(sh, static_cast<const double *>(sig), static_cast<const double *>(grad_log),
                                                        static_cast<double *>(grad_sig), workspace, hip_stream);
    return err == hipSuccess ? SIG_OK : err == hipErrorNotSupported ? SIG_ERR_UNSUPPORTED : SIG_ERR_HIP;
}

int64_t sig_combine_backward_workspace_bytes(int64_t B, int d, int N, sig_dtype dtype)
{
    if (dtype != SIG_F32 && dtype != SIG_F64) return -1;
    sig::Shape sh;
    if (make_rows_shape(B, d, N, sh) != SIG_OK || !sig::combine_supported(sh)) return -1;
    return sig::combine_backward_workspace_bytes(sh, dtype);
}

sig_status sig_combine_backward(const void *a, const void *b, const void *grad_out, int64_t B, int d, int N, sig_dtype dtype,
                                void *grad_a, void *grad_b, void *workspace, int64_t workspace_bytes, hipStream_t hip_stream)
{
    if (dtype != SIG_F32 && dtype != SIG_F64) return SIG_ERR_INVALID_ARG;
    sig::Shape sh;
    const sig_status st = make_rows_shape(B, d, N, sh);
    if (st != SIG_OK) return st;
    if (B == 0) return SIG_OK;
    if (a == nullptr || b == nullptr || grad_out == nullptr || grad_a == nullptr || grad_b == nullptr || grad_a == grad_b ||
        grad_a == grad_out || grad_b == grad_out || grad_a == a || grad_a == b || grad_b == a || grad_b == b)
        return SIG_ERR_INVALID_ARG;
    if (!sig::combine_supported(sh)) return SIG_ERR_UNSUPPORTED;
    const int64_t need = sig::combine_backward_workspace_bytes(sh, dtype);
    if (need > 0 && (workspace == nullptr || workspace_bytes < need || reinterpret_cast<uintptr_t>(workspace) % 16 != 0))
        return SIG_ERR_INVALID_ARG;
    const hipError_t err =
        dtype == SIG_F32
            ? sig::launch_combine_backward_f32(sh, static_cast<const float *>(a), static_cast<const float *>(b),
                                               static_cast<const float *>(grad_out), static_cast<float *>(grad_a),
                                               static_cast<float *>(grad_b), workspace, hip_stream)
            : sig::launch_combine_backward_f64(sh, static_cast<const double *>(a), static_cast<const double *>(b),
                                               static_cast<const double *>(grad_out), static_cast<double *>(grad_a),
                                               static_cast<double *>(grad_b), workspace, hip_stream);
    return err == hipSuccess ? SIG_OK : err == hipErrorNotSupported ? SIG_ERR_UNSUPPORTED : SIG_ERR_HIP;
}

sig_status sig_combine_grouped(const void *a, const void *sigs, int64_t B, int64_t group, int d, int N, sig_dtype dtype,
                               void *out, hipStream_t hip_stream)
{
    if (dtype != SIG_F32 && dtype != SIG_F64) return SIG_ERR_INVALID_ARG;
    if (B < 0 || group < 1 || (B > 0 && group > INT64_MAX / B)) return SIG_ERR_INVALID_ARG;
    sig::Shape sh;
    const sig_status st = make_rows_shape(B * group, d, N, sh);
    if (st != SIG_OK) return st;
    if (B == 0) return SIG_OK;
    if (a == nullptr || sigs == nullptr || out == nullptr || out == a) return SIG_ERR_INVALID_ARG;
    if (!sig::combine_supported(sh)) return SIG_ERR_UNSUPPORTED;
    const size_t elem = dtype == SIG_F32 ? sizeof(float) : sizeof(double);
    if (out != sigs && hipMemcpyAsync(out, sigs, size_t(sh.B) * size_t(sh.S) * elem, hipMemcpyDeviceToDevice, hip_stream) != hipSuccess)
        return SIG_ERR_HIP;
    const hipError_t err =
        dtype == SIG_F32 ? sig::launch_left_mul_f32(sh, static_cast<const float *>(a), group, static_cast<float *>(out), hip_stream)
                         : sig::launch_left_mul_f64(sh, static_cast<const double *>(a), group, static_cast<double *>(out), hip_stream);
    return err == hipSuccess ? SIG_OK : SIG_ERR_HIP;
}

int64_t sig_combine_grouped_backward_workspace_bytes(int64_t B, int64_t group, int d, int N, sig_dtype dtype)
{
    if (dtype != SIG_F32 && dtype != SIG_F64) return -1;
    if (B < 0 || group < 1 || (B > 0 && group > INT64_MAX / B)) return -1;
    sig::Shape sh;
    if (make_rows_shape(B * group, d, N, sh) != SIG_OK || !sig::combine_supported(sh)) return -1;
    return sig::combine_grouped_backward_workspace_bytes(sh, dtype);
}

sig_status sig_combine_grouped_backward(const void *a, const void *sigs, const void *grad_out, int64_t B, int64_t group, int d,
                                        int N, sig_dtype dtype, void *grad_a, void *grad_sigs, void *workspace,
                                        int64_t workspace_bytes, hipStream_t hip_stream)
{
    if (dtype != SIG_F32 && dtype != SIG_F64) return SIG_ERR_INVALID_ARG;
    if (B < 0 || group < 1 || (B > 0 && group > INT64_MAX / B)) return SIG_ERR_INVALID_ARG;
    sig::Shape sh;
    const sig_status st = make_rows_shape(B * group, d, N, sh);
    if (st != SIG_OK) return st;
    if (B == 0) return SIG_OK;
    if (a == nullptr || sigs == nullptr || grad_out == nullptr || grad_a == nullptr || grad_sigs == nullptr ||
        grad_a == grad_sigs || grad_a == grad_out || grad_sigs == grad_out || grad_a == a || grad_a == sigs || grad_sigs == a ||
        grad_sigs == sigs)
        return SIG_ERR_INVALID_ARG;
    if (!sig::combine_supported(sh)) return SIG_ERR_UNSUPPORTED;
    const int64_t need = sig::combine_grouped_backward_workspace_bytes(sh, dtype);
    if (workspace == nullptr || workspace_bytes < need || reinterpret_cast<uintptr_t>(workspace) % 16 != 0)
        return SIG_ERR_INVALID_ARG;
    const hipError_t err =
        dtype == SIG_F32
            ? sig::launch_combine_grouped_backward_f32(sh, group, static_cast<const float *>(a), static_cast<const float *>(sigs),
                                                       static_cast<const float *>(grad_out), static_cast<float *>(grad_a),
                                                       static_cast<float *>(grad_sigs), workspace, hip_stream)
            : sig::launch_combine_grouped_backward_f64(sh, group, static_cast<const double *>(a), static_cast<const double *>(sigs),
                                                       static_cast<const double *>(grad_out), static_cast<double *>(grad_a),
                                                       static_cast<double *>(grad_sigs), workspace, hip_stream);
    return err == hipSuccess ? SIG_OK : err == hipErrorNotSupported ? SIG_ERR_UNSUPPORTED : SIG_ERR_HIP;
}

sig_status sig_lyndon_scatter(const void *grad_logsig, int64_t rows, int d, int N, const int64_t *indices, int64_t n,
                              sig_dtype dtype, void *grad_log, hipStream_t hip_stream)
{
    if (dtype != SIG_F32 && dtype != SIG_F64) return SIG_ERR_INVALID_ARG;
    sig::Shape sh;
    const sig_status st = make_rows_shape(rows, d, N, sh);
    if (st != SIG_OK) return st;
    if (n < 0 || n > sh.S) return SIG_ERR_INVALID_ARG;
    if (rows == 0) return SIG_OK;
    if (grad_log == nullptr || (n > 0 && (grad_logsig == nullptr || indices == nullptr))) return SIG_ERR_INVALID_ARG;
    const hipError_t err =
        dtype == SIG_F32 ? sig::launch_scatter_f32(sh, static_cast<const float *>(grad_logsig), indices, n,
                                                   static_cast<float *>(grad_log), hip_stream)
                         : sig::launch_scatter_f64(sh, static_cast<const double *>(grad_logsig), indices, n,
                                                   static_cast<double *>(grad_log), hip_stream);
    return err == hipSuccess ? SIG_OK : SIG_ERR_HIP;
}

sig_status sig_signature(const void *path, int64_t B, int64_t L, int d, int N, int stream, int basepoint,
                         const void *basepoint_value, const void *initial, int inverse, sig_dtype dtype,
                         void *out, hipStream_t hip_stream)
{
    if (dtype != SIG_F32 && dtype != SIG_F64) return SIG_ERR_INVALID_ARG;
    sig::Shape sh;
    const sig_status st = make_shape(B, L, d, N, stream, basepoint, sh);
    if (st != SIG_OK) return st;
    if (!sh.basepoint && basepoint_value != nullptr) return SIG_ERR_INVALID_ARG;
    if (B == 0) return SIG_OK;
    if (path == nullptr || out == nullptr) return SIG_ERR_INVALID_ARG;
    sh.basepoint_value = basepoint_value;
    if ((initial != nullptr || inverse) && !sig::combine_supported(sh)) return SIG_ERR_UNSUPPORTED;
    const Family family = resolve(sh, dtype, SIG_VARIANT_AUTO, path, out);
    if (family == Family::None) return SIG_ERR_UNSUPPORTED;
    hipError_t err = launch_family(family, sh, dtype, path, out, hip_stream);
    if (err != hipSuccess) return SIG_ERR_HIP;
    // what follows works on the rows of `out`, in place, behind the scan on the same stream
    sig::Shape rows = sh;
    rows.B = sh.B * (sh.stream ? sh.n_inc : 1);
    if (initial != nullptr) {
        const int64_t group = sh.stream ? sh.n_inc : 1;
        err = dtype == SIG_F32
                  ? sig::launch_left_mul_f32(rows, static_cast<const float *>(initial), group, static_cast<float *>(out), hip_stream)
                  : sig::launch_left_mul_f64(rows, static_cast<const double *>(initial), group, static_cast<double *>(out), hip_stream);
        if (err != hipSuccess) return SIG_ERR_HIP;
    }
    if (inverse) {
        err = dtype == SIG_F32
                  ? sig::launch_invert_f32(rows, static_cast<const float *>(out), static_cast<float *>(out), hip_stream)
                  : sig::launch_invert_f64(rows, static_cast<const double *>(out), static_cast<double *>(out), hip_stream);
        if (err != hipSuccess) return SIG_ERR_HIP;
    }
    return SIG_OK;
}

sig_status sig_forward(const void *path, int64_t B, int64_t L, int d, int N,
                       int stream, int basepoint, sig_dtype dtype,
                       void *out, hipStream_t hip_stream)
{
    return sig_forward_variant(path, B, L, d, N, stream, basepoint, dtype, out, hip_stream, SIG_VARIANT_AUTO);
}

const char *sig_variant_name(int64_t B, int64_t L, int d, int N, int stream, int basepoint,
                             sig_dtype dtype, sig_variant variant)
{
    if (!valid_enums(dtype, variant)) return "invalid";
    sig::Shape sh;
    if (make_shape(B, L, d, N, stream, basepoint, sh) != SIG_OK) return "invalid";
    switch (resolve(sh, dtype, variant, nullptr, nullptr)) {
        case Family::Mfma: return sig::mfma_kernel_name(sh);
        case Family::MfmaShard: return sig::mfma_shard_kernel_name(sh);
        case Family::MfmaStream: return sig::mfma_stream_kernel_name(sh);
        case Family::MfmaD16: return sig::mfma_d16_kernel_name(sh);
        case Family::MfmaD8: return sig::mfma_d8_kernel_name(sh);
        case Family::Small: return "small";
        case Family::Tree: return "tree";
        case Family::RowStream: return "row_stream";
        case Family::Wide: return "wide";
        case Family::Depth2: return "depth2";
        case Family::Generic: return "generic";
        case Family::None: break;
    }
    return "unsupported";
}

const char *sig_status_string(sig_status status)
{
    switch (status) {
        case SIG_OK: return "ok";
        case SIG_ERR_INVALID_ARG: return "invalid argument";
        case SIG_ERR_UNSUPPORTED: return "no kernel variant supports this request";
        case SIG_ERR_OVERFLOW: return "size overflow";
        case SIG_ERR_HIP: return "HIP launch failed";
        case SIG_ERR_TOO_LARGE: return "the request needs more scratch memory than the library's fixed buffer holds";
    }
    return "unknown status";
}

}  // extern "C"
