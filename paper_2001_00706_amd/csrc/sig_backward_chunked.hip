// Pieces of the gradient of few long paths, the scan cut into stretches (final mode; paper sections 5.1 and 5.3).
//
// The gradient by reversibility (appendix C.1) walks a path backwards an increment at a time, so one path keeps one
// workgroup busy for its whole length.  Cut into K stretches of m increments, with C_c the signature of stretch c alone
// and S_c = C_0 [x] .. [x] C_c that of the path up to the end of stretch c (Chen's identity, section 2.2), the walk
// over stretch c needs two things at its end: S_c, and the gradient g_c of the loss with respect to S_c.  The first is
// a running product.  The second follows from S_c = S_{c-1} [x] C_c, which is linear in S_{c-1}:
//     g_{c-1}[u] = sum_v g_c[u v] C_c[v],      v over all words with |u v| <= N, the empty one (C[empty] = 1) included,
// starting from g_{K-1} = the gradient with respect to the whole signature.  Given both, the stretches are independent
// and the ordinary gradient kernels serve them as B K short paths.  This file holds the plumbing around them: copying
// the stretches out as paths of their own (m + 1 points, the last point of a path repeated where the last stretch is
// short: increments of zero change no signature), the chain of g_c, and adding the stretches' point gradients up (a
// point shared by two stretches ends an increment of one and starts one of the other; the repeated last points sum to
// the gradient of the increment that ends at the real one).
#include "sig_internal.h"

namespace sig {
namespace {

template <typename T>
__global__ void __launch_bounds__(256)
sig_stretch_gather_kernel(Shape sh, int64_t K, int64_t m, const T *__restrict__ path, T *__restrict__ rows)
{
    const int d = sh.d;
    const int64_t per_row = (m + 1) * d, total = sh.B * K * per_row;
    const T *bpv = static_cast<const T *>(sh.basepoint_value);
    for (int64_t e = int64_t(blockIdx.x) * 256 + threadIdx.x; e < total; e += int64_t(gridDim.x) * 256) {
        const int64_t r = e / per_row, rest = e - r * per_row;
        const int64_t i = rest / d;
        const int ch = int(rest - i * d);
        const int64_t b = r / K, c = r - b * K;
        int64_t k = c * m + i;   // number of the point inside the scan, 0 .. n_inc
        if (k > sh.n_inc) k = sh.n_inc;
        T v;
        if (sh.basepoint)
            v = k == 0 ? (bpv != nullptr ? bpv[b * d + ch] : T(0)) : path[(b * sh.L + k - 1) * d + ch];
        else
            v = path[(b * sh.L + k) * d + ch];
        rows[e] = v;
    }
}

// dst[r][0 .. len) = src[r][0 .. len) for `rows` rows that lie src_stride and dst_stride scalars apart
template <typename T>
__global__ void __launch_bounds__(256)
sig_copy_rows_kernel(const T *__restrict__ src, int64_t src_stride, T *__restrict__ dst, int64_t dst_stride, int64_t len, int64_t rows)
{
    const int64_t total = rows * len;
    for (int64_t e = int64_t(blockIdx.x) * 256 + threadIdx.x; e < total; e += int64_t(gridDim.x) * 256) {
        const int64_t r = e / len, i = e - r * len;
        dst[r * dst_stride + i] = src[r * src_stride + i];
    }
}

// g[b][c - 1] = the gradient g[b][c] carried through the right multiplication by C[b][c] (rows of K signatures per
// path).  For a word u of level i the sum over the words v of level j is a dot product of d^j consecutive scalars of
// level i + j of g with level j of C.  Words whose sums are long (levels up to `wave_levels`) take a wavefront each,
// lanes striding over v, the rest a lane each; either way the order of the additions is fixed.
template <typename T>
__global__ void __launch_bounds__(256)
sig_stretch_adjoint_kernel(Shape sh, int64_t K, int64_t c, int wave_levels, const T *__restrict__ C, T *g)
{
    const int64_t b = blockIdx.y;
    const T *gin = g + (b * K + c) * sh.S, *cs = C + (b * K + c) * sh.S;
    T *gout = g + (b * K + c - 1) * sh.S;
    const int N = sh.N, lane = threadIdx.x & 63;
    const int64_t wave_words = sh.off[wave_levels + 1];   // words of levels 1 .. wave_levels
    const int64_t lane_waves = (sh.S - wave_words + 63) / 64;
    const int64_t waves = wave_words + lane_waves;
    for (int64_t w = int64_t(blockIdx.x) * 4 + (threadIdx.x >> 6); w < waves; w += int64_t(gridDim.x) * 4) {
        if (w < wave_words) {
            const int64_t e = w;
            int i = 1;
            while (e >= sh.off[i + 1]) ++i;
            const int64_t u = e - sh.off[i];
            T acc = T(0);
            for (int j = 1; i + j <= N; ++j) {
                const T *seg = gin + sh.off[i + j] + u * sh.pw[j], *cj = cs + sh.off[j];
                for (int64_t v = lane; v < sh.pw[j]; v += 64) acc += seg[v] * cj[v];
            }
#pragma unroll
            for (int step = 32; step >= 1; step >>= 1) acc += __shfl_xor(acc, step, 64);
            if (lane == 0) gout[e] = gin[e] + acc;
        } else {
            const int64_t e = wave_words + (w - wave_words) * 64 + lane;
            if (e < sh.S) {
                int i = 1;
                while (e >= sh.off[i + 1]) ++i;
                const int64_t u = e - sh.off[i];
                T acc = gin[e];
                for (int j = 1; i + j <= N; ++j) {
                    const T *seg = gin + sh.off[i + j] + u * sh.pw[j], *cj = cs + sh.off[j];
                    for (int64_t v = 0; v < sh.pw[j]; ++v) acc += seg[v] * cj[v];
                }
                gout[e] = acc;
            }
        }
    }
}

// Point gradients of the stretches [B K][m + 1][d] added up into those of the paths (and of the basepoints).
template <typename T>
__global__ void __launch_bounds__(256)
sig_stretch_scatter_kernel(Shape sh, int64_t K, int64_t m, const T *__restrict__ grows, T *__restrict__ gpath, T *__restrict__ gbase)
{
    const int d = sh.d;
    const int64_t n = sh.n_inc, per_path = (n + 1) * d, total = sh.B * per_path, per_row = (m + 1) * d;
    for (int64_t e = int64_t(blockIdx.x) * 256 + threadIdx.x; e < total; e += int64_t(gridDim.x) * 256) {
        const int64_t b = e / per_path, rest = e - b * per_path;
        const int64_t k = rest / d;   // number of the point inside the scan
        const int ch = int(rest - k * d);
        const T *rows = grows + b * K * per_row;
        T sum;
        if (k < n) {
            const int64_t c = k / m, i = k - c * m;
            sum = rows[c * per_row + i * d + ch];
            if (i == 0 && c > 0) sum += rows[(c - 1) * per_row + m * d + ch];   // it also ends the stretch before
        } else {
            // the last point and its copies behind it in the last stretch
            const int64_t c = (n - 1) / m;
            sum = T(0);
            for (int64_t i = n - c * m; i <= m; ++i) sum += rows[c * per_row + i * d + ch];
        }
        if (sh.basepoint) {
            if (k == 0) {
                if (gbase != nullptr) gbase[b * d + ch] = sum;
            } else {
                gpath[(b * sh.L + k - 1) * d + ch] = sum;
            }
        } else {
            gpath[(b * sh.L + k) * d + ch] = sum;
        }
    }
}

unsigned grid_for(int64_t elems)
{
    const int64_t groups = (elems + 255) / 256;
    return unsigned(groups < 1 ? 1 : groups < 65536 ? groups : 65536);
}

template <typename T>
hipError_t stretch_gather(const Shape &sh, int64_t K, int64_t m, const T *path, T *rows, hipStream_t st)
{
    hipLaunchKernelGGL((sig_stretch_gather_kernel<T>), dim3(grid_for(sh.B * K * (m + 1) * sh.d)), dim3(256), 0, st, sh, K, m, path, rows);
    return hipGetLastError();
}

template <typename T>
hipError_t copy_rows(const T *src, int64_t src_stride, T *dst, int64_t dst_stride, int64_t len, int64_t rows, hipStream_t st)
{
    hipLaunchKernelGGL((sig_copy_rows_kernel<T>), dim3(grid_for(rows * len)), dim3(256), 0, st, src, src_stride, dst, dst_stride, len, rows);
    return hipGetLastError();
}

template <typename T>
hipError_t stretch_adjoint_chain(const Shape &sh, int64_t K, const T *C, T *g, hipStream_t st)
{
    // a word's sums are sum_{j = 1 .. N - i} d^j multiply-adds long: a wavefront each from 256 on
    int wave_levels = 0;
    for (int i = 1; i < sh.N; ++i) {
        int64_t cost = 0;
        for (int j = 1; i + j <= sh.N; ++j) cost += sh.pw[j];
        if (cost >= 256) wave_levels = i;
    }
    const int64_t waves = sh.off[wave_levels + 1] + (sh.S - sh.off[wave_levels + 1] + 63) / 64;
    const int64_t groups = (waves + 3) / 4;
    const dim3 grid(unsigned(groups < 4096 ? groups : 4096), unsigned(sh.B / K));   // sh.B counts stretches
    for (int64_t c = K - 1; c >= 1; --c) {
        hipLaunchKernelGGL((sig_stretch_adjoint_kernel<T>), grid, dim3(256), 0, st, sh, K, c, wave_levels, C, g);
        const hipError_t err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    return hipSuccess;
}

template <typename T>
hipError_t stretch_scatter(const Shape &sh, int64_t K, int64_t m, const T *grows, T *gpath, T *gbase, hipStream_t st)
{
    hipLaunchKernelGGL((sig_stretch_scatter_kernel<T>), dim3(grid_for(sh.B * (sh.n_inc + 1) * sh.d)), dim3(256), 0, st, sh, K, m, grows,
                       gpath, gbase);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_stretch_gather(const Shape &sh, sig_dtype dtype, int64_t K, int64_t m, const void *path, void *rows, hipStream_t st)
{
    return dtype == SIG_F32 ? stretch_gather(sh, K, m, static_cast<const float *>(path), static_cast<float *>(rows), st)
                            : stretch_gather(sh, K, m, static_cast<const double *>(path), static_cast<double *>(rows), st);
}

hipError_t launch_copy_rows(sig_dtype dtype, const void *src, int64_t src_stride, void *dst, int64_t dst_stride, int64_t len,
                            int64_t rows, hipStream_t st)
{
    return dtype == SIG_F32
               ? copy_rows(static_cast<const float *>(src), src_stride, static_cast<float *>(dst), dst_stride, len, rows, st)
               : copy_rows(static_cast<const double *>(src), src_stride, static_cast<double *>(dst), dst_stride, len, rows, st);
}

hipError_t launch_stretch_adjoint_chain(const Shape &sh, sig_dtype dtype, int64_t K, const void *C, void *g, hipStream_t st)
{
    return dtype == SIG_F32 ? stretch_adjoint_chain(sh, K, static_cast<const float *>(C), static_cast<float *>(g), st)
                            : stretch_adjoint_chain(sh, K, static_cast<const double *>(C), static_cast<double *>(g), st);
}

hipError_t launch_stretch_scatter(const Shape &sh, sig_dtype dtype, int64_t K, int64_t m, const void *grows, void *gpath, void *gbase,
                                  hipStream_t st)
{
    return dtype == SIG_F32
               ? stretch_scatter(sh, K, m, static_cast<const float *>(grows), static_cast<float *>(gpath), static_cast<float *>(gbase), st)
               : stretch_scatter(sh, K, m, static_cast<const double *>(grows), static_cast<double *>(gpath), static_cast<double *>(gbase),
                                 st);
}

}  // namespace sig
