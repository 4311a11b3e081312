// Gradient of the depth-2 signature with respect to the path, final mode, any channel count, fp32 and fp64, with no
// scan at all (paper section 5.3; the closed form below is what the recurrences of sig_backward.hip sum up to at N = 2).
//
// With increments z_s = b_s - a_s (a_s, b_s the points increment s runs between), p the point the scan starts from
// and q the point it ends at, the depth-2 signature is (sections 2.1, 2.2)
//     A_1 = q - p,     A_2 = sum_s (a_s - p + z_s / 2) (x) z_s.
// z_s enters A_2 as the right factor of its own term, as half of the left factor of its own term, and through a_t - p
// in every later term; with m_s = (a_s + b_s) / 2 the midpoint of increment s and G_1, G_2 the output gradient,
//     dL/dz_s = G_1 + G_2^T (m_s - p) + G_2 (q - m_s),
// and a point's gradient is that of the increment it ends minus that of the increment it starts.  Every increment on
// its own: a thread per point and channel, two dot products of length d with a row and a column of G_2, which a
// workgroup keeps in LDS (rows padded by one scalar, so that walking a column hits different banks).
#include "sig_internal.h"

namespace sig {
namespace {

template <typename T>
__global__ void __launch_bounds__(256)
sig_backward_n2_kernel(Shape sh, int points_per_group, int passes, const T *__restrict__ path, const T *__restrict__ gout,
                       T *__restrict__ gpath, T *__restrict__ gbase)
{
    extern __shared__ __align__(16) unsigned char n2_smem[];
    const int d = sh.d, ld = d + 1;
    T *G2 = reinterpret_cast<T *>(n2_smem);    // [d][d + 1]
    T *G1 = G2 + d * ld;                       // [d]
    T *va = G1 + d;                            // [points_per_group + 1][d]: coefficient vectors of G_2^T, see below
    T *vb = va + (points_per_group + 1) * d;   // the same for G_2
    T *vc = vb + (points_per_group + 1) * d;   // [points_per_group + 1]: coefficient of G_1

    const int tid = threadIdx.x;
    // a workgroup loads the output gradient of its path once and serves `passes` runs of points_per_group points
    const int64_t points_per_wg = int64_t(points_per_group) * passes;
    const int64_t groups_per_path = (sh.L + points_per_wg - 1) / points_per_wg;
    const int64_t b = blockIdx.x / groups_per_path;
    const int64_t l_first = (blockIdx.x % groups_per_path) * points_per_wg;
    const T *x = path + b * sh.L * d;
    const T *go = gout + b * sh.S;
    const T *bpv = static_cast<const T *>(sh.basepoint_value);

    for (int e = tid; e < d * d; e += 256) {
        const int i = e / d, j = e - i * d;
        G2[i * ld + j] = go[d + e];
    }
    for (int e = tid; e < d; e += 256) G1[e] = go[e];

    // Point l (slot r = l - l0) ends increment l - 1 (l with a basepoint) and starts the next one; slot
    // points_per_group of the first workgroup stands for the basepoint, which starts increment 0.  Its gradient is
    //     [ends] (G_1 + G_2^T (m_e - p) + G_2 (q - m_e)) - [starts] (G_1 + G_2^T (m_s - p) + G_2 (q - m_s))
    // = vc G_1 + G_2^T va + G_2 vb with the vectors formed here.
    const int64_t last = sh.L - 1;
    for (int pass = 0; pass < passes; ++pass) {
    const int64_t l0 = l_first + int64_t(pass) * points_per_group;
    if (l0 > last) break;
    __syncthreads();   // the vectors of the pass before have been used
    for (int e = tid; e < (points_per_group + 1) * d; e += 256) {
        const int r = e / d, c = e - r * d;
        const bool base_slot = r == points_per_group;
        const int64_t l = base_slot ? -1 : l0 + r;
        const bool exists = base_slot ? (sh.basepoint && l0 == 0) : l <= last;
        // the increments around the point, numbered inside the scan: inc = l + 1 starts at l; inc = l ends at l
        // (with a basepoint the scan's points are bp, x_0, x_1, ..: point l has number l + 1)
        const int64_t k = sh.basepoint ? l + 1 : l;          // the point's number inside the scan, 0 .. n_inc
        const bool ends = exists && k >= 1, starts = exists && k <= sh.n_inc - 1;
        auto scan_point = [&](int64_t kk) -> T {             // channel c of point number kk of the scan
            if (sh.basepoint) return kk == 0 ? (bpv != nullptr ? bpv[b * d + c] : T(0)) : x[(kk - 1) * d + c];
            return x[kk * d + c];
        };
        T a = T(0), bb = T(0);
        if (exists) {
            // Differences of points only (a path far from the origin loses nothing): m_e - p is (X_{k-1} - p) plus half
            // of increment e, and an interior point keeps m_{k-1} - m_k = (X_{k-1} - X_{k+1}) / 2 alone.
            const T p = scan_point(0), q = scan_point(sh.n_inc), here = scan_point(k);
            if (ends && starts) {
                a = (scan_point(k - 1) - scan_point(k + 1)) * T(0.5);
                bb = -a;
            } else if (ends) {
                const T before = scan_point(k - 1), half = (here - before) * T(0.5);
                a = (before - p) + half;
                bb = (q - here) + half;
            } else if (starts) {
                const T after = scan_point(k + 1), half = (after - here) * T(0.5);
                a = -((here - p) + half);
                bb = -((q - after) + half);
            }
        }
        va[e] = a;
        vb[e] = bb;
        if (c == 0) vc[r] = T(ends ? 1 : 0) - T(starts ? 1 : 0);
    }
    __syncthreads();

    for (int e = tid; e < (points_per_group + 1) * d; e += 256) {
        const int r = e / d, j = e - r * d;
        const bool base_slot = r == points_per_group;
        const int64_t l = l0 + r;
        if (base_slot ? !(sh.basepoint && l0 == 0 && gbase != nullptr) : l > last) continue;
        const T *ar = va + r * d, *br = vb + r * d;
        T acc = vc[r] * G1[j];
        for (int i = 0; i < d; ++i) acc += ar[i] * G2[i * ld + j] + br[i] * G2[j * ld + i];
        if (base_slot)
            gbase[b * d + j] = acc;
        else
            gpath[(b * sh.L + l) * d + j] = acc;
    }
    }
}

template <typename T>
size_t n2_lds_bytes(int d, int points_per_group)
{
    return sizeof(T) * (size_t(d) * (d + 1) + d + size_t(points_per_group + 1) * (2 * d + 1));
}

int n2_points_per_group(int d) { return d >= 128 ? 2 : 256 / d; }

// Runs of points per workgroup: enough that loading the d x d output gradient (once per workgroup) is shared by about
// 64 points, as long as that still leaves a few hundred workgroups.
int n2_passes(const Shape &sh)
{
    const int ppg = n2_points_per_group(sh.d);
    int passes = (64 + ppg - 1) / ppg;
    while (passes > 1 && sh.B * ((sh.L + int64_t(ppg) * passes - 1) / (int64_t(ppg) * passes)) < 512) passes /= 2;
    return passes < 1 ? 1 : passes;
}

template <typename T>
hipError_t launch_backward_n2_t(const Shape &sh, const T *path, const T *gout, T *gpath, T *gbase, hipStream_t st)
{
    const int ppg = n2_points_per_group(sh.d);
    const size_t lds = n2_lds_bytes<T>(sh.d, ppg);
    const int passes = n2_passes(sh);
    const int64_t groups = sh.B * ((sh.L + int64_t(ppg) * passes - 1) / (int64_t(ppg) * passes));
    if (lds > 64 * 1024 || groups > 0x7fffffff) return hipErrorNotSupported;
    hipLaunchKernelGGL((sig_backward_n2_kernel<T>), dim3(unsigned(groups)), dim3(256), lds, st, sh, ppg, passes, path, gout, gpath,
                       gbase);
    return hipGetLastError();
}

}  // namespace

bool backward_n2_supported(const Shape &sh, sig_dtype dtype)
{
    // the closed form is the gradient of a row's own signature: it does not serve a stretch of a longer path
    if (sh.N != 2 || sh.stream || sh.chunks > 1 || !sh.from_identity || sh.d < 1 || sh.d > 255) return false;
    const int ppg = n2_points_per_group(sh.d);
    const size_t lds = dtype == SIG_F32 ? n2_lds_bytes<float>(sh.d, ppg) : n2_lds_bytes<double>(sh.d, ppg);
    return lds <= 64 * 1024 && sh.B * ((sh.L + ppg - 1) / ppg) <= 0x7fffffff;
}

hipError_t launch_backward_n2_f32(const Shape &sh, const float *path, const float *gout, float *gpath, float *gbase, hipStream_t st)
{
    return launch_backward_n2_t<float>(sh, path, gout, gpath, gbase, st);
}

hipError_t launch_backward_n2_f64(const Shape &sh, const double *path, const double *gout, double *gpath, double *gbase,
                                  hipStream_t st)
{
    return launch_backward_n2_t<double>(sh, path, gout, gpath, gbase, st);
}

}  // namespace sig
