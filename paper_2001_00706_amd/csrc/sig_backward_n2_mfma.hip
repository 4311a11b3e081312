// Gradient of the depth-2 signature in final mode on the matrix cores (fp32, 8 to 112 channels).
//
// The closed form of sig_backward_n2.hip (paper section 5.3 at N = 2): with X_0 .. X_n the points of the scan,
// m_s = (X_s + X_{s+1}) / 2, p = X_0, q = X_n and G_1, G_2 the output gradient,
//     dL/dz_s = G_1 + G_2^T (m_s - p) + G_2 (q - m_s),
// and a point's gradient is that of the increment it ends minus that of the increment it starts.  For an interior point
// X_k the two differ by m_{k-1} - m_k = (X_{k-1} - X_{k+1}) / 2 only:
//     dL/dX_k [j] = sum_i v_k[i] (G_2[i][j] - G_2[j][i]),   v_k = (X_{k-1} - X_{k+1}) / 2,
// a product [points x d] [d x d] with the antisymmetric part of G_2.  A workgroup stages G_2 of its path in LDS, serves
// the two end points with vector arithmetic from it (they keep the G_1 term and both products), replaces it by
// G_2 - G_2^T in place and then multiplies: tiles of 16 points x 16 channels, four channels of the sum per
// v_mfma_f32_16x16x4_f32, the rows v_k formed from the path a round of points at a time.
#include "sig_internal.h"

namespace sig {
namespace {

typedef float b2m_f4 __attribute__((ext_vector_type(4)));

struct B2mPlan {
    int tiles;             // T = ceil(d / 16)
    int dk;                // d rounded up to a multiple of 4: rows of the staged matrix, length of a staged row v_k
    int ldg;               // floats per staged row of the matrix: 16 T + 1
    int lda;               // floats per staged v_k: dk + 1
    int round_points;      // interior points per round: 64, 32 or 16
    int rounds;            // rounds per workgroup
    int64_t groups_per_path;
};

__global__ void __launch_bounds__(256)
sig_backward_n2_mfma_kernel(Shape sh, B2mPlan pl, const float *__restrict__ path, const float *__restrict__ gout,
                            float *__restrict__ gpath, float *__restrict__ gbase)
{
    extern __shared__ __align__(16) unsigned char b2m_smem[];
    const int d = sh.d, ldg = pl.ldg, lda = pl.lda, dk = pl.dk, cols = 16 * pl.tiles;
    float *Gs = reinterpret_cast<float *>(b2m_smem);   // [dk][ldg]: G_2, later G_2 - G_2^T; zeros beyond d x d
    float *As = Gs + dk * ldg;                         // [round_points][lda]: the rows v_k of a round
    float *ends = As + pl.round_points * lda;          // [4][d]: m_0 - p, q - m_0, m_e - p, q - m_e

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t b = blockIdx.x / pl.groups_per_path, group = blockIdx.x % pl.groups_per_path;
    const float *x = path + b * sh.L * d;
    const float *go = gout + b * sh.S;
    const float *bpv = static_cast<const float *>(sh.basepoint_value);
    const int shift = sh.basepoint ? 1 : 0;   // with a basepoint the scan's points are bp, x_0, x_1, ..
    const int64_t n = sh.n_inc;               // the scan's points are X_0 .. X_n

    // channel c of point k of the scan; the load is unconditional
    const auto scan_point = [&](int64_t k, int c) -> float {
        const bool from_base = sh.basepoint && k == 0;
        const float *src = from_base ? (bpv != nullptr ? bpv + b * d + c : x) : x + (k - shift) * d + c;
        const float v = *src;
        return from_base && bpv == nullptr ? 0.f : v;
    };

    // G_2 into LDS, zeros around it
#pragma unroll 4
    for (int e = tid; e < dk * cols; e += 256) {
        const int i = e / cols, j = e - i * cols;
        const bool on = i < d && j < d;
        const float v = go[d + (on ? i * d + j : 0)];
        Gs[i * ldg + j] = on ? v : 0.f;
    }
    if (group == 0) {
        for (int e = tid; e < 2 * d; e += 256) {
            const int which = e / d, c = e - which * d;   // 0: the first increment, 1: the last
            const int64_t s = which == 0 ? 0 : n - 1;
            // differences of points only, so that a path far from the origin loses nothing
            const float xs = scan_point(s, c), xt = scan_point(s + 1, c), half = (xt - xs) * 0.5f;
            ends[(2 * which) * d + c] = (xs - scan_point(0, c)) + half;
            ends[(2 * which + 1) * d + c] = (scan_point(n, c) - xt) + half;
        }
    }
    __syncthreads();
    if (group == 0) {
        // the scan's first point starts increment 0 and ends none; its last point ends increment n - 1
        const int which = tid >> 7, j = tid & 127;
        if (j < d) {
            const float *a = ends + (2 * which) * d, *bb = a + d;
            float acc = go[j];
            for (int i = 0; i < d; ++i) acc += a[i] * Gs[i * ldg + j] + bb[i] * Gs[j * ldg + i];
            if (which == 0) {
                if (sh.basepoint) {
                    if (gbase != nullptr) gbase[b * d + j] = -acc;
                } else {
                    gpath[b * sh.L * d + j] = -acc;
                }
            } else {
                gpath[(b * sh.L + sh.L - 1) * d + j] = acc;
            }
        }
        __syncthreads();
    }
    // G_2 - G_2^T in place: the thread of (i, j), i < j, rewrites both entries
    for (int e = tid; e < d * d; e += 256) {
        const int i = e / d, j = e - i * d;
        if (i < j) {
            const float u = Gs[i * ldg + j], l = Gs[j * ldg + i];
            Gs[i * ldg + j] = u - l;
            Gs[j * ldg + i] = l - u;
        } else if (i == j) {
            Gs[i * ldg + j] = 0.f;
        }
    }

    // interior points X_k, k = 1 .. n - 1, a round at a time
    const int64_t k_group = 1 + group * int64_t(pl.round_points) * pl.rounds;
    const int k4 = lane >> 4, c16 = lane & 15;
    const int blocks = pl.round_points / 16, items = blocks * pl.tiles;   // 16 x 16 tiles of a round's result
    for (int round = 0; round < pl.rounds; ++round) {
        const int64_t k0 = k_group + int64_t(round) * pl.round_points;
        if (k0 > n - 1) break;   // the same for every thread
        __syncthreads();   // the matrix is ready; the round before has been multiplied
        for (int e = tid; e < pl.round_points * dk; e += 256) {
            const int pt = e / dk, i = e - pt * dk;
            const int64_t k = k0 + pt;
            const bool on = k <= n - 1 && i < d;
            const int64_t kk = on ? k : 1;
            const int ii = on ? i : 0;
            const float before = scan_point(kk - 1, ii), after = scan_point(kk + 1 <= n ? kk + 1 : n, ii);
            As[pt * lda + i] = on ? (before - after) * 0.5f : 0.f;
        }
        __syncthreads();
        for (int item = wave; item < items; item += 4) {
            const int blk = item / pl.tiles, t = item - blk * pl.tiles;
            if (k0 + 16 * blk > n - 1) continue;   // a block of points past the end
            const float *ap = As + (16 * blk + c16) * lda + k4, *bp = Gs + k4 * ldg + 16 * t + c16;
            b2m_f4 acc = b2m_f4(0.f);
#pragma unroll 4
            for (int kq = 0; kq < dk; kq += 4) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(ap[kq], bp[kq * ldg], acc, 0, 0, 0);
            // register r of lane (k4, c16): point 16 blk + 4 k4 + r of the round, channel 16 t + c16
            const int j = 16 * t + c16;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int64_t k = k0 + 16 * blk + 4 * k4 + r;
                if (k <= n - 1 && j < d) gpath[(b * sh.L + k - shift) * d + j] = acc[r];
            }
        }
    }
}

size_t b2m_lds(const B2mPlan &pl, int d)
{
    return sizeof(float) * (size_t(pl.dk) * pl.ldg + size_t(pl.round_points) * pl.lda + 4 * size_t(d));
}

bool b2m_plan(const Shape &sh, B2mPlan &pl)
{
    if (sh.N != 2 || sh.stream || sh.chunks > 1 || sh.d < 8 || sh.d > 112 || sh.n_inc < 1) return false;
    pl.tiles = (sh.d + 15) / 16;
    pl.dk = (sh.d + 3) / 4 * 4;
    pl.ldg = 16 * pl.tiles + 1;
    pl.lda = pl.dk + 1;
    pl.round_points = 64;
    while (pl.round_points > 16 && b2m_lds(pl, sh.d) > 64 * 1024) pl.round_points /= 2;
    if (b2m_lds(pl, sh.d) > 64 * 1024) return false;
    // a workgroup stages the matrix once and serves up to 8 rounds, fewer while that leaves under 1024 workgroups
    const int64_t interior = sh.n_inc - 1;
    pl.rounds = 8;
    const auto groups = [&]() { return interior <= 0 ? int64_t(1) : (interior + int64_t(pl.round_points) * pl.rounds - 1) / (int64_t(pl.round_points) * pl.rounds); };
    while (pl.rounds > 1 && sh.B * groups() < 1024) pl.rounds /= 2;
    pl.groups_per_path = groups();
    return sh.B * pl.groups_per_path <= 0x7fffffff;
}

}  // namespace

bool backward_n2_mfma_supported(const Shape &sh)
{
    B2mPlan pl;
    return b2m_plan(sh, pl);
}

hipError_t launch_backward_n2_mfma_f32(const Shape &sh, const float *path, const float *gout, float *gpath, float *gbase,
                                       hipStream_t st)
{
    B2mPlan pl;
    if (!b2m_plan(sh, pl)) return hipErrorNotSupported;
    hipLaunchKernelGGL(sig_backward_n2_mfma_kernel, dim3(unsigned(sh.B * pl.groups_per_path)), dim3(256), b2m_lds(pl, sh.d), st, sh, pl,
                       path, gout, gpath, gbase);
    return hipGetLastError();
}

}  // namespace sig
