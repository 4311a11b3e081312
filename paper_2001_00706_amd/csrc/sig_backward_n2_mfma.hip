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
// v_mfma_f32_16x16x4_f32.  The path is staged a round of points at a time as it lies in memory (every point read once);
// a lane forms its scalar of v_k from the two neighbours' rows as it feeds the matrix instruction.  The next round's
// points are fetched into registers before the current round is multiplied, and the barriers order LDS traffic only,
// so loads and stores stay in flight across rounds.
#include "sig_internal.h"
#include "sig_lane_ops.h"

namespace sig {
namespace {

typedef float b2m_f4 __attribute__((ext_vector_type(4)));
// loads of a round's points a thread has in flight: 6 of 16 bytes where rows allow them, else 8 of 4 bytes
constexpr int b2m_slots(int V) { return V == 4 ? 6 : 8; }

struct B2mPlan {
    int tiles;             // T = ceil(d / 16)
    int dk;                // d rounded up to a multiple of 4: rows of the staged matrix, length of a staged row v_k
    int ldg;               // floats per staged row of the matrix: 16 T + 1
    int lda;               // floats per staged point: dk or dk + 4
    int round_points;      // interior points per round: 64, 32 or 16
    int rounds;            // rounds per workgroup
    int64_t groups_per_path;
    int V;                 // scalars per load of the path: 4 (d a multiple of four, 16-byte aligned rows) or 1
};

template <int V>
__global__ void __launch_bounds__(256)
sig_backward_n2_mfma_kernel(Shape sh, B2mPlan pl, const float *__restrict__ path, const float *__restrict__ gout,
                            float *__restrict__ gpath, float *__restrict__ gbase)
{
    extern __shared__ __align__(16) unsigned char b2m_smem[];
    const int d = sh.d, ldg = pl.ldg, lda = pl.lda, dk = pl.dk, cols = 16 * pl.tiles;
    float *Gs = reinterpret_cast<float *>(b2m_smem);   // [dk][ldg]: G_2, later G_2 - G_2^T; zeros beyond d x d
    float *Xs = Gs + dk * ldg;                         // [round_points + 2][lda]: the points k0 - 1 .. k0 + round_points
    float *ends = Xs + (pl.round_points + 2) * lda;    // [4][d]: m_0 - p, q - m_0, m_e - p, q - m_e

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
    constexpr int kSlots = b2m_slots(V);
    typedef float b2m_load __attribute__((ext_vector_type(V)));
    const int per_row = dk / V, entries = (pl.round_points + 2) * per_row;   // loads per point, per round
    b2m_load ahead[kSlots];
    // the points k0 - 1 .. k0 + round_points of the scan (clamped at its end) into registers: loads only, every one
    // unconditional on a clamped index, so they are all in flight together
    const auto fetch = [&](int64_t k0) {
#pragma unroll
        for (int u = 0; u < kSlots; ++u) {
            if (256 * u < entries) {   // the same for every thread
                const int e = tid + 256 * u < entries ? tid + 256 * u : 0;
                const int pt = e / per_row, i = (e - pt * per_row) * V;
                int64_t k = k0 - 1 + pt;
                k = k <= n ? k : n;
                const bool from_base = sh.basepoint && k == 0;
                const float *src = from_base ? (bpv != nullptr ? bpv + b * d : x) : x + (k - shift) * d;
                const b2m_load v = *reinterpret_cast<const b2m_load *>(src + (i < d ? i : 0));
                ahead[u] = from_base && bpv == nullptr ? b2m_load(0.f) : v;
            }
        }
    };
    if (k_group <= n - 1) fetch(k_group);
    for (int round = 0; round < pl.rounds; ++round) {
        const int64_t k0 = k_group + int64_t(round) * pl.round_points;
        if (k0 > n - 1) break;   // the same for every thread
#pragma unroll
        for (int u = 0; u < kSlots; ++u) {
            if (256 * u < entries && tid + 256 * u < entries) {
                const int e = tid + 256 * u;
                const int pt = e / per_row, i = (e - pt * per_row) * V;
                if constexpr (V == 4) {   // d is a multiple of four here: no columns beyond it
                    *reinterpret_cast<b2m_load *>(Xs + pt * lda + i) = ahead[u];   // rows are a multiple of 16 bytes
                } else {
                    Xs[pt * lda + i] = i < d ? ahead[u][0] : 0.f;
                }
            }
        }
        lds_barrier();   // the points are staged (and, before the first round, the matrix is ready)
        if (round + 1 < pl.rounds && k0 + pl.round_points <= n - 1) fetch(k0 + pl.round_points);
        for (int item = wave; item < items; item += 4) {
            const int blk = item / pl.tiles, t = item - blk * pl.tiles;
            if (k0 + 16 * blk > n - 1) continue;   // a block of points past the end
            // point 16 blk + c16 of the round is X_k with its neighbours in rows 16 blk + c16 and 16 blk + c16 + 2
            const float *xp = Xs + (16 * blk + c16) * lda + k4, *bp = Gs + k4 * ldg + 16 * t + c16;
            b2m_f4 acc = b2m_f4(0.f);
#pragma unroll 4
            for (int kq = 0; kq < dk; kq += 4)
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32((xp[kq] - xp[2 * lda + kq]) * 0.5f, bp[kq * ldg], acc, 0, 0, 0);
            // register r of lane (k4, c16): point 16 blk + 4 k4 + r of the round, channel 16 t + c16
            const int j = 16 * t + c16;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int64_t k = k0 + 16 * blk + 4 * k4 + r;
                if (k <= n - 1 && j < d) gpath[(b * sh.L + k - shift) * d + j] = acc[r];
            }
        }
        lds_barrier();   // the round has been multiplied: its points may be overwritten
    }
}

size_t b2m_lds(const B2mPlan &pl, int d)
{
    return sizeof(float) * (size_t(pl.dk) * pl.ldg + size_t(pl.round_points + 2) * pl.lda + 4 * size_t(d));
}

bool b2m_plan(const Shape &sh, bool vector_loads, B2mPlan &pl)
{
    if (sh.N != 2 || sh.stream || sh.chunks > 1 || !sh.from_identity || sh.d < 8 || sh.d > 112 || sh.n_inc < 1) return false;
    pl.tiles = (sh.d + 15) / 16;
    pl.dk = (sh.d + 3) / 4 * 4;
    pl.ldg = 16 * pl.tiles + 1;
    // an odd multiple of four scalars: the 64 lanes' reads of a matrix instruction's left operand (16 rows, 4 consecutive
    // columns) then fall on every LDS bank exactly twice
    pl.lda = (pl.dk / 4) % 2 == 1 ? pl.dk : pl.dk + 4;
    pl.round_points = 64;
    pl.V = vector_loads && sh.d % 4 == 0 ? 4 : 1;
    const auto fits = [&]() { return b2m_lds(pl, sh.d) <= 64 * 1024 && (pl.round_points + 2) * (pl.dk / pl.V) <= b2m_slots(pl.V) * 256; };
    while (pl.round_points > 16 && !fits()) pl.round_points /= 2;
    if (!fits()) return false;
    // a workgroup stages the matrix once and serves up to 16 rounds, fewer while that leaves under 1024 workgroups
    const int64_t interior = sh.n_inc - 1;
    pl.rounds = 16;
    const auto groups = [&]() { return interior <= 0 ? int64_t(1) : (interior + int64_t(pl.round_points) * pl.rounds - 1) / (int64_t(pl.round_points) * pl.rounds); };
    while (pl.rounds > 1 && sh.B * groups() < 1024) pl.rounds /= 2;
    pl.groups_per_path = groups();
    return sh.B * pl.groups_per_path <= 0x7fffffff;
}

}  // namespace

bool backward_n2_mfma_supported(const Shape &sh)
{
    B2mPlan pl;
    return b2m_plan(sh, false, pl);
}

hipError_t launch_backward_n2_mfma_f32(const Shape &sh, const float *path, const float *gout, float *gpath, float *gbase,
                                       hipStream_t st)
{
    B2mPlan pl;
    const bool aligned = (reinterpret_cast<uintptr_t>(path) | reinterpret_cast<uintptr_t>(sh.basepoint_value)) % 16 == 0;
    if (!b2m_plan(sh, aligned, pl)) return hipErrorNotSupported;
    const dim3 grid(unsigned(sh.B * pl.groups_per_path));
    if (pl.V == 4)
        hipLaunchKernelGGL(sig_backward_n2_mfma_kernel<4>, grid, dim3(256), b2m_lds(pl, sh.d), st, sh, pl, path, gout, gpath, gbase);
    else
        hipLaunchKernelGGL(sig_backward_n2_mfma_kernel<1>, grid, dim3(256), b2m_lds(pl, sh.d), st, sh, pl, path, gout, gpath, gbase);
    return hipGetLastError();
}

}  // namespace sig
