// Depth-2 signature in final mode without a scan (any channel count, fp32 and fp64).
//
// With increments z_s = b_s - a_s (a_s, b_s the points increment s runs between), p the point the scan starts from and
// q the point it ends at, Chen's identity applied increment by increment (paper sections 2.1, 2.2, eq. "iterative")
// sums up to
//     A_1 = q - p,     A_2 = sum_s (a_s - p + z_s / 2) (x) z_s = sum_s (m_s - p) (x) z_s,
// m_s = (a_s + b_s) / 2 the midpoint of increment s: the left factor of term s is the level-1 signature before the
// increment plus half the increment, which is what the fused multiply-exponentiate (section 4.1) adds at depth 2.
// Level 2 is therefore a contraction over the increments, [d x n_inc] [n_inc x d], with no dependence between them:
// a thread per 4 x 4 block of output coefficients.  A tile of consecutive points of the path is copied to LDS as it
// lies in memory (16 bytes per load where the rows allow it, every point read once, rows padded with zeros to a
// multiple of four channels); per increment a thread reads the two 4-channel pieces of the new point that its block
// needs (the old point's stay in registers), forms its pieces of 2 (m_s - p) = (a_s - p) + (b_s - p) and of z_s (differences of
// points only: where the path lies does not matter) and does 16 multiply-adds; the sums are halved at the end.
// Paths with fewer than 256 blocks share a workgroup once there are enough workgroups; threads left over split a
// tile's increments between them and add their partial sums up through LDS at the end.
// The sum may also be split over the length of a path (a chunked scan: a row is then a stretch of a path, its terms
// still taken against the first point of the whole path; a second kernel adds the stretches).
#include "sig_internal.h"
#include "sig_lane_ops.h"

namespace sig {
namespace {

constexpr int kBatch = 4;   // staging loads a thread has in flight: a tile is at most 256 * kBatch loads

struct N2Plan {
    int dq;                   // ceil(d / 4): blocks per row of level 2
    int paths_per_group;      // paths sharing a workgroup (1 when a path has 256 blocks or more)
    int64_t groups_per_path;  // workgroups per path (1 when paths share a workgroup)
    int tile;                 // increments per staged tile (tile + 1 points)
    int splits;               // threads per block of coefficients, each with its share of a tile's increments
    int vec;                  // scalars per staging load: 16 or 8 bytes' worth, or 1
};

template <typename T, int V>
__global__ void __launch_bounds__(256)
sig_forward_n2_kernel(Shape sh, N2Plan pl, const T *__restrict__ path, T *__restrict__ out)
{
    typedef T T4 __attribute__((ext_vector_type(4)));
    typedef T TV __attribute__((ext_vector_type(V)));
    extern __shared__ __align__(32) unsigned char fn2_smem[];
    const int d = sh.d, dpad = 4 * pl.dq, blocks = pl.dq * pl.dq;
    const int rows = pl.tile + 1;
    T *pts = reinterpret_cast<T *>(fn2_smem);          // [paths_per_group][tile + 1][dpad]: points of the scan
    T *start = pts + pl.paths_per_group * rows * dpad;  // [paths_per_group][dpad]: p

    const int tid = threadIdx.x;
    const bool shared_group = blocks < 256;
    const int per_split = blocks * pl.paths_per_group;   // threads of one split (shared workgroups only)
    const int ks = shared_group ? tid / per_split : 0;
    const int in_split = shared_group ? tid - ks * per_split : tid;
    const int slot = shared_group ? in_split / blocks : 0;
    const int64_t w = shared_group ? in_split - slot * blocks : int64_t(blockIdx.x % pl.groups_per_path) * 256 + tid;   // the block
    const int64_t row0 = shared_group ? int64_t(blockIdx.x) * pl.paths_per_group : int64_t(blockIdx.x / pl.groups_per_path);
    const int64_t row = row0 + slot;
    const bool works = w < blocks && ks < pl.splits && row < sh.B;
    const bool live = works && ks == 0;   // writes the block
    const int ib = int((works ? w : 0) / pl.dq), jb = int((works ? w : 0) - int64_t(ib) * pl.dq);
    const T *bpv = static_cast<const T *>(sh.basepoint_value);
    const int shift = sh.basepoint ? 1 : 0;   // with a basepoint the scan's points are bp, x_0, x_1, ..

    // V channels from c on of point number k of the scan of path r (c a multiple of V; V > 1 only where d is one too)
    auto scan_point = [&](int64_t r, int64_t k, int c) -> TV {
        const bool from_base = sh.basepoint && k == 0;
        const T *src = from_base ? (bpv != nullptr ? bpv + r * d + c : path) : path + (r * sh.L + k - shift) * d + c;
        TV v = *reinterpret_cast<const TV *>(src);
        if (from_base && bpv == nullptr) v = TV(0);
        return v;
    };

    const int cvecs = dpad / V;   // loads per staged row
    for (int e = tid; e < pl.paths_per_group * cvecs; e += 256) {
        const int p = e / cvecs, c = (e - p * cvecs) * V;
        const bool on = row0 + p < sh.B && c < d;
        const TV v = scan_point(on ? chunk_view(row0 + p, sh.chunks, sh.chunk_len, sh.n_inc).path : 0, 0, on ? c : 0);
        *reinterpret_cast<TV *>(start + p * dpad + c) = on ? v : TV(0);
    }

    T acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = T(0);
    T4 p_i = T4(0);
    const int staged = pl.paths_per_group * rows * cvecs;   // at most 256 * kBatch: a tile is one batch of loads
    // Every load is unconditional, on indices clamped into a path, so that the loads of a tile are in flight together;
    // rows past the end of the batch, points past the end of the path and the padding behind the last channel become
    // zeros when the tile is written to LDS.  The loads of the next tile are issued before this tile's arithmetic.
    // Which point of which path an entry of the tile holds does not change from tile to tile: worked out once.
    TV held[kBatch];
    const T *entry_row[kBatch];   // channel c of the first point of the entry's row (of path 0 for entries that stay zero)
    int entry_point[kBatch];      // the entry's point inside the tile
    int64_t entry_n[kBatch];      // increments of the entry's row; -1 for entries that stay zero
    bool entry_first[kBatch];     // the row starts at the scan's first point
    const T *entry_base[kBatch];  // the entry's channels of a basepoint given by value
#pragma unroll
    for (int k = 0; k < kBatch; ++k) {
        const int e = 256 * k + tid < staged ? 256 * k + tid : staged - 1;
        const int p = e / (rows * cvecs), rem = e - p * rows * cvecs, pt = rem / cvecs, c = (rem - pt * cvecs) * V;
        const ChunkView cv = chunk_view(row0 + p < sh.B ? row0 + p : 0, sh.chunks, sh.chunk_len, sh.n_inc);
        const bool on = row0 + p < sh.B && c < d && cv.n > 0;
        entry_point[k] = pt;
        entry_n[k] = on ? cv.n : -1;
        entry_first[k] = cv.inc0 == 0;
        entry_row[k] = path + (on ? (cv.path * sh.L + cv.inc0) * d + c : 0);
        entry_base[k] = bpv != nullptr && on ? bpv + cv.path * d + c : bpv;
    }
    const auto load_tile = [&](int64_t t0) {
#pragma unroll
        for (int k = 0; k < kBatch; ++k) {
            if (256 * k >= staged) break;   // the same for every thread
            const int64_t point = t0 + entry_point[k];
            const bool on = point <= entry_n[k];
            const bool from_base = on && sh.basepoint && entry_first[k] && point == 0;
            const T *src = from_base && bpv != nullptr ? entry_base[k] : entry_row[k] + (on && !from_base ? point - shift : 0) * d;
            held[k] = *reinterpret_cast<const TV *>(src);
        }
    };
    // a row is a whole path, or a stretch of chunk_len increments of one (the last stretches of a path may be shorter or empty)
    const ChunkView mine = chunk_view(row < sh.B ? row : 0, sh.chunks, sh.chunk_len, sh.n_inc);
    const int64_t n_longest = sh.chunks > 1 ? sh.chunk_len : sh.n_inc;
    load_tile(0);
    for (int64_t t0 = 0; t0 < n_longest; t0 += pl.tile) {
        lds_barrier();   // not __syncthreads(): the loads of the next tile stay in flight
#pragma unroll
        for (int k = 0; k < kBatch; ++k) {
            if (256 * k >= staged) break;
            const int64_t point = t0 + entry_point[k];
            const bool zero = point > entry_n[k] || (sh.basepoint && entry_first[k] && point == 0 && bpv == nullptr);
            if (256 * k + tid < staged) *reinterpret_cast<TV *>(pts + int64_t(256 * k + tid) * V) = zero ? TV(0) : held[k];
        }
        if (t0 + pl.tile < n_longest) load_tile(t0 + pl.tile);
        lds_barrier();
        if (t0 == 0) p_i = *reinterpret_cast<const T4 *>(start + slot * dpad + 4 * ib);
        const T *lp = pts + slot * rows * dpad + 4 * ib, *rp = pts + slot * rows * dpad + 4 * jb;
        const int64_t left = mine.n - t0;
        const int nt = int(left < 0 ? 0 : left < pl.tile ? left : pl.tile);
        const int share = (nt + pl.splits - 1) / pl.splits;
        const int lo = works ? ks * share : nt, hi = lo + share < nt ? lo + share : nt;   // this thread's increments
        if (lo < hi) {
            // Only differences of points enter (a path far from the origin loses nothing): twice the left factor is
            // (a - p) + (b - p), each term rounded relative to its own size; the sums are halved at the end.
            T4 ya_i = *reinterpret_cast<const T4 *>(lp + lo * dpad) - p_i, a_j = *reinterpret_cast<const T4 *>(rp + lo * dpad);
#pragma unroll 4
            for (int s = lo + 1; s <= hi; ++s) {
                const T4 yb_i = *reinterpret_cast<const T4 *>(lp + s * dpad) - p_i, b_j = *reinterpret_cast<const T4 *>(rp + s * dpad);
                const T4 l = ya_i + yb_i, r = b_j - a_j;
#pragma unroll
                for (int a = 0; a < 4; ++a)
#pragma unroll
                    for (int b = 0; b < 4; ++b) acc[a][b] += l[a] * r[b];
                ya_i = yb_i;
                a_j = b_j;
            }
        }
        // the last tile ends at the scan's last point: level 1, by the threads of the first row of blocks
        if (live && ib == 0 && sh.chunks <= 1 && t0 + pl.tile >= sh.n_inc) {
            const T4 q_j = *reinterpret_cast<const T4 *>(rp + nt * dpad), p_j = *reinterpret_cast<const T4 *>(start + slot * dpad + 4 * jb);
#pragma unroll
            for (int b = 0; b < 4; ++b)
                if (4 * jb + b < d) out[row * sh.S + 4 * jb + b] = q_j[b] - p_j[b];
        }
    }
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] *= T(0.5);
    if (pl.splits > 1) {
        // partial sums of the splits, coefficient-major so that a wavefront's accesses spread over the banks
        __syncthreads();
        T *red = reinterpret_cast<T *>(fn2_smem);   // [16][256]
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b) red[(a * 4 + b) * 256 + tid] = acc[a][b];
        __syncthreads();
        if (live) {
            for (int k = 1; k < pl.splits; ++k)
#pragma unroll
                for (int a = 0; a < 4; ++a)
#pragma unroll
                    for (int b = 0; b < 4; ++b) acc[a][b] += red[(a * 4 + b) * 256 + tid + k * per_split];
        }
    }
    if (live) {
        T *o = out + row * sh.S;
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b)
                if (4 * ib + a < d && 4 * jb + b < d) o[d + (4 * ib + a) * d + 4 * jb + b] = acc[a][b];
    }
}

size_t n2_lds(const N2Plan &pl, size_t elem)
{
    const size_t points = elem * size_t(pl.paths_per_group) * size_t(4 * pl.dq) * size_t(pl.tile + 2);
    const size_t sums = pl.splits > 1 ? elem * 16 * 256 : 0;
    return points > sums ? points : sums;
}

// Adds up the rows of the stretches of a path (level 2: the terms of the sum over increments in any grouping) and forms
// level 1 from the scan's end points: out[b] = (q - p, sum_c partial[b][c]).  A workgroup serves 16 scalars of a path:
// thread (part, w) adds the stretches part, part + 16, .., the 16 parts meet in LDS and are added in order.
template <typename T>
__global__ void __launch_bounds__(256)
sig_forward_n2_sum_kernel(Shape sh, const T *__restrict__ path, const T *__restrict__ partial, T *__restrict__ out)
{
    __shared__ T parts[16][17];
    const int d = sh.d;
    const int64_t groups_per_path = (sh.S + 15) / 16;
    const int64_t b = blockIdx.x / groups_per_path;
    const int part = threadIdx.x >> 4, lane16 = threadIdx.x & 15;
    const int64_t w = (blockIdx.x % groups_per_path) * 16 + lane16;
    T acc = T(0);
    if (w >= d && w < sh.S) {
        const T *q = partial + b * sh.chunks * sh.S + w;
        for (int c = part; c < sh.chunks; c += 16) acc += q[int64_t(c) * sh.S];
    }
    parts[part][lane16] = acc;
    __syncthreads();
    if (part == 0 && w < sh.S) {
        if (w < d) {
            const T *x = path + b * sh.L * d;
            const T *bpv = static_cast<const T *>(sh.basepoint_value);
            const T first = sh.basepoint ? (bpv != nullptr ? bpv[b * d + w] : T(0)) : x[w];
            out[b * sh.S + w] = x[(sh.L - 1) * d + w] - first;
        } else {
            T total = parts[0][lane16];
#pragma unroll
            for (int k = 1; k < 16; ++k) total += parts[k][lane16];
            out[b * sh.S + w] = total;
        }
    }
}

// `stretches`: rows may be stretches of a path (Shape::chunks > 1), their level-2 sums going to a workspace
bool n2_plan(const Shape &sh, size_t elem, const void *path, N2Plan &pl, bool stretches = false)
{
    if (sh.N != 2 || sh.stream || (sh.chunks > 1 && !stretches) || sh.d < 1 || sh.d > 1024) return false;
    pl.dq = (sh.d + 3) / 4;
    const int64_t blocks = int64_t(pl.dq) * pl.dq;
    if (blocks >= 256) {
        pl.paths_per_group = 1;
        pl.groups_per_path = (blocks + 255) / 256;
        pl.splits = 1;
    } else {
        // The work of a path is small and a workgroup's time is a chain of trips to memory, one per batch of staged
        // scalars: paths share a workgroup only once there are enough workgroups to fill the chip several times.
        const int fit = int(256 / blocks);
        int share = fit < 64 ? fit : 64;
        while (share > 1 && (sh.B + share - 1) / share < 1024) share /= 2;
        pl.paths_per_group = share;
        pl.groups_per_path = 1;
        const int spare = int(256 / (blocks * share));
        pl.splits = spare < 16 ? spare : 16;
    }
    // a tile of points within 32 KB
    int64_t tile = int64_t(32 * 1024) / (int64_t(elem) * pl.paths_per_group * 4 * pl.dq) - 1;
    pl.tile = int(tile < 1 ? 1 : tile > 128 ? 128 : tile);
    // 16-byte (else 8-byte) loads where every row of d scalars, and so every point, starts on such a boundary
    pl.vec = 1;
    for (int v = int(16 / elem); v > 1; v /= 2) {
        const auto aligned = [&](const void *q) { return reinterpret_cast<uintptr_t>(q) % (v * elem) == 0; };
        if (sh.d % v == 0 && aligned(path) && aligned(sh.basepoint_value)) {
            pl.vec = v;
            break;
        }
    }
    // ... and within one batch of loads: (tile + 1) points of dpad / vec loads each for every path of the workgroup
    const int64_t loads_per_point = int64_t(pl.paths_per_group) * (4 * pl.dq / pl.vec);
    if (2 * loads_per_point > 256 * kBatch) return false;
    if ((pl.tile + 1) * loads_per_point > 256 * kBatch) pl.tile = int(256 * kBatch / loads_per_point) - 1;
    const int64_t groups = blocks >= 256 ? sh.B * pl.groups_per_path : (sh.B + pl.paths_per_group - 1) / pl.paths_per_group;
    return groups <= 0x7fffffff && n2_lds(pl, elem) <= 64 * 1024;
}

template <typename T>
hipError_t launch_forward_n2_t(const Shape &sh, const T *path, T *out, hipStream_t st, bool stretches = false)
{
    N2Plan pl;
    if (!n2_plan(sh, sizeof(T), path, pl, stretches)) return hipErrorNotSupported;
    const int64_t blocks = int64_t(pl.dq) * pl.dq;
    const int64_t groups = blocks >= 256 ? sh.B * pl.groups_per_path : (sh.B + pl.paths_per_group - 1) / pl.paths_per_group;
    const dim3 grid{unsigned(groups)}, block{256};
    const size_t lds = n2_lds(pl, sizeof(T));
    switch (pl.vec * int(sizeof(T))) {
        case 16: hipLaunchKernelGGL((sig_forward_n2_kernel<T, 16 / int(sizeof(T))>), grid, block, lds, st, sh, pl, path, out); break;
        case 8: hipLaunchKernelGGL((sig_forward_n2_kernel<T, 8 / int(sizeof(T))>), grid, block, lds, st, sh, pl, path, out); break;
        default: hipLaunchKernelGGL((sig_forward_n2_kernel<T, 1>), grid, block, lds, st, sh, pl, path, out); break;
    }
    return hipGetLastError();
}

}  // namespace

bool forward_n2_supported(const Shape &sh, sig_dtype dtype)
{
    N2Plan pl;
    return n2_plan(sh, dtype == SIG_F32 ? sizeof(float) : sizeof(double), nullptr, pl);
}

template <typename T>
hipError_t launch_forward_n2_chunked_t(const Shape &sh, const T *path, T *partial, T *out, hipStream_t st)
{
    const hipError_t err = launch_forward_n2_t<T>(sh, path, partial, st, true);
    if (err != hipSuccess) return err;
    const int64_t groups = sh.B / sh.chunks * ((sh.S + 15) / 16);
    if (groups > 0x7fffffff) return hipErrorNotSupported;
    hipLaunchKernelGGL((sig_forward_n2_sum_kernel<T>), dim3(unsigned(groups)), dim3(256), 0, st, sh, path, partial, out);
    return hipGetLastError();
}

bool forward_n2_chunked_supported(const Shape &sh, sig_dtype dtype)
{
    N2Plan pl;
    return sh.chunks > 1 && n2_plan(sh, dtype == SIG_F32 ? sizeof(float) : sizeof(double), nullptr, pl, true);
}

hipError_t launch_forward_n2_chunked_f32(const Shape &sh, const float *path, float *partial, float *out, hipStream_t st)
{
    return launch_forward_n2_chunked_t<float>(sh, path, partial, out, st);
}

hipError_t launch_forward_n2_chunked_f64(const Shape &sh, const double *path, double *partial, double *out, hipStream_t st)
{
    return launch_forward_n2_chunked_t<double>(sh, path, partial, out, st);
}

hipError_t launch_forward_n2_f32(const Shape &sh, const float *path, float *out, hipStream_t st)
{
    return launch_forward_n2_t<float>(sh, path, out, st);
}

hipError_t launch_forward_n2_f64(const Shape &sh, const double *path, double *out, hipStream_t st)
{
    return launch_forward_n2_t<double>(sh, path, out, st);
}

}  // namespace sig
