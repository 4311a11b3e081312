// Depth-2 signature in final mode on the matrix cores (fp32, 17 to 256 channels, many paths).
//
// As in sig_forward_n2.hip, level 2 is the contraction over the increments
//     A_2 = sum_s (m_s - p) (x) z_s,      A_1 = q - p
// (m_s the midpoint of increment s, z_s the increment, p and q the scan's first and last point; paper sections 2.1,
// 2.2): a product [d x n_inc] [n_inc x d] per path.  Here a wavefront owns a strip of up to four 16 x 16 tiles of
// A_2 and advances four increments per v_mfma_f32_16x16x4_f32: lane (k, c), k = lane / 16, c = lane % 16, forms the
// operand scalars 2 (m - p)[16 ti + c] = (a - p) + (b - p) and z[16 tj + c] of increment s + k from two consecutive points of
// the staged tile (differences of points only; the sums are halved at the end).  A point is kept in LDS with the channels c, 16 + c, 32 + c, 48 + c of a strip side by side, so that one
// 16-byte read fetches a lane's scalars for all four tiles of its strip (an LDS read instruction costs about 6 clocks
// of the compute unit's LDS port whatever its width; with one 4-byte read per scalar the port, not the matrix cores,
// bounded the kernel).  The tile of points is staged as in the vector kernel: the next tile's loads are issued before
// this tile's arithmetic.
#include "sig_internal.h"
#include "sig_lane_ops.h"

#include <type_traits>

namespace sig {
namespace {

typedef float n2m_f4 __attribute__((ext_vector_type(4)));

constexpr int kN2mBatch = 4;   // staging loads a thread has in flight: a tile is at most 256 * kN2mBatch loads

struct N2mPlan {
    int tiles;            // T = ceil(d / 16): tiles per side of level 2
    int strips;           // strips of four tiles per row of tiles: ceil(T / 4)
    int stride;           // floats per staged point: 64 per strip
    int items;            // strips per path: T * strips, one wavefront each
    int paths_per_group;  // paths sharing a workgroup of four wavefronts
    int groups_per_path;  // workgroups per path
    int tile;             // increments per staged tile (a multiple of 4; tile + 1 points)
    int vec;              // scalars per staging load: 4, 2 or 1
};

// where channel c of a point lies inside its staged row: [strip][c % 16][tile inside the strip]
__device__ __forceinline__ int n2m_pos(int c) { return (c >> 6) * 64 + (c & 15) * 4 + ((c >> 4) & 3); }

template <int V>
__global__ void __launch_bounds__(256)
sig_forward_n2_mfma_kernel(Shape sh, N2mPlan pl, const float *__restrict__ path, float *__restrict__ out)
{
    typedef float TV __attribute__((ext_vector_type(V)));
    extern __shared__ __align__(16) unsigned char n2m_smem[];
    const int d = sh.d, stride = pl.stride;
    const int rows = pl.tile + 1;
    float *pts = reinterpret_cast<float *>(n2m_smem);        // [paths_per_group][tile + 1][stride]: points of the scan
    float *start = pts + pl.paths_per_group * rows * stride;   // [paths_per_group][stride]: p

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // in a scalar register: what follows from it is uniform
    const bool shared_group = pl.paths_per_group > 1 || pl.groups_per_path == 1;
    const int slot = pl.paths_per_group > 1 ? wave / pl.items : 0;
    const int item = pl.paths_per_group > 1 ? wave - slot * pl.items : int(blockIdx.x % pl.groups_per_path) * 4 + wave;
    const int64_t row0 = shared_group ? int64_t(blockIdx.x) * pl.paths_per_group : int64_t(blockIdx.x / pl.groups_per_path);
    const int64_t row = row0 + slot;
    const bool live = item < pl.items && slot < pl.paths_per_group && row < sh.B;   // the same in every lane of a wavefront
    const int ti = (live ? item : 0) / pl.strips, strip = (live ? item : 0) - ti * pl.strips;
    const int strip_tiles = pl.tiles - 4 * strip < 4 ? pl.tiles - 4 * strip : 4;
    const float *bpv = static_cast<const float *>(sh.basepoint_value);
    const int shift = sh.basepoint ? 1 : 0;   // with a basepoint the scan's points are bp, x_0, x_1, ..

    // p of every path of the workgroup, zeros behind the d-th channel
    const int cvecs = stride / V;   // loads per staged point
    for (int e = tid; e < pl.paths_per_group * cvecs; e += 256) {
        const int p = e / cvecs, c = (e - p * cvecs) * V;
        const bool on = row0 + p < sh.B && c < d;
        const int64_t r = on ? row0 + p : 0;
        const int cc = on ? c : 0;
        const float *src = sh.basepoint ? (bpv != nullptr ? bpv + r * d + cc : path) : path + r * sh.L * d + cc;
        const TV v = *reinterpret_cast<const TV *>(src);
#pragma unroll
        for (int j = 0; j < V; ++j) start[p * stride + n2m_pos(c + j)] = on && !(sh.basepoint && bpv == nullptr) ? v[j] : 0.f;
    }

    n2m_f4 acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = n2m_f4(0.f);

    // Which point of which path an entry of the staged tile holds does not change from tile to tile.  Every load is
    // unconditional, on indices clamped into a path; entries of rows past the end of the batch, of points past the end
    // of the path and of the padding behind the last channel become zeros when the tile is written to LDS.
    const int staged = pl.paths_per_group * rows * cvecs;   // at most 256 * kN2mBatch
    TV held[kN2mBatch];
    const float *entry_row[kN2mBatch];    // channel c of point 0 of the entry's path
    const float *entry_base[kN2mBatch];   // the entry's channels of a basepoint given by value
    int entry_point[kN2mBatch], entry_lds[kN2mBatch];
    bool entry_on[kN2mBatch];
#pragma unroll
    for (int k = 0; k < kN2mBatch; ++k) {
        const int e = 256 * k + tid < staged ? 256 * k + tid : staged - 1;
        const int p = e / (rows * cvecs), rem = e - p * rows * cvecs, pt = rem / cvecs, c = (rem - pt * cvecs) * V;
        entry_on[k] = row0 + p < sh.B && c < d;
        entry_point[k] = pt;
        entry_lds[k] = (p * rows + pt) * stride + n2m_pos(c);   // the entry's V channels lie 4 floats apart
        entry_row[k] = path + (entry_on[k] ? (row0 + p) * sh.L * d + c : 0);
        entry_base[k] = bpv != nullptr && entry_on[k] ? bpv + (row0 + p) * d + c : bpv;
    }
    const auto load_tile = [&](int64_t t0) {
#pragma unroll
        for (int k = 0; k < kN2mBatch; ++k) {
            if (256 * k >= staged) break;   // the same for every thread
            const int64_t point = t0 + entry_point[k];
            const bool on = entry_on[k] && point <= sh.n_inc;
            const bool from_base = on && sh.basepoint && point == 0;
            const float *src = from_base && bpv != nullptr ? entry_base[k] : entry_row[k] + (on && !from_base ? point - shift : 0) * d;
            held[k] = *reinterpret_cast<const TV *>(src);
        }
    };

    const int k4 = lane >> 4, c16 = lane & 15;
    const float *my_pts = pts + slot * rows * stride + strip * 64 + c16 * 4;   // this lane's four scalars of a point
    const int a_off = n2m_pos(16 * ti + c16) - (strip * 64 + c16 * 4);          // its row scalar, relative to them
    const bool a_in_strip = ti >> 2 == strip;
    float p_i = 0.f;
    load_tile(0);
    for (int64_t t0 = 0; t0 < sh.n_inc; t0 += pl.tile) {
        lds_barrier();   // not __syncthreads(): the loads of the next tile stay in flight
#pragma unroll
        for (int k = 0; k < kN2mBatch; ++k) {
            if (256 * k >= staged) break;
            const int64_t point = t0 + entry_point[k];
            const bool zero = !entry_on[k] || point > sh.n_inc || (sh.basepoint && point == 0 && bpv == nullptr);
            if (256 * k + tid < staged) {
#pragma unroll
                for (int j = 0; j < V; ++j) pts[entry_lds[k] + 4 * j] = zero ? 0.f : held[k][j];
            }
        }
        if (t0 + pl.tile < sh.n_inc) load_tile(t0 + pl.tile);
        lds_barrier();
        if (t0 == 0) p_i = start[slot * stride + n2m_pos(16 * ti + c16)];
        const int nt = int(sh.n_inc - t0 < pl.tile ? sh.n_inc - t0 : pl.tile);
        if (live) {
            // four increments at a time, increment s + k4 in lane (k4, c16); MASKED: the step that runs past the tile's
            // end, whose missing increments count as zeros (read from the tile's last one)
            const auto step = [&](int s, auto masked) {
                constexpr bool MASKED = decltype(masked)::value;
                const bool on = !MASKED || s + k4 < nt;
                const float *x0 = my_pts + (on ? s + k4 : nt - 1) * stride, *x1 = x0 + stride;
                const n2m_f4 b0 = *reinterpret_cast<const n2m_f4 *>(x0), b1 = *reinterpret_cast<const n2m_f4 *>(x1);
                float a0, a1;
                if (a_in_strip) {   // the same for the whole wavefront
                    a0 = b0[ti & 3];
                    a1 = b1[ti & 3];
                } else {
                    a0 = x0[a_off];
                    a1 = x1[a_off];
                }
                const float l = on ? (a0 - p_i) + (a1 - p_i) : 0.f;   // twice m - p, from differences of points only
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    if (t < strip_tiles) {   // the same for the whole wavefront
                        const float r = on ? b1[t] - b0[t] : 0.f;
                        acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(l, r, acc[t], 0, 0, 0);
                    }
                }
            };
            int s = 0;
#pragma unroll 2
            for (; s + 4 <= nt; s += 4) step(s, std::false_type{});
            if (s < nt) step(s, std::true_type{});
        }
        // the last tile ends at the scan's last point: level 1, by the path's first workgroup
        if (t0 + pl.tile >= sh.n_inc && (shared_group || blockIdx.x % pl.groups_per_path == 0)) {
            for (int e = tid; e < pl.paths_per_group * d; e += 256) {
                const int p = e / d, c = e - p * d;
                if (row0 + p < sh.B)
                    out[(row0 + p) * sh.S + c] = pts[(p * rows + nt) * stride + n2m_pos(c)] - start[p * stride + n2m_pos(c)];
            }
        }
    }
    if (live) {
        // register r of lane (k4, c16) holds twice A_2[16 ti + 4 k4 + r][16 tj + c16]
        float *o = out + row * sh.S + d;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int j = 16 * (4 * strip + t) + c16;
            if (t < strip_tiles && j < d) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int i = 16 * ti + 4 * k4 + r;
                    if (i < d) o[int64_t(i) * d + j] = 0.5f * acc[t][r];
                }
            }
        }
    }
}

size_t n2m_lds(const N2mPlan &pl) { return sizeof(float) * size_t(pl.paths_per_group) * size_t(pl.stride) * size_t(pl.tile + 2); }

bool n2m_plan(const Shape &sh, const void *path, N2mPlan &pl)
{
    if (sh.N != 2 || sh.stream || sh.chunks > 1 || sh.d < 17 || sh.d > 256) return false;
    pl.tiles = (sh.d + 15) / 16;
    pl.strips = (pl.tiles + 3) / 4;
    pl.stride = 64 * pl.strips;
    pl.items = pl.tiles * pl.strips;
    if (pl.items <= 4) {
        pl.paths_per_group = 4 / pl.items;
        pl.groups_per_path = 1;
    } else {
        pl.paths_per_group = 1;
        pl.groups_per_path = (pl.items + 3) / 4;
    }
    // 16-byte (else 8-byte) loads where every row of d scalars, and so every point, starts on such a boundary
    pl.vec = 1;
    for (int v = 4; v > 1; v /= 2) {
        const auto aligned = [&](const void *q) { return reinterpret_cast<uintptr_t>(q) % (v * sizeof(float)) == 0; };
        if (sh.d % v == 0 && aligned(path) && aligned(sh.basepoint_value)) {
            pl.vec = v;
            break;
        }
    }
    // a tile of points within 32 KB and within one batch of loads, a multiple of four increments
    const int64_t loads_per_point = int64_t(pl.paths_per_group) * (pl.stride / pl.vec);
    int64_t tile = int64_t(32 * 1024) / (int64_t(sizeof(float)) * pl.paths_per_group * pl.stride) - 2;
    const int64_t by_loads = 256 * kN2mBatch / loads_per_point - 1;
    tile = tile < by_loads ? tile : by_loads;
    tile = tile > 128 ? 128 : tile;
    pl.tile = int(tile / 4 * 4);
    if (pl.tile < 4) return false;
    const int64_t groups = pl.groups_per_path > 1 ? sh.B * pl.groups_per_path : (sh.B + pl.paths_per_group - 1) / pl.paths_per_group;
    return groups <= 0x7fffffff && n2m_lds(pl) <= 64 * 1024;
}

template <int V>
hipError_t launch_n2m_v(const Shape &sh, const N2mPlan &pl, const float *path, float *out, hipStream_t st)
{
    const int64_t groups = pl.groups_per_path > 1 ? sh.B * pl.groups_per_path : (sh.B + pl.paths_per_group - 1) / pl.paths_per_group;
    hipLaunchKernelGGL((sig_forward_n2_mfma_kernel<V>), dim3(unsigned(groups)), dim3(256), n2m_lds(pl), st, sh, pl, path, out);
    return hipGetLastError();
}

}  // namespace

bool forward_n2_mfma_supported(const Shape &sh)
{
    N2mPlan pl;
    return n2m_plan(sh, nullptr, pl);
}

bool forward_n2_mfma_preferred(const Shape &sh)
{
    if (sh.d < 49 || !forward_n2_mfma_supported(sh)) return false;
    const int64_t padded = 16 * ((sh.d + 15) / 16);
    return 10 * padded * padded <= 13 * int64_t(sh.d) * sh.d;
}

hipError_t launch_forward_n2_mfma_f32(const Shape &sh, const float *path, float *out, hipStream_t st)
{
    N2mPlan pl;
    if (!n2m_plan(sh, path, pl)) return hipErrorNotSupported;
    switch (pl.vec) {
        case 4: return launch_n2m_v<4>(sh, pl, path, out, st);
        case 2: return launch_n2m_v<2>(sh, pl, path, out, st);
        default: return launch_n2m_v<1>(sh, pl, path, out, st);
    }
}

}  // namespace sig
