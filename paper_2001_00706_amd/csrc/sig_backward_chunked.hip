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
#include "sig_lane_ops.h"

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

// How the words of each level are spread over a wavefront's lanes in the chain of gradients: a word of level i sums
// sum_{j = 1 .. N - i} d^j products, and teams of 2^team_log2[i] lanes (1, 4, 16 or 64) share a word's sums.
struct ChainTeams {
    unsigned char team_log2[SIG_MAX_DEPTH + 1];
};

// gout = the gradient gin carried through the right multiplication by the signature cs.  For a word u of level i the
// sum over the words v of level j is a dot product of d^j consecutive scalars of level i + j of gin with level j of cs.
// An item is a wavefront's worth of teams of one level; the calling wavefront takes the items item0, item0 + step, .. of
// every level (STEP > 0: step is that constant, and the levels' items are dealt out in turn so that no wavefront is
// always first).  The order of the additions is fixed.  The result goes to gout and, if given, to gout2 as well.
// `lv` is the level table in LDS (see below): d^j and the offsets of levels j and i + j are built up as j grows.
struct ChainLevels {
    int words[SIG_MAX_DEPTH + 2];   // d^i
    int off[SIG_MAX_DEPTH + 2];     // offset of level i; off[N + 1] = S
    int team_log2[SIG_MAX_DEPTH + 2];
};

// The level tables as 32-bit numbers in LDS (S < 2^31), written by one thread at positions known at compile time: the
// shape sits in scalar registers, where a run-time index would move it to scratch memory.  Needs a barrier after it.
__device__ __forceinline__ void chain_levels_fill(const Shape &sh, const ChainTeams &teams, ChainLevels *lv)
{
    if (threadIdx.x == 0) {
#pragma unroll
        for (int k = 0; k <= SIG_MAX_DEPTH; ++k) {
            lv->words[k] = int(sh.pw[k]);
            lv->off[k] = int(sh.off[k]);
            lv->team_log2[k] = teams.team_log2[k];
        }
        lv->off[SIG_MAX_DEPTH + 1] = int(sh.off[SIG_MAX_DEPTH + 1]);
    }
}

template <typename T, int STEP>
__device__ __forceinline__ void stretch_adjoint_items(int N, int d, const ChainLevels *lv, const T *gin, const T *cs, T *gout, T *gout2,
                                                      int item0, int step_runtime)
{
    const int lane = threadIdx.x & 63;
    const int step = STEP > 0 ? STEP : step_runtime;
    int dealt = 0;
    for (int i = 1; i <= N; ++i) {
        const int words = lv->words[i], base = lv->off[i], after = lv->off[i + 1];
        const int log2 = lv->team_log2[i], team = 1 << log2, per_item = 64 >> log2;
        const int items = (words + per_item - 1) >> (6 - log2);
        const int member = lane & (team - 1);
        const int first = STEP > 0 ? ((item0 - dealt) & (STEP - 1)) : item0;
        for (int t = first; t < items; t += step) {
            const int word = t * per_item + (lane >> log2);
            const bool on = word < words;
            T acc = T(0);
            if (on) {
                int pwj = 1, offj = 0, offn = after;   // d^j, the offset of level j, the offset of level i + j
                for (int j = 1; j <= N - i; ++j) {
                    pwj *= d;
                    const T *seg = gin + offn + word * pwj, *cj = cs + offj;
#pragma unroll 4
                    for (int v = member; v < pwj; v += team) acc += seg[v] * cj[v];
                    offj += pwj;
                    offn += words * pwj;
                }
            }
            for (int hop = team >> 1; hop >= 1; hop >>= 1) acc += __shfl_xor(acc, hop, 64);   // the same for every lane
            if (on && member == 0) {
                acc += gin[base + word];
                gout[base + word] = acc;
                if (gout2 != nullptr) gout2[base + word] = acc;
            }
        }
        if (STEP > 0) dealt = (dealt + items) & (STEP - 1);
    }
}

// One step of the chain, g[b][c - 1] from g[b][c] and C[b][c], spread over the grid (rows of K signatures per path).
template <typename T>
__global__ void __launch_bounds__(256)
sig_stretch_adjoint_kernel(Shape sh, ChainTeams teams, int64_t K, int64_t c, const T *__restrict__ C, T *g)
{
    __shared__ ChainLevels lv;
    chain_levels_fill(sh, teams, &lv);
    __syncthreads();
    const int64_t b = blockIdx.y;
    stretch_adjoint_items<T, 0>(sh.N, sh.d, &lv, g + (b * K + c) * sh.S, C + (b * K + c) * sh.S, g + (b * K + c - 1) * sh.S, nullptr,
                                int(blockIdx.x) * 4 + (threadIdx.x >> 6), int(gridDim.x) * 4);
}

constexpr int kChainPerThread = 8;   // scalars of a stretch's signature a thread fetches ahead: `used` <= 8192

// The whole chain of a path in one workgroup of 16 wavefronts, while two gradients and the `used` scalars of a signature
// that take part (its levels below N) fit the LDS: the
// gradient being carried stays in LDS (two buffers take turns as source and result), the next stretch's signature is
// fetched into registers while the current step computes, and the barriers order LDS traffic only, so a step waits
// for no memory access but its own signature's arrival.
template <typename T>
__global__ void __launch_bounds__(1024)
sig_stretch_adjoint_chain_kernel(Shape sh, ChainTeams teams, int64_t K, int used, const T *__restrict__ C, T *__restrict__ g)
{
    extern __shared__ __align__(16) unsigned char chain_smem[];
    __shared__ ChainLevels lv;
    chain_levels_fill(sh, teams, &lv);   // the barrier of the first step comes before its first use
    const int S = int(sh.S), tid = threadIdx.x;
    T *from = reinterpret_cast<T *>(chain_smem), *to = from + S, *cl = to + S;
    const int64_t b = blockIdx.x;
    // of a stretch's signature the levels below N are used: the words v of the sums have at most N - 1 letters
    T creg[kChainPerThread];
    const T *c_next = C + (b * K + K - 1) * sh.S, *g_last = g + (b * K + K - 1) * sh.S;
#pragma unroll
    for (int r = 0; r < kChainPerThread; ++r) {
        const int e = tid + 1024 * r;
        creg[r] = e < used ? c_next[e] : T(0);
    }
    for (int e = tid; e < S; e += 1024) from[e] = g_last[e];
    for (int64_t c = K - 1; c >= 1; --c) {
#pragma unroll
        for (int r = 0; r < kChainPerThread; ++r) {
            const int e = tid + 1024 * r;
            if (e < used) cl[e] = creg[r];
        }
        lds_barrier();
        if (c > 1) {
            c_next = C + (b * K + c - 1) * sh.S;
#pragma unroll
            for (int r = 0; r < kChainPerThread; ++r) {
                const int e = tid + 1024 * r;
                creg[r] = e < used ? c_next[e] : T(0);
            }
        }
        stretch_adjoint_items<T, 16>(sh.N, sh.d, &lv, from, cl, to, g + (b * K + c - 1) * sh.S, tid >> 6, 16);
        lds_barrier();
        T *spare = from;
        from = to;
        to = spare;
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
    if (K < 2) return hipSuccess;
    ChainTeams teams;
    int64_t items = 0;
    for (int i = 0; i <= SIG_MAX_DEPTH; ++i) teams.team_log2[i] = 0;
    for (int i = 1; i <= sh.N; ++i) {
        int64_t cost = 0;
        for (int j = 1; i + j <= sh.N; ++j) cost += sh.pw[j];
        teams.team_log2[i] = cost <= 8 ? 0 : cost <= 64 ? 2 : cost <= 512 ? 4 : 6;
        const int64_t per_item = 64 >> teams.team_log2[i];
        items += (sh.pw[i] + per_item - 1) / per_item;
    }
    const int64_t paths = sh.B / K;   // sh.B counts stretches
    const int64_t used = sh.off[sh.N];   // levels 1 .. N - 1 of a stretch's signature
    const size_t lds = (2 * size_t(sh.S) + size_t(used)) * sizeof(T);
    if (lds + sizeof(ChainLevels) <= 64 * 1024 && used <= 1024 * kChainPerThread) {
        hipLaunchKernelGGL((sig_stretch_adjoint_chain_kernel<T>), dim3(unsigned(paths)), dim3(1024), lds, st, sh, teams, K, int(used), C,
                           g);
        return hipGetLastError();
    }
    const int64_t groups = (items + 3) / 4;
    const dim3 grid(unsigned(groups < 4096 ? groups : 4096), unsigned(paths));
    for (int64_t c = K - 1; c >= 1; --c) {
        hipLaunchKernelGGL((sig_stretch_adjoint_kernel<T>), grid, dim3(256), 0, st, sh, teams, K, c, C, g);
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
