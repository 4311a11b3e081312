// Prefix-tree kernel family (fp32 and fp64, final and stream mode): d = 2..8 at depths 2..9 and d = 9..16 at depths 2..6,
// for states too large for the
// small-state kernel and that the matrix-core families do not serve - in particular few paths with a large
// signature, where the state of one path (up to millions of scalars) has to be spread over the whole chip.
//
// The fused multiply-exponentiate (paper section 4.1, eq. "fusedterm") updates the coefficient of a word
// from the coefficients of that word's prefixes only.  So a thread that stands for a word u of P = N - U
// letters can carry, with no communication at all, the coefficients of u and of its prefixes (the same
// prefix is carried, and updated identically, by every thread below it) together with the whole subtree of
// the words u c and u c c' below it (U = 2 levels, d + d^2 scalars in registers).  Per increment a thread
// runs the Horner chains along its own word (scalars), then the chains into its subtree; the top level,
// which is most of the work, is touched exactly once.  A path of d^P such threads never exchanges a value,
// so the threads of one path may sit in any number of workgroups: the grid is (words / 256) x paths.
// When a path has fewer than 256 such words, several paths share a workgroup.
#ifndef SIG_TREE_IMPL_H_
#define SIG_TREE_IMPL_H_

#include "sig_internal.h"

namespace sig {
namespace {

constexpr int kTreeTile = 32;      // increments staged in LDS at a time
constexpr int kTreeMaxPaths = 16;  // paths that may share a workgroup

__host__ __device__ constexpr int64_t tree_off(int d, int k)   // offset of level k (1-based) in a flat element
{
    int64_t off = 0, p = 1;
    for (int j = 1; j < k; ++j) {
        p *= d;
        off += p;
    }
    return off;
}

template <int D, int N>
struct TreeShape {
    // levels kept per thread below its word: two (d + d^2 scalars) up to 8 channels, one (d scalars) beyond
    static constexpr int U = N - 1 < (D <= 8 ? 2 : 1) ? N - 1 : (D <= 8 ? 2 : 1);
    static constexpr int P = N - U;                       // letters of a thread's word
    static constexpr int64_t kWords = tree_off(D, P + 1) - tree_off(D, P);   // d^P words of P letters per path
    static constexpr int kPathsPerGroup =                 // paths sharing a workgroup
        kWords >= 256 ? 1 : (256 / kWords < kTreeMaxPaths ? int(256 / kWords) : kTreeMaxPaths);
    static constexpr int64_t kGroupsPerPath = kWords >= 256 ? (kWords + 255) / 256 : 1;
    static constexpr int64_t kS = tree_off(D, N + 1);
};

__device__ __forceinline__ float fma_t(float a, float b, float c) { return __builtin_fmaf(a, b, c); }
__device__ __forceinline__ double fma_t(double a, double b, double c) { return __builtin_fma(a, b, c); }

template <typename T, int D, int N>
__global__ void __launch_bounds__(256)
sig_tree_kernel(Shape sh, const T *__restrict__ path, T *__restrict__ out)
{
    using TS = TreeShape<D, N>;
    constexpr int U = TS::U, P = TS::P, PPG = TS::kPathsPerGroup;
    constexpr int H1 = U >= 1 ? D : 1, H2 = U >= 2 ? D * D : 1;
    __shared__ T zt[PPG * kTreeTile * D];

    const int tid = threadIdx.x;
    // which path of the workgroup, which word of the path
    const int slot_raw = TS::kWords >= 256 ? 0 : tid / int(TS::kWords);
    const int slot = slot_raw < PPG ? slot_raw : PPG - 1;   // threads beyond the last path of the workgroup idle along
    const int64_t u = TS::kWords >= 256 ? int64_t(blockIdx.x % TS::kGroupsPerPath) * 256 + tid : tid % int(TS::kWords);
    const int64_t row = TS::kWords >= 256 ? int64_t(blockIdx.x / TS::kGroupsPerPath) : int64_t(blockIdx.x) * PPG + slot;
    const bool live = u < TS::kWords && slot_raw < PPG && row < sh.B;

    int cl[P + 1];   // letters of this thread's word
    {
        int64_t rest = live ? u : 0;
#pragma unroll
        for (int i = P; i >= 1; --i) {
            cl[i] = int(rest % D);
            rest /= D;
        }
    }
    T rk[N + 2];
#pragma unroll
    for (int m = 1; m <= N + 1; ++m) rk[m] = T(1) / T(m);

    T A[P + 1];      // coefficients of the prefixes of the word, and of the word itself (level P)
    T B1[H1];        // words u c
    T B2[H2];        // words u c c'
#pragma unroll
    for (int i = 0; i <= P; ++i) A[i] = T(0);
#pragma unroll
    for (int c = 0; c < H1; ++c) B1[c] = T(0);
#pragma unroll
    for (int c = 0; c < H2; ++c) B2[c] = T(0);

    // the rows (paths or chunks of paths) this workgroup serves, for the staging of their increments
    const int64_t row0 = TS::kWords >= 256 ? int64_t(blockIdx.x / TS::kGroupsPerPath) : int64_t(blockIdx.x) * PPG;
    int64_t n_max = 0;   // most increments among them
    for (int p = 0; p < PPG; ++p)
        if (row0 + p < sh.B) {
            const ChunkView cv = chunk_view(row0 + p, sh.chunks, sh.chunk_len, sh.n_inc);
            n_max = cv.n > n_max ? cv.n : n_max;
        }
    const T *bpv = static_cast<const T *>(sh.basepoint_value);
    // chunks laid out in a stream-mode output: this thread's chunk, and the rows it reads and writes
    const ChunkView mine = chunk_view(live ? row : 0, sh.chunks, sh.chunk_len, sh.n_inc);
    const int64_t first_row = mine.path * sh.n_inc + mine.inc0;   // the row of the chunk's first increment
    if (sh.rows_in_stream && sh.stream && live && mine.inc0 > 0 && mine.n > 0) {
        const T *o = out + (first_row - 1) * TS::kS;   // the signature of everything before the chunk
        int64_t q = u;
#pragma unroll
        for (int i = P; i >= 1; --i) {
            A[i] = o[tree_off(D, i) + q];
            q /= D;
        }
        if constexpr (U >= 1) {
#pragma unroll
            for (int c = 0; c < D; ++c) B1[c] = o[tree_off(D, P + 1) + u * D + c];
        }
        if constexpr (U >= 2) {
#pragma unroll
            for (int c = 0; c < D * D; ++c) B2[c] = o[tree_off(D, P + 2) + u * (D * D) + c];
        }
    }

    // this thread's words of one signature; a prefix is written by the first thread below it
    auto store = [&](T *o) {
        int64_t q = u, width = 1;
#pragma unroll
        for (int i = P; i >= 1; --i) {
            if (u % width == 0) o[tree_off(D, i) + q] = A[i];
            q /= D;
            width *= D;
        }
        if constexpr (U >= 1) {
#pragma unroll
            for (int c = 0; c < D; ++c) o[tree_off(D, P + 1) + u * D + c] = B1[c];
        }
        if constexpr (U >= 2) {
#pragma unroll
            for (int c = 0; c < D * D; ++c) o[tree_off(D, P + 2) + u * (D * D) + c] = B2[c];
        }
    };

    for (int64_t t0 = 0; t0 < n_max; t0 += kTreeTile) {
        __syncthreads();
        for (int e = tid; e < PPG * kTreeTile * D; e += 256) {
            const int p = e / (kTreeTile * D), i = (e / D) % kTreeTile, c = e % D;
            // rows past the end of the batch and increments past the end of a row add nothing; both loads are
            // unconditional, on indices clamped into a path, so that they are in flight together
            const ChunkView cv = chunk_view(row0 + p < sh.B ? row0 + p : 0, sh.chunks, sh.chunk_len, sh.n_inc);
            const bool on = row0 + p < sh.B && t0 + i < cv.n;
            const T *x = path + cv.path * sh.L * D;
            const int64_t i_hi = on ? cv.inc0 + t0 + i + (sh.basepoint ? 0 : 1) : (sh.basepoint ? 0 : 1);
            const bool first = i_hi == 0;   // the increment from the basepoint
            const T hi = x[i_hi * D + c];
            const T lo = bpv != nullptr && first ? bpv[cv.path * D + c] : x[(first ? 0 : i_hi - 1) * D + c];
            zt[e] = on ? hi - (first && bpv == nullptr ? T(0) : lo) : T(0);
        }
        __syncthreads();
        const int nt = int(n_max - t0 < kTreeTile ? n_max - t0 : kTreeTile);
        const T *zrow = zt + slot * kTreeTile * D;
        for (int s = 0; s < nt; ++s, zrow += D) {
            // Horner terms along the word: Hn[k] = T^(k)_i for the level i just passed, k > i
            T Hn[N + 2];
            {
                const T zc = zrow[cl[1]];
#pragma unroll
                for (int k = 2; k <= N; ++k) Hn[k] = fma_t(zc, rk[k], A[1]);
                A[1] += zc;
            }
#pragma unroll
            for (int i = 2; i <= P; ++i) {
                const T zc = zrow[cl[i]];
                const T a = A[i];
                A[i] = fma_t(Hn[i], zc, a);
#pragma unroll
                for (int k = i + 1; k <= N; ++k) Hn[k] = fma_t(Hn[k], zc * rk[k - i + 1], a);
            }
            if constexpr (U >= 1) {
                T zu[D];
#pragma unroll
                for (int c = 0; c < D; ++c) zu[c] = zrow[c];
                if constexpr (U == 1) {
#pragma unroll
                    for (int c = 0; c < D; ++c) B1[c] = fma_t(Hn[P + 1], zu[c], B1[c]);
                } else {
#pragma unroll
                    for (int c = 0; c < D; ++c) {
                        const T t1 = fma_t(Hn[P + 2], zu[c] * rk[2], B1[c]);   // T^(N)_{P+1}[u c]
                        B1[c] = fma_t(Hn[P + 1], zu[c], B1[c]);
#pragma unroll
                        for (int j = 0; j < D; ++j) B2[c * D + j] = fma_t(t1, zu[j], B2[c * D + j]);
                    }
                }
            }
            // stream mode: the signature so far (a chunk leaves out its last row, which holds its final value already)
            if (sh.stream && live) {
                if (!sh.rows_in_stream)
                    store(out + (row * sh.n_inc + t0 + s) * TS::kS);
                else if (t0 + s + 1 < mine.n)
                    store(out + (first_row + t0 + s) * TS::kS);
            }
        }
    }

    if (live && !sh.stream) {
        if (!sh.rows_in_stream)
            store(out + row * TS::kS);
        else if (mine.n > 0)
            store(out + (first_row + mine.n - 1) * TS::kS);
    }
}

template <typename T, int D, int N>
hipError_t launch_tree_dn(const Shape &sh, const T *path, T *out, hipStream_t st)
{
    using TS = TreeShape<D, N>;
    const int64_t groups = TS::kWords >= 256 ? sh.B * TS::kGroupsPerPath : (sh.B + TS::kPathsPerGroup - 1) / TS::kPathsPerGroup;
    if (groups > 0x7fffffff) return hipErrorNotSupported;
    hipLaunchKernelGGL((sig_tree_kernel<T, D, N>), dim3(unsigned(groups)), dim3(256), 0, st, sh, path, out);
    return hipGetLastError();
}

constexpr int kTreeMaxDepth = 9;       // d = 2..8
constexpr int kTreeWideMaxDepth = 6;   // d = 9..16

template <typename T, int D>
hipError_t launch_tree_d(const Shape &sh, const T *path, T *out, hipStream_t st)
{
    switch (sh.N) {
        case 2: return launch_tree_dn<T, D, 2>(sh, path, out, st);
        case 3: return launch_tree_dn<T, D, 3>(sh, path, out, st);
        case 4: return launch_tree_dn<T, D, 4>(sh, path, out, st);
        case 5: return launch_tree_dn<T, D, 5>(sh, path, out, st);
        case 6: return launch_tree_dn<T, D, 6>(sh, path, out, st);
    }
    if constexpr (D <= 8) {
        switch (sh.N) {
            case 7: return launch_tree_dn<T, D, 7>(sh, path, out, st);
            case 8: return launch_tree_dn<T, D, 8>(sh, path, out, st);
            case 9: return launch_tree_dn<T, D, 9>(sh, path, out, st);
        }
    }
    return hipErrorNotSupported;
}

}  // namespace
}  // namespace sig

#endif  // SIG_TREE_IMPL_H_
