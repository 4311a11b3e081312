// Prefix-tree kernel family (fp32, final mode): any d = 2..8 at depths 2..9 whose state is too large for the
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
    static constexpr int U = N >= 3 ? 2 : N - 1;          // levels kept per thread below its word
    static constexpr int P = N - U;                       // letters of a thread's word
    static constexpr int64_t kWords = tree_off(D, P + 1) - tree_off(D, P);   // d^P words of P letters per path
    static constexpr int kPathsPerGroup =                 // paths sharing a workgroup
        kWords >= 256 ? 1 : (256 / kWords < kTreeMaxPaths ? int(256 / kWords) : kTreeMaxPaths);
    static constexpr int64_t kGroupsPerPath = kWords >= 256 ? (kWords + 255) / 256 : 1;
    static constexpr int64_t kS = tree_off(D, N + 1);
};

template <int D, int N>
__global__ void __launch_bounds__(256)
sig_tree_kernel(Shape sh, const float *__restrict__ path, float *__restrict__ out)
{
    using TS = TreeShape<D, N>;
    constexpr int U = TS::U, P = TS::P, PPG = TS::kPathsPerGroup;
    constexpr int H1 = U >= 1 ? D : 1, H2 = U >= 2 ? D * D : 1;
    __shared__ float zt[PPG * kTreeTile * D];

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
    float rk[N + 2];
#pragma unroll
    for (int m = 1; m <= N + 1; ++m) rk[m] = 1.0f / float(m);

    float A[P + 1];      // coefficients of the prefixes of the word, and of the word itself (level P)
    float B1[H1];        // words u c
    float B2[H2];        // words u c c'
#pragma unroll
    for (int i = 0; i <= P; ++i) A[i] = 0.0f;
#pragma unroll
    for (int c = 0; c < H1; ++c) B1[c] = 0.0f;
#pragma unroll
    for (int c = 0; c < H2; ++c) B2[c] = 0.0f;

    // the rows (paths or chunks of paths) this workgroup serves, for the staging of their increments
    const int64_t row0 = TS::kWords >= 256 ? int64_t(blockIdx.x / TS::kGroupsPerPath) : int64_t(blockIdx.x) * PPG;
    int64_t n_max = 0;   // most increments among them
    for (int p = 0; p < PPG; ++p)
        if (row0 + p < sh.B) {
            const ChunkView cv = chunk_view(row0 + p, sh.chunks, sh.chunk_len, sh.n_inc);
            n_max = cv.n > n_max ? cv.n : n_max;
        }
    const float *bpv = static_cast<const float *>(sh.basepoint_value);

    for (int64_t t0 = 0; t0 < n_max; t0 += kTreeTile) {
        __syncthreads();
        for (int e = tid; e < PPG * kTreeTile * D; e += 256) {
            const int p = e / (kTreeTile * D), i = (e / D) % kTreeTile, c = e % D;
            float z = 0.0f;   // rows past the end of the batch and increments past the end of a row add nothing
            if (row0 + p < sh.B) {
                const ChunkView cv = chunk_view(row0 + p, sh.chunks, sh.chunk_len, sh.n_inc);
                if (t0 + i < cv.n) {
                    const float *x = path + cv.path * sh.L * D;
                    const int64_t i_hi = cv.inc0 + t0 + i + (sh.basepoint ? 0 : 1);
                    const float lo = i_hi > 0 ? x[(i_hi - 1) * D + c] : bpv != nullptr ? bpv[cv.path * D + c] : 0.0f;
                    z = x[i_hi * D + c] - lo;
                }
            }
            zt[e] = z;
        }
        __syncthreads();
        const int nt = int(n_max - t0 < kTreeTile ? n_max - t0 : kTreeTile);
        const float *zrow = zt + slot * kTreeTile * D;
        for (int s = 0; s < nt; ++s, zrow += D) {
            // Horner terms along the word: T[k] = T^(k)_i for the level i just passed, k > i
            float T[N + 2];
            {
                const float zc = zrow[cl[1]];
#pragma unroll
                for (int k = 2; k <= N; ++k) T[k] = __builtin_fmaf(zc, rk[k], A[1]);
                A[1] += zc;
            }
#pragma unroll
            for (int i = 2; i <= P; ++i) {
                const float zc = zrow[cl[i]];
                const float a = A[i];
                A[i] = __builtin_fmaf(T[i], zc, a);
#pragma unroll
                for (int k = i + 1; k <= N; ++k) T[k] = __builtin_fmaf(T[k], zc * rk[k - i + 1], a);
            }
            if constexpr (U >= 1) {
                float zu[D];
#pragma unroll
                for (int c = 0; c < D; ++c) zu[c] = zrow[c];
                if constexpr (U == 1) {
#pragma unroll
                    for (int c = 0; c < D; ++c) B1[c] = __builtin_fmaf(T[P + 1], zu[c], B1[c]);
                } else {
#pragma unroll
                    for (int c = 0; c < D; ++c) {
                        const float t1 = __builtin_fmaf(T[P + 2], zu[c] * rk[2], B1[c]);   // T^(N)_{P+1}[u c]
                        B1[c] = __builtin_fmaf(T[P + 1], zu[c], B1[c]);
#pragma unroll
                        for (int j = 0; j < D; ++j) B2[c * D + j] = __builtin_fmaf(t1, zu[j], B2[c * D + j]);
                    }
                }
            }
        }
    }

    if (!live) return;
    float *o = out + row * TS::kS;
    // a prefix is written by the first thread below it
    {
        int64_t q = u, width = 1;
#pragma unroll
        for (int i = P; i >= 1; --i) {
            if (u % width == 0) o[tree_off(D, i) + q] = A[i];
            q /= D;
            width *= D;
        }
    }
    if constexpr (U >= 1) {
#pragma unroll
        for (int c = 0; c < D; ++c) o[tree_off(D, P + 1) + u * D + c] = B1[c];
    }
    if constexpr (U >= 2) {
#pragma unroll
        for (int c = 0; c < D * D; ++c) o[tree_off(D, P + 2) + u * (D * D) + c] = B2[c];
    }
}

template <int D, int N>
hipError_t launch_tree_dn(const Shape &sh, const float *path, float *out, hipStream_t st)
{
    using TS = TreeShape<D, N>;
    const int64_t groups = TS::kWords >= 256 ? sh.B * TS::kGroupsPerPath : (sh.B + TS::kPathsPerGroup - 1) / TS::kPathsPerGroup;
    if (groups > 0x7fffffff) return hipErrorNotSupported;
    hipLaunchKernelGGL((sig_tree_kernel<D, N>), dim3(unsigned(groups)), dim3(256), 0, st, sh, path, out);
    return hipGetLastError();
}

template <int D>
hipError_t launch_tree_d(const Shape &sh, const float *path, float *out, hipStream_t st)
{
    switch (sh.N) {
        case 2: return launch_tree_dn<D, 2>(sh, path, out, st);
        case 3: return launch_tree_dn<D, 3>(sh, path, out, st);
        case 4: return launch_tree_dn<D, 4>(sh, path, out, st);
        case 5: return launch_tree_dn<D, 5>(sh, path, out, st);
        case 6: return launch_tree_dn<D, 6>(sh, path, out, st);
        case 7: return launch_tree_dn<D, 7>(sh, path, out, st);
        case 8: return launch_tree_dn<D, 8>(sh, path, out, st);
        case 9: return launch_tree_dn<D, 9>(sh, path, out, st);
    }
    return hipErrorNotSupported;
}

}  // namespace

bool tree_supported(const Shape &sh)
{
    return !sh.stream && sh.d >= 2 && sh.d <= 8 && sh.N >= 2 && sh.N <= 9 && sh.S < (int64_t(1) << 31);
}

hipError_t launch_tree_f32(const Shape &sh, const float *path, float *out, hipStream_t st)
{
    if (!tree_supported(sh)) return hipErrorNotSupported;
    switch (sh.d) {
        case 2: return launch_tree_d<2>(sh, path, out, st);
        case 3: return launch_tree_d<3>(sh, path, out, st);
        case 4: return launch_tree_d<4>(sh, path, out, st);
        case 5: return launch_tree_d<5>(sh, path, out, st);
        case 6: return launch_tree_d<6>(sh, path, out, st);
        case 7: return launch_tree_d<7>(sh, path, out, st);
        case 8: return launch_tree_d<8>(sh, path, out, st);
    }
    return hipErrorNotSupported;
}

}  // namespace sig
