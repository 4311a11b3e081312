// Gradient of the signature with respect to the path, prefix-tree family (d = 2..8 at N = 2..9, d = 9..16 at N = 2..6,
// final and stream mode): the recurrences of sig_backward.hip with no communication between threads, so that the
// state of one path can be spread over any number of workgroups (paper section 5.3, appendix C).
//
// A thread stands for a word u of P = N - U letters and owns the subtree of the words u c and u c c'
// below it (U = 2 levels, in registers; U = 1 beyond 8 channels), exactly as in sig_tree_impl.h.
//   * "Up" (undo the increment, Horner terms T^(k)_i) needs the signature at the prefixes of u only; every
//     thread carries its own copy of them.
//   * "Down" moves cotangent from a word to its prefixes, D^(k)_{i-1}[p] = sum_c D^(k)_i[p c] z[c]/(k-i+1).
//     Inside the subtree that sum is local.  Above it, the map from the output cotangent to the gradient is
//     linear, so the cotangent of a prefix may stay split into the parts that arrived through each thread:
//     a thread keeps, for each of its prefixes, only the part that came up through its own word, and the
//     gradient of an increment is the sum of every thread's contribution.  (The cotangent a prefix has of
//     its own in the output gradient is given to the first thread below it.)
//   * That one sum, over all threads of a path and per increment, is finished by a second kernel: every
//     workgroup (for paths of at most 64 words: every thread) writes its partial sums to a workspace
//     [row][group][increment][d].
#ifndef SIG_TREE_BACKWARD_IMPL_H_
#define SIG_TREE_BACKWARD_IMPL_H_

#include "sig_internal.h"
#include "sig_lane_ops.h"

namespace sig {
namespace {


constexpr int kTbTile = 32;      // increments staged in LDS at a time
constexpr int kTbMaxPaths = 16;  // paths that may share a workgroup

__host__ __device__ constexpr int64_t tb_off(int d, int k)   // offset of level k (1-based) in a flat element
{
    int64_t off = 0, p = 1;
    for (int j = 1; j < k; ++j) {
        p *= d;
        off += p;
    }
    return off;
}

template <int D, int N>
struct TbShape {
    // levels kept per thread below its word: two (d + d^2 scalars) up to 8 channels, one (d scalars) beyond
    static constexpr int U = N - 1 < (D <= 8 ? 2 : 1) ? N - 1 : (D <= 8 ? 2 : 1);
    static constexpr int P = N - U;
    static constexpr int64_t kWords = tb_off(D, P + 1) - tb_off(D, P);   // threads a path needs
    static constexpr bool kMulti = kWords >= 256;   // a path spans several workgroups
    // From 65 words on, a path takes whole wavefronts (2..4, idle lanes at the end), each wavefront sums its lanes'
    // parts of an increment's gradient and the sums meet in LDS once per tile: one partial sum per path and
    // workgroup.  Shorter paths are packed thread after thread and every thread writes its own part (summing
    // over a wavefront costs d x 7 instructions per increment, which a path of one wavefront does not win back).
    static constexpr bool kWide = kWords > 64;
    static constexpr int kWavesPerPath = kMulti ? 4 : int((kWords + 63) / 64);
    static constexpr int kPathsPerGroup =
        kWide ? (kMulti ? 1 : 4 / kWavesPerPath) : (256 / kWords < kTbMaxPaths ? int(256 / kWords) : kTbMaxPaths);
    static constexpr int64_t kGroupsPerPath = kMulti ? (kWords + 255) / 256 : 1;   // workgroups per path
    static constexpr int64_t kPartials = kWide ? kGroupsPerPath : kWords;          // partial sums per path and increment
    static constexpr int64_t kS = tb_off(D, N + 1);
};

__device__ __forceinline__ float fma_t(float a, float b, float c) { return __builtin_fmaf(a, b, c); }
__device__ __forceinline__ double fma_t(double a, double b, double c) { return __builtin_fma(a, b, c); }

template <typename T, int D, int N, bool STREAM>
__global__ void __launch_bounds__(256)
sig_tree_backward_kernel(Shape sh, const T *__restrict__ path, const T *__restrict__ sig,
                         const T *__restrict__ gout, T *__restrict__ partial)
{
    using TS = TbShape<D, N>;
    constexpr int U = TS::U, P = TS::P, PPG = TS::kPathsPerGroup;
    constexpr int H1 = U >= 1 ? D : 1, H2 = U >= 2 ? D * D : 1;
    constexpr int64_t kS = TS::kS;
    __shared__ T zt[PPG * kTbTile * D];
    __shared__ T part[TS::kWide ? kTbTile * 4 * D : 1];   // [increment of the tile][wavefront][channel]

    constexpr int WPP = TS::kWavesPerPath;
    const int tid = threadIdx.x;
    const int slot_raw = TS::kMulti ? 0 : TS::kWide ? (tid >> 6) / WPP : tid / int(TS::kWords);
    const int slot = slot_raw < PPG ? slot_raw : PPG - 1;
    const int64_t u_raw = TS::kMulti  ? int64_t(blockIdx.x % TS::kGroupsPerPath) * 256 + tid
                          : TS::kWide ? int64_t(tid - slot_raw * WPP * 64)
                                      : int64_t(tid % int(TS::kWords));
    const int64_t row = TS::kMulti ? int64_t(blockIdx.x / TS::kGroupsPerPath) : int64_t(blockIdx.x) * PPG + slot;
    const bool live = u_raw < TS::kWords && slot_raw < PPG && row < sh.B;
    const int64_t u = live ? u_raw : 0;   // idle threads shadow word 0 of a valid row and contribute nothing
    const int64_t my_row = live ? row : (row < sh.B ? row : 0);

    int cl[P + 1];        // letters of the word
    int64_t pre[P + 1];   // index of its prefix of i letters inside level i
    bool first[P + 1];    // whether this thread is the first one below that prefix
    {
        int64_t rest = u, width = 1;
#pragma unroll
        for (int i = P; i >= 1; --i) {
            pre[i] = rest;
            first[i] = live && (u % width == 0);
            cl[i] = int(rest % D);
            rest /= D;
            width *= D;
        }
    }
    T rk[N + 2];
#pragma unroll
    for (int m = 1; m <= N + 1; ++m) rk[m] = T(1) / T(m);

    const int64_t per_row = STREAM ? sh.n_inc * kS : kS;
    const T *sg = sig + my_row * per_row;
    const T *go = gout + my_row * per_row;

    struct Share {
        T lo[P + 1];
        T h1[H1];
        T h2[H2];
    };
    // A thread's share of one flat element.  `own_only`: a prefix's value counts for the first thread below it
    // only (cotangents); otherwise every thread takes it (the signature).
    auto load_share = [&](const T *e, bool own_only, bool with_h1, bool with_h2) {
        Share s = {};
#pragma unroll
        for (int i = 1; i <= P; ++i) s.lo[i] = (!own_only || first[i]) ? e[tb_off(D, i) + pre[i]] : T(0);
        if constexpr (U >= 1) {
            if (with_h1) {
#pragma unroll
                for (int c = 0; c < D; ++c) s.h1[c] = e[tb_off(D, P + 1) + u * D + c];
            }
        }
        if constexpr (U >= 2) {
            if (with_h2) {
#pragma unroll
                for (int c = 0; c < D * D; ++c) s.h2[c] = e[tb_off(D, P + 2) + u * (D * D) + c];
            }
        }
        return s;
    };

    Share G = load_share(STREAM ? go + (sh.n_inc - 1) * kS : go, true, true, true);
    if (!live) G = Share{};
    Share A = {};
    if constexpr (!STREAM) A = load_share(sg, false, U >= 2, false);
    // Stream mode reads a row of the forward output and a row of its cotangent at every increment.  In fp32 both are
    // fetched an increment ahead of their use, so that a trip to memory is not part of every step of the chain.  In
    // fp64 they are fetched where they are used: two more shares of a flat element (up to 94 registers each at d = 6)
    // take these kernels to 350 and more registers per lane, and the code generated for d = 4, N = 8; d = 5, N = 7;
    // d = 6, N = 6 and d = 8, N = 6 then lost the cotangent of the levels above a thread's word at the first
    // increment (tests/test_backward_gpu.py: test_tree_gradient_every_shape).
    constexpr bool kAhead = STREAM && sizeof(T) == 4;
    Share A_ahead = {};
    if constexpr (kAhead) {
        if (sh.n_inc >= 2) A_ahead = load_share(sg + (sh.n_inc - 2) * kS, false, U >= 2, false);
    }

    // rows served by this workgroup, for the staging of their increments
    const int64_t row0 = TS::kMulti ? int64_t(blockIdx.x / TS::kGroupsPerPath) : int64_t(blockIdx.x) * PPG;
    const T *bpv = static_cast<const T *>(sh.basepoint_value);
    // where the partial sums go: [row][group][increment][D]; group = the workgroup's number inside its path (wavefront
    // sums) or the thread's word (short paths)
    const int64_t wg_group = TS::kMulti ? int64_t(blockIdx.x % TS::kGroupsPerPath) : 0;
    T *pp = partial + (my_row * TS::kPartials + (TS::kWide ? wg_group : u)) * sh.n_inc * D;

    for (int64_t t0 = ((sh.n_inc - 1) / kTbTile) * kTbTile; t0 >= 0; t0 -= kTbTile) {
        const int nt = int(sh.n_inc - t0 < kTbTile ? sh.n_inc - t0 : kTbTile);
        __syncthreads();
        for (int e = tid; e < PPG * kTbTile * D; e += 256) {
            const int p = e / (kTbTile * D), i = (e / D) % kTbTile, c = e % D;
            T z = T(0);
            if (row0 + p < sh.B && i < nt) {
                const T *x = path + (row0 + p) * sh.L * D;
                const int64_t i_hi = t0 + i + (sh.basepoint ? 0 : 1);
                const T lo = i_hi > 0 ? x[(i_hi - 1) * D + c] : bpv != nullptr ? bpv[(row0 + p) * D + c] : T(0);
                z = x[i_hi * D + c] - lo;
            }
            zt[e] = z;
        }
        __syncthreads();

        for (int i = nt - 1; i >= 0; --i) {
            const int64_t s = t0 + i;
            const T *zrow = zt + (slot * kTbTile + i) * D;
            T zc[P + 1];
#pragma unroll
            for (int j = 1; j <= P; ++j) zc[j] = zrow[cl[j]];
            T zu[D];
#pragma unroll
            for (int c = 0; c < D; ++c) zu[c] = zrow[c];

            Share G_ahead = {};
            if constexpr (kAhead) {
                // the signature after s increments is output entry s-1 (the identity for s = 0)
                A = s > 0 ? A_ahead : Share{};
                if (s >= 2) A_ahead = load_share(sg + (s - 2) * kS, false, U >= 2, false);
                if (s > 0 && live) G_ahead = load_share(go + (s - 1) * kS, true, true, true);   // added at the end of this step
            } else if constexpr (STREAM) {
                A = s > 0 ? load_share(sg + (s - 1) * kS, false, U >= 2, false) : Share{};
            }

            // ---- up: Hn[j][k] = T^(k)_j at this thread's word; the signature before the increment
            T Hn[P + 1][N + 2];
            T a_lo[P + 1];
            a_lo[1] = STREAM ? A.lo[1] : A.lo[1] - zc[1];
#pragma unroll
            for (int k = 2; k <= N; ++k) Hn[1][k] = fma_t(zc[1], rk[k], a_lo[1]);
#pragma unroll
            for (int j = 2; j <= P; ++j) {
                if (j < N) {
                    a_lo[j] = STREAM ? A.lo[j] : fma_t(-Hn[j - 1][j], zc[j], A.lo[j]);
#pragma unroll
                    for (int k = j + 1; k <= N; ++k) Hn[j][k] = fma_t(Hn[j - 1][k], zc[j] * rk[k - j + 1], a_lo[j]);
                } else {
                    a_lo[j] = T(0);
                }
            }
            T a_h1[H1], Th1[H1];
            if constexpr (U >= 2) {
#pragma unroll
                for (int c = 0; c < D; ++c) {
                    a_h1[c] = STREAM ? A.h1[c] : fma_t(-Hn[P][P + 1], zu[c], A.h1[c]);
                    Th1[c] = fma_t(Hn[P][N], zu[c] * rk[2], a_h1[c]);
                }
            }
            if constexpr (!STREAM) {
#pragma unroll
                for (int j = 1; j <= P; ++j) A.lo[j] = a_lo[j];
                if constexpr (U >= 2) {
#pragma unroll
                    for (int c = 0; c < D; ++c) A.h1[c] = a_h1[c];
                }
            }

            // ---- down
            T dz[D];
#pragma unroll
            for (int c = 0; c < D; ++c) dz[c] = T(0);
            T Dc[N + 2];   // Dc[k] = this thread's part of D^(k)_j at its prefix of the level j being processed
#pragma unroll
            for (int k = 0; k <= N + 1; ++k) Dc[k] = T(0);
            T Dh[H1];
            if constexpr (U >= 2) {
#pragma unroll
                for (int c = 0; c < D; ++c) {
                    T acc = T(0);
#pragma unroll
                    for (int j = 0; j < D; ++j) {
                        acc = fma_t(G.h2[c * D + j], zu[j], acc);
                        dz[j] = fma_t(Th1[c], G.h2[c * D + j], dz[j]);
                    }
                    Dh[c] = acc;
                }
            }
            if constexpr (U >= 1) {
                T acc1 = T(0), acc2 = T(0);
#pragma unroll
                for (int c = 0; c < D; ++c) {
                    dz[c] = fma_t(Hn[P][P + 1], G.h1[c], dz[c]);
                    acc1 = fma_t(G.h1[c], zu[c], acc1);
                    if constexpr (U >= 2) {
                        dz[c] = fma_t(Hn[P][P + 2] * rk[2], Dh[c], dz[c]);
                        acc2 = fma_t(Dh[c], zu[c], acc2);
                        G.h1[c] += Dh[c];
                    }
                }
                Dc[P + 1] = acc1;
                if constexpr (U >= 2) Dc[P + 2] = acc2 * rk[2];
            }
            // levels P .. 1 along the word: one scalar per chain, this thread's part only
#pragma unroll
            for (int j = P; j >= 1; --j) {
                T contrib = j >= 2 ? Hn[j >= 2 ? j - 1 : 1][j] * G.lo[j] : G.lo[j];   // T^(k)_0 = 1
                T g_add = T(0);
#pragma unroll
                for (int k = j + 1; k <= N; ++k) {
                    const T tp = j >= 2 ? Hn[j >= 2 ? j - 1 : 1][k] * rk[k - j + 1] : rk[k - j + 1];
                    contrib = fma_t(tp, Dc[k], contrib);
                    g_add += Dc[k];
                }
                if (j >= 2) {
#pragma unroll
                    for (int k = N; k >= j + 1; --k) Dc[k] = Dc[k] * (zc[j] * rk[k - j + 1]);
                    Dc[j] = G.lo[j] * zc[j];
                }
                G.lo[j] += g_add;
#pragma unroll
                for (int c = 0; c < D; ++c) dz[c] += cl[j] == c ? contrib : T(0);
            }

            // ---- this thread's (wavefront's) part of the increment's gradient
            if constexpr (TS::kWide) {
                // the wavefronts do not wait for one another inside a tile: their sums meet in LDS at its end
#pragma unroll
                for (int c = 0; c < D; ++c) {
                    const T total = group_sum<0, 6, T>(live ? dz[c] : T(0));
                    if ((tid & 63) == c) part[(i * 4 + (tid >> 6)) * D + c] = total;
                }
            } else {
                if (live) {
#pragma unroll
                    for (int c = 0; c < D; ++c) pp[s * D + c] = dz[c];
                }
            }

            if constexpr (STREAM) {
                if (s > 0 && live) {
                    if constexpr (!kAhead) G_ahead = load_share(go + (s - 1) * kS, true, true, true);
                    const Share &add = G_ahead;
#pragma unroll
                    for (int j = 1; j <= P; ++j) G.lo[j] += add.lo[j];
                    if constexpr (U >= 1) {
#pragma unroll
                        for (int c = 0; c < D; ++c) G.h1[c] += add.h1[c];
                    }
                    if constexpr (U >= 2) {
#pragma unroll
                        for (int c = 0; c < D * D; ++c) G.h2[c] += add.h2[c];
                    }
                }
            }
        }
        if constexpr (TS::kWide) {
            __syncthreads();
            for (int e = tid; e < PPG * nt * D; e += 256) {
                const int p = e / (nt * D), i = (e / D) % nt, c = e % D;
                if (row0 + p >= sh.B) continue;
                const T *q = part + (i * 4 + p * WPP) * D + c;
                T total = q[0];
#pragma unroll
                for (int w = 1; w < WPP; ++w) total += q[w * D];
                partial[(((row0 + p) * TS::kPartials + wg_group) * sh.n_inc + t0 + i) * D + c] = total;
            }
        }
    }
}

// gpath[row][point] = (sum of the partial gradients of the increment the point ends) - (of the one it starts);
// a basepoint only starts increment 0.
template <typename T, int D>
__global__ void __launch_bounds__(256)
sig_tree_backward_reduce_kernel(Shape sh, int64_t n_partials, const T *__restrict__ partial, T *__restrict__ gpath,
                                T *__restrict__ gbase)
{
    const int64_t per_row = (sh.n_inc + 1) * D;   // one extra "increment" -1 / n_inc at the ends
    const int64_t total = sh.B * per_row;
    for (int64_t e = blockIdx.x * int64_t(blockDim.x) + threadIdx.x; e < total; e += int64_t(gridDim.x) * blockDim.x) {
        const int64_t row = e / per_row, rem = e % per_row;
        const int64_t j = rem / D;   // output slot j: ends increment j-1, starts increment j
        const int c = int(rem % D);
        const T *pr = partial + row * n_partials * sh.n_inc * D;
        T ends = T(0), starts = T(0);
        for (int64_t g = 0; g < n_partials; ++g) {
            if (j >= 1) ends += pr[(g * sh.n_inc + (j - 1)) * D + c];
            if (j < sh.n_inc) starts += pr[(g * sh.n_inc + j) * D + c];
        }
        const T v = ends - starts;
        if (sh.basepoint) {
            // slot 0 is the basepoint, slot j >= 1 the point j-1
            if (j == 0) {
                if (gbase != nullptr) gbase[row * D + c] = v;
            } else {
                gpath[(row * sh.L + (j - 1)) * D + c] = v;
            }
        } else {
            gpath[(row * sh.L + j) * D + c] = v;
        }
    }
}

template <typename T, int D, int N>
hipError_t launch_tb_dn(const Shape &sh, const T *path, const T *sig, const T *gout, T *gpath,
                        T *gbase, T *partial, hipStream_t st)
{
    using TS = TbShape<D, N>;
    const int64_t groups = TS::kMulti ? sh.B * TS::kGroupsPerPath : (sh.B + TS::kPathsPerGroup - 1) / TS::kPathsPerGroup;
    if (groups > 0x7fffffff) return hipErrorNotSupported;
    if (sh.stream)
        hipLaunchKernelGGL((sig_tree_backward_kernel<T, D, N, true>), dim3(unsigned(groups)), dim3(256), 0, st, sh, path, sig,
                           gout, partial);
    else
        hipLaunchKernelGGL((sig_tree_backward_kernel<T, D, N, false>), dim3(unsigned(groups)), dim3(256), 0, st, sh, path, sig,
                           gout, partial);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    const int64_t total = sh.B * (sh.n_inc + 1) * D;
    const unsigned grid = unsigned((total + 255) / 256 < 65536 ? (total + 255) / 256 : 65536);
    hipLaunchKernelGGL((sig_tree_backward_reduce_kernel<T, D>), dim3(grid), dim3(256), 0, st, sh, TS::kPartials, partial, gpath,
                       gbase);
    return hipGetLastError();
}

template <int D, int N>
int64_t tb_partials() { return TbShape<D, N>::kPartials; }

constexpr int kTbMaxDepth = 9;       // d = 2..8
constexpr int kTbWideMaxDepth = 6;   // d = 9..16

template <int D>
int64_t tb_partials_d(int N)
{
    switch (N) {
        case 2: return tb_partials<D, 2>();
        case 3: return tb_partials<D, 3>();
        case 4: return tb_partials<D, 4>();
        case 5: return tb_partials<D, 5>();
        case 6: return tb_partials<D, 6>();
    }
    if constexpr (D <= 8) {
        switch (N) {
            case 7: return tb_partials<D, 7>();
            case 8: return tb_partials<D, 8>();
            case 9: return tb_partials<D, 9>();
        }
    }
    return -1;
}

template <typename T, int D>
hipError_t launch_tb_d(const Shape &sh, const T *path, const T *sig, const T *gout, T *gpath, T *gbase,
                       T *partial, hipStream_t st)
{
    switch (sh.N) {
        case 2: return launch_tb_dn<T, D, 2>(sh, path, sig, gout, gpath, gbase, partial, st);
        case 3: return launch_tb_dn<T, D, 3>(sh, path, sig, gout, gpath, gbase, partial, st);
        case 4: return launch_tb_dn<T, D, 4>(sh, path, sig, gout, gpath, gbase, partial, st);
        case 5: return launch_tb_dn<T, D, 5>(sh, path, sig, gout, gpath, gbase, partial, st);
        case 6: return launch_tb_dn<T, D, 6>(sh, path, sig, gout, gpath, gbase, partial, st);
    }
    if constexpr (D <= 8) {
        switch (sh.N) {
            case 7: return launch_tb_dn<T, D, 7>(sh, path, sig, gout, gpath, gbase, partial, st);
            case 8: return launch_tb_dn<T, D, 8>(sh, path, sig, gout, gpath, gbase, partial, st);
            case 9: return launch_tb_dn<T, D, 9>(sh, path, sig, gout, gpath, gbase, partial, st);
        }
    }
    return hipErrorNotSupported;
}


// Bytes of partial gradients for this shape with elements of `elem` bytes; -1 if the family does not serve it.
inline int64_t tb_workspace_bytes(const Shape &sh, int64_t elem)
{
    if (sh.d < 2 || sh.d > 16 || sh.N < 2 || sh.N > (sh.d <= 8 ? kTbMaxDepth : kTbWideMaxDepth) || sh.S >= (int64_t(1) << 31))
        return -1;
    int64_t partials = -1;
    switch (sh.d) {
        case 2: partials = tb_partials_d<2>(sh.N); break;
        case 3: partials = tb_partials_d<3>(sh.N); break;
        case 4: partials = tb_partials_d<4>(sh.N); break;
        case 5: partials = tb_partials_d<5>(sh.N); break;
        case 6: partials = tb_partials_d<6>(sh.N); break;
        case 7: partials = tb_partials_d<7>(sh.N); break;
        case 8: partials = tb_partials_d<8>(sh.N); break;
        case 9: partials = tb_partials_d<9>(sh.N); break;
        case 10: partials = tb_partials_d<10>(sh.N); break;
        case 11: partials = tb_partials_d<11>(sh.N); break;
        case 12: partials = tb_partials_d<12>(sh.N); break;
        case 13: partials = tb_partials_d<13>(sh.N); break;
        case 14: partials = tb_partials_d<14>(sh.N); break;
        case 15: partials = tb_partials_d<15>(sh.N); break;
        case 16: partials = tb_partials_d<16>(sh.N); break;
    }
    if (partials < 0) return -1;
    return sh.B * partials * sh.n_inc * sh.d * elem;
}

// WIDE: the translation unit that instantiates d = 9..16; the other one instantiates d = 2..8 and hands wider calls on.
template <typename T, bool WIDE>
hipError_t launch_tb(const Shape &sh, const T *path, const T *sig, const T *gout, T *gpath, T *gbase, void *workspace,
                     int64_t workspace_bytes, hipStream_t st)
{
    const int64_t need = tb_workspace_bytes(sh, int64_t(sizeof(T)));
    if (need < 0) return hipErrorNotSupported;
    if (workspace == nullptr || workspace_bytes < need) return hipErrorInvalidValue;
    T *partial = static_cast<T *>(workspace);
    if constexpr (WIDE) {
        switch (sh.d) {
            case 9: return launch_tb_d<T, 9>(sh, path, sig, gout, gpath, gbase, partial, st);
            case 10: return launch_tb_d<T, 10>(sh, path, sig, gout, gpath, gbase, partial, st);
            case 11: return launch_tb_d<T, 11>(sh, path, sig, gout, gpath, gbase, partial, st);
            case 12: return launch_tb_d<T, 12>(sh, path, sig, gout, gpath, gbase, partial, st);
            case 13: return launch_tb_d<T, 13>(sh, path, sig, gout, gpath, gbase, partial, st);
            case 14: return launch_tb_d<T, 14>(sh, path, sig, gout, gpath, gbase, partial, st);
            case 15: return launch_tb_d<T, 15>(sh, path, sig, gout, gpath, gbase, partial, st);
            case 16: return launch_tb_d<T, 16>(sh, path, sig, gout, gpath, gbase, partial, st);
        }
    } else {
        if (sh.d > 8) return launch_tree_backward_wide(sh, path, sig, gout, gpath, gbase, workspace, workspace_bytes, st);
        switch (sh.d) {
            case 2: return launch_tb_d<T, 2>(sh, path, sig, gout, gpath, gbase, partial, st);
            case 3: return launch_tb_d<T, 3>(sh, path, sig, gout, gpath, gbase, partial, st);
            case 4: return launch_tb_d<T, 4>(sh, path, sig, gout, gpath, gbase, partial, st);
            case 5: return launch_tb_d<T, 5>(sh, path, sig, gout, gpath, gbase, partial, st);
            case 6: return launch_tb_d<T, 6>(sh, path, sig, gout, gpath, gbase, partial, st);
            case 7: return launch_tb_d<T, 7>(sh, path, sig, gout, gpath, gbase, partial, st);
            case 8: return launch_tb_d<T, 8>(sh, path, sig, gout, gpath, gbase, partial, st);
        }
    }
    return hipErrorNotSupported;
}

}  // namespace
}  // namespace sig

#endif  // SIG_TREE_BACKWARD_IMPL_H_
