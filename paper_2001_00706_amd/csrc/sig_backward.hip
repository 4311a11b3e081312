// Gradient of the signature with respect to the path (paper section 5.3, appendix C): any d <= 64, any
// N, fp32 or fp64, final and stream mode.  One workgroup scans one path backwards.
//
// Forward, one increment z takes the state A to A' by the fused multiply-exponentiate (section 4.1,
// eq. "fusedterm"): for every level k,
//     T^(k)_0 = 1,   T^(k)_i = T^(k)_{i-1} (x) z/(k-i+1) + A_i   (i < k),   A'_k = T^(k)_{k-1} (x) z + A_k.
// Backward, per increment (last one first), with G = d(loss)/dA':
//   up    for i = 1..N: A_i = A'_i - T^(i)_{i-1} (x) z, then T^(k)_i for every k > i from it.  This undoes the
//         forward step exactly and yields, in the same pass, the state before the increment (appendix C.1
//         recovers it as A' [x] exp(-z); subtracting what the forward step added is the same map with the
//         Horner terms as a by-product) and every Horner term the product rule needs.  Nothing from the
//         forward pass is stored (appendix C.1, reversibility).  In stream mode the earlier state is simply
//         the previous entry of the forward output and nothing is undone.
//   down  D^(k)_k = G_k; for i = N..1 and every chain k >= i:
//             dz[c]          += T^(k)_{i-1}[p] * D^(k)_i[p c] / (k-i+1)            (gradient of the increment)
//             D^(k)_{i-1}[p]  = sum_c D^(k)_i[p c] * z[c] / (k-i+1)                (cotangent of T^(k)_{i-1})
//             dA_i            = G_i + sum_{k > i} D^(k)_i                          (cotangent of the old state)
//         which is the transpose of the forward recurrences line by line.
// The gradient of point x_j is dz of the increment it ends minus dz of the increment it starts.
//
// Every sum is taken in a fixed order (no atomics): results are deterministic.
#include "sig_internal.h"

namespace sig {
namespace {

constexpr int64_t kBackwardMaxGrid = 1024;      // persistent workgroups when the arena lives in global memory
constexpr size_t kLdsDefaultLimit = 64 * 1024;  // dynamic LDS a kernel may use without asking for more

// Per-workgroup arena, in elements: the state A (final mode only), its cotangent G, the Horner terms
// T^(k)_i (k > i: N-i arrays of d^i at tbase[i]) and two buffers for the chains D^(k)_i.
struct BackwardPlan {
    int tbase[SIG_MAX_DEPTH + 1];
    int a_off, g_off, t_off, d0_off, d1_off;
    int big_elems;     // A + G + T + 2 D
    int small_elems;   // scaled increments, reciprocals, two increment gradients, one partial sum per thread
};

template <typename T, int NT, bool kLds>
__global__ void __launch_bounds__(NT)
sig_backward_kernel(Shape sh, BackwardPlan pl, const T *__restrict__ path, const T *__restrict__ sig,
                    const T *__restrict__ gout, T *__restrict__ gpath, T *__restrict__ gbase, T *__restrict__ ws)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int d = sh.d, N = sh.N, S = int(sh.S);
    const int tid = threadIdx.x;

    T *zs = reinterpret_cast<T *>(smem_raw);   // zs[(m-1)*d + c] = z[c]/m
    T *rc = zs + N * d;                        // rc[m] = 1/m
    T *dzv = rc + (N + 1);                     // dzv[c]: gradient of this increment; dzv[d+c]: of the one after it
    T *zraw = dzv + 2 * d;                     // the increment itself
    T *red = zraw + d;                         // one partial sum per thread
    T *big;
    if constexpr (kLds)
        big = red + NT;
    else
        big = ws + int64_t(blockIdx.x) * pl.big_elems;
    T *A = big + pl.a_off;
    T *G = big + pl.g_off;
    T *Tt = big + pl.t_off;

    // thread t handles the words q = t, t + NT, ...: their last letter and the index of the rest advance by
    // fixed amounts, so no division is needed inside the loops
    const int c0 = tid % d, p0 = tid / d;
    const int step_c = NT % d, step_p = NT / d;
    // for the per-letter sums only the first NS threads work, with stride NS, so that a thread keeps its letter
    const int NS = (NT / d) * d;

    for (int64_t b = blockIdx.x; b < sh.B; b += gridDim.x) {
        const T *x = path + b * sh.L * d;
        const T *bpv = static_cast<const T *>(sh.basepoint_value);
        T *gp = gpath + b * sh.L * d;
        const int64_t per_path = sh.stream ? sh.n_inc * int64_t(S) : int64_t(S);
        const T *sg = sig + b * per_path;
        const T *go = gout + b * per_path;

        for (int i = tid; i < S; i += NT) {
            G[i] = sh.stream ? go[(sh.n_inc - 1) * S + i] : go[i];
            if (!sh.stream) A[i] = sg[i];
        }
        if (tid <= N) rc[tid] = tid > 0 ? T(1) / T(tid) : T(0);
        if (tid < d) dzv[d + tid] = T(0);

        // component tid of increment s (threads below d), fetched one step ahead
        auto fetch = [&](int64_t s) -> T {
            if (tid >= d || s < 0) return T(0);
            const int64_t hi = sh.basepoint ? s : s + 1;
            const T lo = hi > 0 ? x[(hi - 1) * d + tid] : bpv != nullptr ? bpv[b * d + tid] : T(0);
            return x[hi * d + tid] - lo;
        };
        T z_next = fetch(sh.n_inc - 1);

        for (int64_t s = sh.n_inc - 1; s >= 0; --s) {
            if (tid < d) zraw[tid] = z_next;
            z_next = fetch(s - 1);
            __syncthreads();
            {
                int m1 = p0, c = c0;   // entry i = (m-1)*d + c
                for (int i = tid; i < N * d; i += NT) {
                    zs[i] = zraw[c] / T(m1 + 1);
                    c += step_c;
                    m1 += step_p;
                    if (c >= d) {
                        c -= d;
                        ++m1;
                    }
                }
            }
            __syncthreads();

            // ---- up: the state before this increment and the Horner terms
            const T *Ap = sg + (s > 0 ? s - 1 : 0) * int64_t(S);   // stream mode, s > 0: signature after s increments
            for (int i = 1; i <= N; ++i) {
                const int n_i = int(sh.pw[i]), n_p = int(sh.pw[i - 1]), off_i = int(sh.off[i]);
                T *Ti = Tt + pl.tbase[i];
                const T *Tp = Tt + pl.tbase[i - 1];
                int p = p0, c = c0;
                for (int q = tid; q < n_i; q += NT) {
                    T a;
                    if (sh.stream) {
                        a = s > 0 ? Ap[off_i + q] : T(0);
                    } else {
                        a = A[off_i + q] - (i == 1 ? T(1) : Tp[p]) * zs[c];
                        A[off_i + q] = a;
                    }
                    for (int k = i + 1; k <= N; ++k) {
                        const T tp = i == 1 ? T(1) : Tp[(k - i) * n_p + p];
                        Ti[(k - i - 1) * n_i + q] = tp * zs[(k - i) * d + c] + a;
                    }
                    c += step_c;
                    p += step_p;
                    if (c >= d) {
                        c -= d;
                        ++p;
                    }
                }
                __syncthreads();
            }

            // ---- down: cotangents of the Horner terms, of the increment and of the earlier state
            T *Dc = big + pl.d0_off, *Dn = big + pl.d1_off;
            T dz_acc = T(0);
            for (int i = N; i >= 1; --i) {
                const int n_i = int(sh.pw[i]), n_p = int(sh.pw[i - 1]), off_i = int(sh.off[i]);
                const T *Tp = Tt + pl.tbase[i - 1];
                // chains contracted with the increment: D^(k)_{i-1}, k = i..N
                if (i >= 2) {
                    for (int p = tid; p < n_p; p += NT) {
                        for (int k = i; k <= N; ++k) {
                            const T *src = k == i ? G + off_i : Dc + (k - i - 1) * n_i;
                            const T *zk = zs + (k - i) * d;
                            T acc = T(0);
                            for (int c = 0; c < d; ++c) acc += src[p * d + c] * zk[c];
                            Dn[(k - i) * n_p + p] = acc;
                        }
                    }
                    __syncthreads();
                }
                // gradient of the increment, and the cotangent of level i of the earlier state
                if (tid < NS) {
                    int p = p0;
                    for (int q = tid; q < n_i; q += NS) {
                        const T g = G[off_i + q];
                        T acc = (i == 1 ? T(1) : Tp[p]) * g;     // chain k = i, divisor 1
                        T h = g;
                        for (int k = i + 1; k <= N; ++k) {
                            const T val = Dc[(k - i - 1) * n_i + q];
                            const T tp = i == 1 ? T(1) : Tp[(k - i) * n_p + p];
                            acc += rc[k - i + 1] * tp * val;
                            h += val;
                        }
                        dz_acc += acc;
                        G[off_i + q] = h;
                        p += NS / d;
                    }
                }
                __syncthreads();
                T *t = Dc;
                Dc = Dn;
                Dn = t;
            }

            // ---- gradient of this increment: sum over the threads that share a letter, in a fixed order
            red[tid] = tid < NS ? dz_acc : T(0);
            __syncthreads();
            if (tid < d) {
                T sum = T(0);
                for (int j = tid; j < NS; j += d) sum += red[j];
                // the point above this increment ends it and starts the next one
                const int64_t point = sh.basepoint ? s : s + 1;
                gp[point * d + tid] = sum - dzv[d + tid];
                dzv[d + tid] = sum;
            }
            // stream mode: the signature after s increments is output entry s-1
            if (sh.stream && s > 0)
                for (int i = tid; i < S; i += NT) G[i] += go[(s - 1) * int64_t(S) + i];
            __syncthreads();
        }
        // the first point only starts increment 0 (with a basepoint it was written above: it ends increment 0)
        if (!sh.basepoint && tid < d) gp[tid] = -dzv[d + tid];
        // a basepoint only starts increment 0
        if (sh.basepoint && gbase != nullptr && tid < d) gbase[b * d + tid] = -dzv[d + tid];
        __syncthreads();
    }
}

// Arena layout for a shape; false if an index would not fit 31 bits.
bool make_plan(const Shape &sh, int threads, BackwardPlan &pl)
{
    const int64_t cap = int64_t(1) << 30;
    if (sh.S >= cap) return false;
    int64_t t = 0, dmax = 1;
    for (int i = 0; i <= SIG_MAX_DEPTH; ++i) pl.tbase[i] = 0;
    for (int i = 1; i <= sh.N - 1; ++i) {
        pl.tbase[i] = int(t);
        t += int64_t(sh.N - i) * sh.pw[i];
        if (t >= cap) return false;
    }
    // stage i writes the chains k = i..N at level i-1
    for (int i = 2; i <= sh.N; ++i) {
        const int64_t need = int64_t(sh.N - i + 1) * sh.pw[i - 1];
        if (need > dmax) dmax = need;
    }
    int64_t off = 0;
    pl.a_off = int(off);
    if (!sh.stream) off += sh.S;
    pl.g_off = int(off);
    off += sh.S;
    pl.t_off = int(off);
    off += t;
    pl.d0_off = int(off);
    off += dmax;
    pl.d1_off = int(off);
    off += dmax;
    if (off >= cap) return false;
    pl.big_elems = int(off);
    pl.small_elems = sh.N * sh.d + (sh.N + 1) + 3 * sh.d + threads;
    return true;
}

// Threads per workgroup.  (A single wavefront per path, which needs no hardware barriers, was measured too: twice
// as slow on 1024 paths of d = 4, N = 6, since nothing hides the LDS latency of the one wavefront.)
constexpr int kBackwardThreads = 256;

// Most dynamic LDS one workgroup may have on this device (0 if the query fails).
size_t lds_limit()
{
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess) return 0;
    return v > 0 ? size_t(v) : 0;
}

template <typename T>
bool fits_lds(const BackwardPlan &pl)
{
    return (size_t(pl.small_elems) + size_t(pl.big_elems)) * sizeof(T) <= lds_limit();
}

template <typename T, int NT>
hipError_t launch_backward_nt(const Shape &sh, const BackwardPlan &pl, const T *path, const T *sig, const T *gout,
                              T *gpath, T *gbase, void *workspace, int64_t workspace_bytes, hipStream_t st)
{
    if (fits_lds<T>(pl)) {
        const size_t lds = (size_t(pl.small_elems) + size_t(pl.big_elems)) * sizeof(T);
        auto kernel = sig_backward_kernel<T, NT, true>;
        if (lds > kLdsDefaultLimit) {
            const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, int(lds));
            if (e != hipSuccess) return e;
        }
        const unsigned grid = unsigned(sh.B < (int64_t(1) << 20) ? sh.B : (int64_t(1) << 20));
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(NT), lds, st, sh, pl, path, sig, gout, gpath, gbase,
                           static_cast<T *>(nullptr));
        return hipGetLastError();
    }
    const int64_t grid = sh.B < kBackwardMaxGrid ? sh.B : kBackwardMaxGrid;
    if (workspace == nullptr || workspace_bytes < grid * int64_t(pl.big_elems) * int64_t(sizeof(T)))
        return hipErrorInvalidValue;
    const size_t lds = size_t(pl.small_elems) * sizeof(T);
    hipLaunchKernelGGL((sig_backward_kernel<T, NT, false>), dim3(unsigned(grid)), dim3(NT), lds, st, sh, pl, path, sig,
                       gout, gpath, gbase, static_cast<T *>(workspace));
    return hipGetLastError();
}

template <typename T>
hipError_t launch_backward(const Shape &sh, const T *path, const T *sig, const T *gout, T *gpath, T *gbase,
                           void *workspace, int64_t workspace_bytes, hipStream_t st)
{
    BackwardPlan pl;
    if (!backward_supported(sh) || !make_plan(sh, kBackwardThreads, pl)) return hipErrorNotSupported;
    return launch_backward_nt<T, kBackwardThreads>(sh, pl, path, sig, gout, gpath, gbase, workspace, workspace_bytes, st);
}

}  // namespace

bool backward_supported(const Shape &sh)
{
    BackwardPlan pl;
    // a thread keeps one letter in the per-letter sums; the limit leaves room for a one-wavefront workgroup
    return sh.d <= 64 && make_plan(sh, kBackwardThreads, pl);
}

// Final mode at depths 3 to 6 from 9 channels on, where the prefix-tree kernels also keep one level per thread: the
// kernel for many channels is ahead from 12 channels on (128 points, N = 3, d = 16: 98 us against 274 at 32 paths, 183
// against 336 at 1024; d = 12, N = 4: 144 against 261 and 1260 against 1500) and below 256 paths from 9 on (d = 9,
// N = 3: 128 against 167 at 32 paths, 204 against 176 at 1024).  d = 16, N = 4 has a kernel of its own.
bool wide_backward_preferred(const Shape &sh, sig_dtype dtype)
{
    if (sh.N == 5 || sh.N == 6)   // d = 16: 1.4 to 1.65 times the prefix-tree kernels, d = 12: 1.0 to 1.15, d = 9: 0.6 to 0.7
        return !sh.stream && sh.d >= 13 && sh.d <= 16 && wide_backward_supported(sh, dtype);
    return !sh.stream && (sh.N == 3 || sh.N == 4) && sh.d >= 9 && sh.d <= 16 && (sh.d >= 12 || sh.B < 256) &&
           !(sh.d == 16 && sh.N == 4) && wide_backward_supported(sh, dtype);
}

int64_t backward_workspace_bytes(const Shape &sh, sig_dtype dtype)
{
    // signatures of up to 8 channels and depth 9 never reach the generic kernel
    if (backward_n2_supported(sh, dtype)) return 0;   // depth 2 in final mode: a closed form, nothing to keep
    if (wide_backward_preferred(sh, dtype)) return wide_backward_workspace_bytes(sh, dtype);
    if (tree_backward_supported(sh)) return tree_backward_workspace_bytes(sh, dtype);
    if (wide_backward_supported(sh, dtype)) return wide_backward_workspace_bytes(sh, dtype);   // beyond 16 channels
    BackwardPlan pl;
    if (!backward_supported(sh) || !make_plan(sh, kBackwardThreads, pl)) return -1;
    const bool lds = dtype == SIG_F32 ? fits_lds<float>(pl) : fits_lds<double>(pl);
    if (lds) return 0;
    const int64_t grid = sh.B < kBackwardMaxGrid ? sh.B : kBackwardMaxGrid;
    return grid * int64_t(pl.big_elems) * int64_t(dtype == SIG_F32 ? sizeof(float) : sizeof(double));
}

hipError_t launch_backward_f32(const Shape &sh, const float *path, const float *sig, const float *gout, float *gpath,
                               float *gbase, void *workspace, int64_t workspace_bytes, hipStream_t st)
{
    // depth 2 in final mode: the closed form, from 8 channels on as a product on the matrix cores (1024 paths of 128
    // points: d = 16: 14.5 us against 24, d = 64: 50 against 192, d = 100: 136 against 665)
    if (backward_n2_mfma_supported(sh)) return launch_backward_n2_mfma_f32(sh, path, gout, gpath, gbase, st);
    if (backward_n2_supported(sh, SIG_F32)) return launch_backward_n2_f32(sh, path, gout, gpath, gbase, st);
    const bool aligned = (reinterpret_cast<uintptr_t>(path) | reinterpret_cast<uintptr_t>(sig) |
                          reinterpret_cast<uintptr_t>(gout) | reinterpret_cast<uintptr_t>(sh.basepoint_value)) % 16 == 0;
    // Measured at L = 128 over B = 1..2048: with one gradient per path (final mode) the prefix-tree kernels beat the
    // two register-resident families (by up to 3.6 times at d = 8) except at d = 4, N >= 5 below 512 paths; with a
    // gradient per prefix (stream mode) the register-resident families stay ahead.
    // d = 4, N = 6 in final mode: the top level's cotangent in registers, two wavefronts per path (105 us against 172
    // on the prefix-tree kernels at 1024 paths of 128 points, 77 against 95 on the register-resident family at 32)
    const bool ws_aligned = workspace != nullptr && reinterpret_cast<uintptr_t>(workspace) % 16 == 0;
    if (aligned && ws_aligned && backward_d4n6_supported(sh) && workspace_bytes >= backward_d4n6_workspace_bytes(sh))
        return launch_backward_d4n6_f32(sh, path, sig, gout, gpath, gbase, workspace, workspace_bytes, st);
    const bool tree_first = !sh.stream && tree_backward_supported(sh) && !(sh.d == 4 && sh.N >= 5 && sh.B < 512);
    if (aligned && !tree_first && backward_d4_supported(sh))
        return launch_backward_d4_f32(sh, path, sig, gout, gpath, gbase, st);
    if (aligned && !tree_first && backward_pow2_supported(sh))
        return launch_backward_pow2_f32(sh, path, sig, gout, gpath, gbase, st);
    // d = 16, N = 4 (10 ms on the prefix-tree kernels at 256 paths of 1024 points); its workspace is a sixteenth of
    // theirs, which is what sig_backward_workspace_bytes reports for the shape
    if (aligned && backward_d16_supported(sh) && workspace != nullptr && workspace_bytes >= backward_d16_workspace_bytes(sh) &&
        reinterpret_cast<uintptr_t>(workspace) % 16 == 0)
        return launch_backward_d16_f32(sh, path, sig, gout, gpath, gbase, workspace, workspace_bytes, st);
    if (wide_backward_preferred(sh, SIG_F32))
        return launch_wide_backward_f32(sh, path, sig, gout, gpath, gbase, workspace, workspace_bytes, st);
    if (tree_backward_supported(sh))
        return launch_tree_backward_f32(sh, path, sig, gout, gpath, gbase, workspace, workspace_bytes, st);
    if (wide_backward_supported(sh, SIG_F32))
        return launch_wide_backward_f32(sh, path, sig, gout, gpath, gbase, workspace, workspace_bytes, st);
    return launch_backward<float>(sh, path, sig, gout, gpath, gbase, workspace, workspace_bytes, st);
}

hipError_t launch_backward_f64(const Shape &sh, const double *path, const double *sig, const double *gout, double *gpath,
                               double *gbase, void *workspace, int64_t workspace_bytes, hipStream_t st)
{
    if (backward_n2_supported(sh, SIG_F64)) return launch_backward_n2_f64(sh, path, gout, gpath, gbase, st);
    if (wide_backward_preferred(sh, SIG_F64))
        return launch_wide_backward_f64(sh, path, sig, gout, gpath, gbase, workspace, workspace_bytes, st);
    if (tree_backward_supported(sh))
        return launch_tree_backward_f64(sh, path, sig, gout, gpath, gbase, workspace, workspace_bytes, st);
    if (wide_backward_supported(sh, SIG_F64))
        return launch_wide_backward_f64(sh, path, sig, gout, gpath, gbase, workspace, workspace_bytes, st);
    return launch_backward<double>(sh, path, sig, gout, gpath, gbase, workspace, workspace_bytes, st);
}

}  // namespace sig
