// Small-state kernel family: signatures of at most 512 scalars (e.g. d = 2 up to depth 8, d = 3 up
// to depth 5, any d at depth 1 or 2 while S <= 512), fp32 or fp64, final and stream mode.
//
// One wavefront scans one path; the state lives in LDS and every lane owns up to 8 words of it.
// The fused multiply-exponentiate (paper section 4.1, eq. "fusedterm") is applied element-wise:
// the new coefficient of a word w = w_1..w_k is the end of the scalar Horner chain
//     u_1 = z[w_1]/k + A_1[w_1],  u_i = u_{i-1} * z[w_i]/(k-i+1) + A_i[w_1..w_i],  A_k[w] <- u_k
// over the prefixes of w.  Which prefixes and letters a lane needs never changes, so they are
// decoded once, before the scan, into registers; a step is then a handful of LDS reads and FMAs.
// All words are updated at once from the old state: read everything, barrier, write back.
#include "sig_internal.h"

namespace sig {
namespace {

constexpr int kSmallMaxWords = 512;   // S this family accepts
constexpr int kSmallWordsPerLane = 8;
constexpr int kSmallTile = 64;        // increments staged in LDS at a time

template <typename T, int N>
__global__ void __launch_bounds__(64)
sig_small_kernel(Shape sh, const T *__restrict__ path, T *__restrict__ out)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    T *st = reinterpret_cast<T *>(smem_raw);          // state, S scalars (padded to kSmallMaxWords)
    T *zs = st + kSmallMaxWords;                      // zs[(m-1)*d + c] = z[c]/m for the current increment
    T *inc = zs + N * sh.d;                           // staged increments [kSmallTile][d]

    const int lane = threadIdx.x;
    const int d = sh.d;
    const int S = int(sh.S);

    // decode this lane's words once: level, letters and prefix offsets
    int level[kSmallWordsPerLane];
    int where[kSmallWordsPerLane][N];  // where[j][i-1] = (offset of the i-letter prefix) << 8 | (i-th letter)
#pragma unroll
    for (int j = 0; j < kSmallWordsPerLane; ++j) {
        const int wi = lane + 64 * j;
        level[j] = 0;
#pragma unroll
        for (int i = 0; i < N; ++i) where[j][i] = 0;
        if (wi < S) {
            int k = 1;
            while (k < N && wi >= int(sh.off[k + 1])) ++k;
            level[j] = k;
            int idx = wi - int(sh.off[k]);  // index inside level k
#pragma unroll
            for (int i = N; i >= 1; --i) {
                if (i <= k) {
                    where[j][i - 1] = ((int(sh.off[i]) + idx) << 8) | (idx % d);
                    idx /= d;
                }
            }
        }
    }

    for (int64_t b = blockIdx.x; b < sh.B; b += gridDim.x) {
        const T *x = path + b * sh.L * d;
        T *o = out + b * (sh.stream ? sh.n_inc * int64_t(S) : int64_t(S));
        for (int i = lane; i < S; i += 64) st[i] = T(0);

        for (int64_t t0 = 0; t0 < sh.n_inc; t0 += kSmallTile) {
            const int nt = int(sh.n_inc - t0 < kSmallTile ? sh.n_inc - t0 : kSmallTile);
            __syncthreads();
            for (int i = lane; i < nt * d; i += 64) {
                const int64_t s = t0 + i / d;
                const int c = i % d;
                T hi, lo;
                if (sh.basepoint) {
                    hi = x[s * d + c];
                    lo = s == 0 ? T(0) : x[(s - 1) * d + c];
                } else {
                    hi = x[(s + 1) * d + c];
                    lo = x[s * d + c];
                }
                inc[i] = hi - lo;
            }
            __syncthreads();
            for (int s = 0; s < nt; ++s) {
                for (int i = lane; i < N * d; i += 64) {
                    const int m = i / d + 1;
                    zs[i] = inc[s * d + (i - (m - 1) * d)] / T(m);
                }
                __syncthreads();
                T fresh[kSmallWordsPerLane];
#pragma unroll
                for (int j = 0; j < kSmallWordsPerLane; ++j) {
                    const int k = level[j];
                    T u = T(0);
#pragma unroll
                    for (int i = 1; i <= N; ++i) {
                        if (i <= k) {
                            const int wd = where[j][i - 1];
                            const T zi = zs[(k - i) * d + (wd & 255)];   // z[w_i] / (k - i + 1)
                            const T a = st[wd >> 8];
                            u = i == 1 ? zi + a : u * zi + a;
                        }
                    }
                    fresh[j] = u;
                }
                __syncthreads();
#pragma unroll
                for (int j = 0; j < kSmallWordsPerLane; ++j) {
                    const int wi = lane + 64 * j;
                    if (wi < S) {
                        st[wi] = fresh[j];
                        if (sh.stream) o[(t0 + s) * S + wi] = fresh[j];
                    }
                }
                // the next step's zs and reads come after the barrier at the top of that step
            }
        }
        __syncthreads();
        if (!sh.stream)
            for (int i = lane; i < S; i += 64) o[i] = st[i];
        __syncthreads();
    }
}

template <typename T, int N>
hipError_t launch_small_n(const Shape &sh, const T *path, T *out, hipStream_t st)
{
    const size_t lds = sizeof(T) * (size_t(kSmallMaxWords) + size_t(N) * size_t(sh.d) + size_t(kSmallTile) * size_t(sh.d));
    const int64_t max_grid = 1 << 20;
    const unsigned grid = unsigned(sh.B < max_grid ? sh.B : max_grid);
    hipLaunchKernelGGL((sig_small_kernel<T, N>), dim3(grid), dim3(64), lds, st, sh, path, out);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_small(const Shape &sh, const T *path, T *out, hipStream_t st)
{
    switch (sh.N) {
        case 1: return launch_small_n<T, 1>(sh, path, out, st);
        case 2: return launch_small_n<T, 2>(sh, path, out, st);
        case 3: return launch_small_n<T, 3>(sh, path, out, st);
        case 4: return launch_small_n<T, 4>(sh, path, out, st);
        case 5: return launch_small_n<T, 5>(sh, path, out, st);
        case 6: return launch_small_n<T, 6>(sh, path, out, st);
        case 7: return launch_small_n<T, 7>(sh, path, out, st);
        case 8: return launch_small_n<T, 8>(sh, path, out, st);
    }
    return hipErrorNotSupported;
}

}  // namespace

bool small_supported(const Shape &sh)
{
    // letters are packed into 8 bits; the state, the per-step scalings and one tile of increments
    // (at most (512 + 8*64 + 64*64) scalars) must fit the 64 KB of LDS a workgroup gets by default
    return sh.S <= kSmallMaxWords && sh.N <= 8 && sh.d <= 64;
}

hipError_t launch_small_f32(const Shape &sh, const float *path, float *out, hipStream_t st)
{
    return small_supported(sh) ? launch_small<float>(sh, path, out, st) : hipErrorNotSupported;
}

hipError_t launch_small_f64(const Shape &sh, const double *path, double *out, hipStream_t st)
{
    return small_supported(sh) ? launch_small<double>(sh, path, out, st) : hipErrorNotSupported;
}

}  // namespace sig
