// Logarithm of signatures in the truncated tensor algebra and the logsignature in the basis of paper
// appendix A.2.4 (sections 2.3 and 4.3).
//
// log: with x the signature without its constant term,  log(1 + x) = sum_{m=1..N} c_m x^{[x] m},
// c_m = (-1)^{m+1} / m, evaluated by Horner's rule from the inside out:
//     R_N = c_N x,   R_m = c_m x + x [x] R_{m+1},   log = R_1.
// R_m is needed at levels 1..N-m+1 only (a product of m or more factors has no lower levels to feed), so
// the top level is computed once.  A product x [x] R reads strictly lower levels of R, so R is updated in
// place, levels highest first, with a workgroup barrier between levels; one workgroup per signature, with
// the signature and R in LDS when they fit (else in global memory, R in `out`).
//
// logsignature: psi(log(Sig)) is the vector of coefficients of the Lyndon words (appendix A.2.4): a gather
// with an index table that `sig_lyndon_indices` computes on the host.
#include "sig_internal.h"

#include <type_traits>
#include <vector>

namespace sig {
namespace {

// kLds: the signature and R are kept in LDS (2 S scalars) and R is copied out at the end; otherwise both stay in
// global memory (R in `out`).
// D: the channel count when it is one of the common ones (the letters of a word are then peeled off with
// divisions by a constant), 0 for any other d.
template <typename T, bool kLds, int D>
__global__ void __launch_bounds__(256)
sig_log_kernel(Shape sh, const T *__restrict__ in, T *__restrict__ out)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    __shared__ uint32_t off[SIG_MAX_DEPTH + 2];   // level offsets: indexed by loop variables, so not left in the kernel arguments
    const uint32_t d = D > 0 ? uint32_t(D) : uint32_t(sh.d);
    const int N = sh.N;
    if (threadIdx.x <= unsigned(N) + 1) off[threadIdx.x] = uint32_t(sh.off[threadIdx.x]);
    __syncthreads();
    for (int64_t r = blockIdx.x; r < sh.B; r += gridDim.x) {
        const T *x;
        T *R;
        if constexpr (kLds) {
            T *xs = reinterpret_cast<T *>(smem_raw);
            for (uint32_t i = threadIdx.x; i < uint32_t(sh.S); i += blockDim.x) xs[i] = in[r * sh.S + i];
            x = xs;
            R = xs + sh.S;
            __syncthreads();
        } else {
            x = in + r * sh.S;
            R = out + r * sh.S;
        }
        for (int m = N; m >= 1; --m) {
            const T c = (m & 1 ? T(1) : T(-1)) / T(m);
            for (int k = N - m + 1; k >= 1; --k) {
                const uint32_t off_k = off[k], n_k = off[k + 1] - off_k;
                for (uint32_t idx = threadIdx.x; idx < n_k; idx += blockDim.x) {
                    T acc = c * x[off_k + idx];
                    // splits of the word into a prefix of x (j letters) and a suffix of R (k - j letters)
                    uint32_t prefix = idx, suffix = 0, scale = 1;
                    for (int j = k - 1; j >= 1; --j) {
                        const uint32_t letter = prefix % d;
                        prefix /= d;
                        suffix += letter * scale;
                        scale *= d;
                        acc += x[off[j] + prefix] * R[off[k - j] + suffix];
                    }
                    R[off_k + idx] = acc;
                }
                __syncthreads();
            }
        }
        if constexpr (kLds) {
            for (uint32_t i = threadIdx.x; i < uint32_t(sh.S); i += blockDim.x) out[r * sh.S + i] = R[i];
            __syncthreads();
        }
    }
}

__host__ __device__ constexpr uint32_t fixed_off(int d, int k)   // offset of level k (1-based) for d channels
{
    uint32_t off = 0, p = 1;
    for (int j = 1; j < k; ++j) {
        p *= uint32_t(d);
        off += p;
    }
    return off;
}

// The same computation for a channel count and depth known at compile time, signature and R in LDS: every loop
// over passes, levels and splits is unrolled, so the offsets are constants, the letters come off with shifts or
// multiplications, and the operands of all splits of a word are fetched before any of them is used (the generic
// kernel above waits for two LDS round trips per split).
template <typename T, int D, int N>
__global__ void __launch_bounds__(256)
sig_log_fixed_kernel(int64_t rows, const T *__restrict__ in, T *__restrict__ out)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    constexpr uint32_t S = fixed_off(D, N + 1);
    T *x = reinterpret_cast<T *>(smem_raw);
    T *R = x + S;
    for (int64_t r = blockIdx.x; r < rows; r += gridDim.x) {
        for (uint32_t i = threadIdx.x; i < S; i += 256) x[i] = in[r * S + i];
        __syncthreads();
#pragma unroll
        for (int m = N; m >= 1; --m) {
            const T c = (m & 1 ? T(1) : T(-1)) / T(m);
#pragma unroll
            for (int k = N - m + 1; k >= 1; --k) {
                const uint32_t off_k = fixed_off(D, k), n_k = fixed_off(D, k + 1) - off_k;
                for (uint32_t idx = threadIdx.x; idx < n_k; idx += 256) {
                    T xv[N], rv[N];
                    uint32_t prefix = idx, suffix = 0, scale = 1;
#pragma unroll
                    for (int j = k - 1; j >= 1; --j) {
                        const uint32_t letter = prefix % uint32_t(D);
                        prefix /= uint32_t(D);
                        suffix += letter * scale;
                        scale *= uint32_t(D);
                        xv[j] = x[fixed_off(D, j) + prefix];
                        rv[j] = R[fixed_off(D, k - j) + suffix];
                    }
                    T acc = c * x[off_k + idx];
#pragma unroll
                    for (int j = k - 1; j >= 1; --j) acc += xv[j] * rv[j];
                    R[off_k + idx] = acc;
                }
                __syncthreads();
            }
        }
        for (uint32_t i = threadIdx.x; i < S; i += 256) out[r * S + i] = R[i];
        __syncthreads();
    }
}

// Depths up to 9 at any size, with no pass structure at all: one thread per word w of the result, which sums
// the power series term by term,
//     log(1 + x)[w] = sum_m c_m sum over the ways to cut w into m consecutive pieces of  prod x[piece],
// by dynamic programming over the cuts: P_m[j] = sum_{i < j} P_{m-1}[i] x[w_{i+1}..w_j] is the sum over the cuts
// of the first j letters into m pieces, P_0[0] = 1, and the result is sum_m c_m P_m[k].  A word of k letters
// reads the k(k+1)/2 coefficients of its sub-words (neighbouring threads share all but k of them) and spends
// about k^3/6 multiply-adds.  Nothing is written but the result, so signatures of any size spread over the
// whole chip without synchronisation.
constexpr int kDirectMaxDepth = 9;

template <int I, int End, typename F>
__device__ __forceinline__ void static_for(F &&f)   // f(integral_constant<int, I>), ..., f(integral_constant<int, End - 1>)
{
    if constexpr (I < End) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, End>(f);
    }
}

template <typename T, int D, int K>
__device__ __forceinline__ T log_of_word(const T *__restrict__ x, uint32_t idx, uint32_t d, const uint32_t (&off)[kDirectMaxDepth + 2])
{
    uint32_t w[K];   // letters, first to last
    {
        uint32_t rest = idx;
#pragma unroll
        for (int t = K - 1; t >= 0; --t) {
            w[t] = D > 0 ? rest % uint32_t(D) : rest % d;
            rest = D > 0 ? rest / uint32_t(D) : rest / d;
        }
    }
    // xs[at(i, j)] = x[w_{i+1}..w_j], 0 <= i < j <= K, packed.  Every index below is a compile-time constant
    // (static_for, not a loop the compiler may or may not unroll: at K = 9 it left some of them rolled, which put
    // this array in scratch memory and made the kernel 6 times slower), so the arrays live in registers.
    constexpr auto at = [](int i, int j) { return i * K - i * (i - 1) / 2 + (j - i - 1); };
    T xs[K * (K + 1) / 2];
    static_for<0, K>([&](auto ic) {
        constexpr int i = decltype(ic)::value;
        uint32_t val = 0;
        static_for<i + 1, K + 1>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            val = val * (D > 0 ? uint32_t(D) : d) + w[j - 1];
            xs[at(i, j)] = x[off[j - i] + val];
        });
    });
    // P_1[j] = x[w_1..w_j]; P_m[j] = sum_{m-1 <= i < j} P_{m-1}[i] x[w_{i+1}..w_j]
    T prev[K + 1], cur[K + 1];
    static_for<1, K + 1>([&](auto jc) { prev[decltype(jc)::value] = xs[at(0, decltype(jc)::value)]; });
    T result = prev[K];
    static_for<2, K + 1>([&](auto mc) {
        constexpr int m = decltype(mc)::value;
        static_for<m, K + 1>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            T acc = T(0);
            static_for<m - 1, j>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                acc += prev[i] * xs[at(i, j)];
            });
            cur[j] = acc;
        });
        result += ((m & 1) ? T(1) : T(-1)) / T(m) * cur[K];
        static_for<m, K + 1>([&](auto jc) { prev[decltype(jc)::value] = cur[decltype(jc)::value]; });
    });
    return result;
}

template <typename T, int D>
__global__ void __launch_bounds__(256)
sig_log_direct_kernel(Shape sh, const T *__restrict__ in, T *__restrict__ out)
{
    const uint32_t d = uint32_t(sh.d);
    const int N = sh.N;
    uint32_t off[kDirectMaxDepth + 2];
#pragma unroll
    for (int k = 0; k <= kDirectMaxDepth + 1; ++k) off[k] = k <= N + 1 ? uint32_t(sh.off[k]) : 0xffffffffu;
    const uint32_t S = uint32_t(sh.S);
    const int64_t total = sh.B * int64_t(S);
    for (int64_t e = blockIdx.x * int64_t(blockDim.x) + threadIdx.x; e < total; e += int64_t(gridDim.x) * blockDim.x) {
        const int64_t r = e / S;
        const uint32_t i = uint32_t(e - r * S);
        const T *x = in + r * S;
        int k = 1;
#pragma unroll
        for (int j = 2; j <= kDirectMaxDepth; ++j) k += (j <= N && i >= off[j]) ? 1 : 0;
        // off[k] as a select over constants indices (the array lives in registers)
        uint32_t base = 0;
#pragma unroll
        for (int j = 2; j <= kDirectMaxDepth; ++j) base = (j == k) ? off[j] : base;
        const uint32_t idx = i - base;
        T v;
        switch (k) {
            case 1: v = x[i]; break;
            case 2: v = log_of_word<T, D, 2>(x, idx, d, off); break;
            case 3: v = log_of_word<T, D, 3>(x, idx, d, off); break;
            case 4: v = log_of_word<T, D, 4>(x, idx, d, off); break;
            case 5: v = log_of_word<T, D, 5>(x, idx, d, off); break;
            case 6: v = log_of_word<T, D, 6>(x, idx, d, off); break;
            case 7: v = log_of_word<T, D, 7>(x, idx, d, off); break;
            case 8: v = log_of_word<T, D, 8>(x, idx, d, off); break;
            default: v = log_of_word<T, D, 9>(x, idx, d, off); break;
        }
        out[e] = v;
    }
}

template <typename T, int D>
void launch_direct(const Shape &sh, const T *in, T *out, hipStream_t st)
{
    const int64_t total = sh.B * sh.S;
    const unsigned grid = unsigned((total + 255) / 256 < (1 << 20) ? (total + 255) / 256 : (1 << 20));
    hipLaunchKernelGGL((sig_log_direct_kernel<T, D>), dim3(grid), dim3(256), 0, st, sh, in, out);
}

template <typename T, int D, int N>
bool try_fixed(const Shape &sh, const T *in, T *out, unsigned grid, hipStream_t st)
{
    constexpr size_t lds = 2 * size_t(fixed_off(D, N + 1)) * sizeof(T);
    if constexpr (lds <= 64 * 1024) {
        if (sh.d == D && sh.N == N) {
            hipLaunchKernelGGL((sig_log_fixed_kernel<T, D, N>), dim3(grid), dim3(256), lds, st, sh.B, in, out);
            return true;
        }
    }
    return false;
}

template <typename T>
__global__ void __launch_bounds__(256)
sig_gather_kernel(const T *__restrict__ in, int64_t in_stride, const int64_t *__restrict__ index, int64_t n,
                  int64_t rows, T *__restrict__ out)
{
    for (int64_t r = blockIdx.y; r < rows; r += gridDim.y)
        for (int64_t i = blockIdx.x * int64_t(blockDim.x) + threadIdx.x; i < n; i += int64_t(gridDim.x) * blockDim.x)
            out[r * n + i] = in[r * in_stride + index[i]];
}

template <typename T>
hipError_t launch_log(const Shape &sh, const T *in, T *out, hipStream_t st)
{
    const unsigned grid = unsigned(sh.B < (int64_t(1) << 20) ? sh.B : (int64_t(1) << 20));
    if (try_fixed<T, 2, 2>(sh, in, out, grid, st) || try_fixed<T, 2, 3>(sh, in, out, grid, st) ||
        try_fixed<T, 2, 4>(sh, in, out, grid, st) || try_fixed<T, 2, 5>(sh, in, out, grid, st) ||
        try_fixed<T, 2, 6>(sh, in, out, grid, st) || try_fixed<T, 2, 7>(sh, in, out, grid, st) ||
        try_fixed<T, 3, 2>(sh, in, out, grid, st) || try_fixed<T, 3, 3>(sh, in, out, grid, st) ||
        try_fixed<T, 3, 4>(sh, in, out, grid, st) || try_fixed<T, 3, 5>(sh, in, out, grid, st) ||
        try_fixed<T, 3, 6>(sh, in, out, grid, st) || try_fixed<T, 4, 2>(sh, in, out, grid, st) ||
        try_fixed<T, 4, 3>(sh, in, out, grid, st) || try_fixed<T, 4, 4>(sh, in, out, grid, st) ||
        try_fixed<T, 4, 5>(sh, in, out, grid, st) || try_fixed<T, 4, 6>(sh, in, out, grid, st) ||
        try_fixed<T, 8, 2>(sh, in, out, grid, st) || try_fixed<T, 8, 3>(sh, in, out, grid, st) ||
        try_fixed<T, 8, 4>(sh, in, out, grid, st))
        return hipGetLastError();
    if (sh.N <= kDirectMaxDepth) {
        switch (sh.d) {
            case 2: launch_direct<T, 2>(sh, in, out, st); break;
            case 3: launch_direct<T, 3>(sh, in, out, st); break;
            case 4: launch_direct<T, 4>(sh, in, out, st); break;
            case 5: launch_direct<T, 5>(sh, in, out, st); break;
            case 6: launch_direct<T, 6>(sh, in, out, st); break;
            case 7: launch_direct<T, 7>(sh, in, out, st); break;
            case 8: launch_direct<T, 8>(sh, in, out, st); break;
            default: launch_direct<T, 0>(sh, in, out, st); break;
        }
        return hipGetLastError();
    }
    const size_t lds = 2 * size_t(sh.S) * sizeof(T);
    const bool in_lds = lds <= 64 * 1024;
#define SIG_LOG_LAUNCH(DD)                                                                                        \
    do {                                                                                                          \
        if (in_lds)                                                                                               \
            hipLaunchKernelGGL((sig_log_kernel<T, true, DD>), dim3(grid), dim3(256), lds, st, sh, in, out);       \
        else                                                                                                      \
            hipLaunchKernelGGL((sig_log_kernel<T, false, DD>), dim3(grid), dim3(256), 0, st, sh, in, out);        \
    } while (0)
    SIG_LOG_LAUNCH(0);
#undef SIG_LOG_LAUNCH
    return hipGetLastError();
}

template <typename T>
hipError_t launch_gather(const Shape &sh, const T *in, const int64_t *index, int64_t n, T *out, hipStream_t st)
{
    const unsigned bx = unsigned((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
    const unsigned by = unsigned(sh.B < 65535 ? sh.B : 65535);
    hipLaunchKernelGGL((sig_gather_kernel<T>), dim3(bx, by), dim3(256), 0, st, in, sh.S, index, n, sh.B, out);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_log_f32(const Shape &sh, const float *in, float *out, hipStream_t st) { return launch_log(sh, in, out, st); }
hipError_t launch_log_f64(const Shape &sh, const double *in, double *out, hipStream_t st) { return launch_log(sh, in, out, st); }
hipError_t launch_gather_f32(const Shape &sh, const float *in, const int64_t *index, int64_t n, float *out, hipStream_t st)
{
    return launch_gather(sh, in, index, n, out, st);
}
hipError_t launch_gather_f64(const Shape &sh, const double *in, const int64_t *index, int64_t n, double *out, hipStream_t st)
{
    return launch_gather(sh, in, index, n, out, st);
}

// Offsets of the coefficients of all Lyndon words of length 1..N inside a flat element: by length, and
// lexicographically inside a length.  The words come from Duval's generation scheme: starting from the
// single letter 0, the successor of a Lyndon word w is obtained by repeating w up to length N, dropping
// trailing maximal letters and incrementing the last one left; every word so produced whose length is a
// fixed point of that repetition (length = that of the generating prefix) is a Lyndon word, in
// lexicographic order over all lengths together.  Returns the number of words, or -1 on overflow of `cap`.
int64_t lyndon_indices_host(const Shape &sh, int64_t *indices, int64_t cap)
{
    const int d = sh.d, N = sh.N;
    std::vector<std::vector<int64_t>> by_length(size_t(N) + 1);
    std::vector<int> w(size_t(N), 0);
    int len = 1;
    w[0] = 0;
    while (len > 0) {
        // w[0..len) is a Lyndon word
        int64_t flat = 0;
        for (int i = 0; i < len; ++i) flat = flat * d + w[size_t(i)];
        by_length[size_t(len)].push_back(sh.off[len] + flat);
        // repeat to length N
        for (int i = len; i < N; ++i) w[size_t(i)] = w[size_t(i - len)];
        len = N;
        while (len > 0 && w[size_t(len - 1)] == d - 1) --len;
        if (len > 0) ++w[size_t(len - 1)];
    }
    int64_t n = 0;
    for (int k = 1; k <= N; ++k)
        for (int64_t v : by_length[size_t(k)]) {
            if (indices != nullptr) {
                if (n >= cap) return -1;
                indices[n] = v;
            }
            ++n;
        }
    return n;
}

}  // namespace sig
