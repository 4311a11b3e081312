// Group operations on batches of signatures that are already in memory (paper sections 5.4, 5.5):
//   * the inverse, Sig(x_1..x_L)^{-1} = Sig(x_L..x_1) (section 5.4).  Reversing a path negates its
//     increments and reverses their order.  Negating the increments multiplies level k by (-1)^k
//     (each level-k term is a product of k increments, section 2.2); reversing the order of the factors
//     of exp(z_1) [x] ... [x] exp(z_n) reverses every word, because the coefficient of a word in a product
//     A [x] B collects the splits of the word into a prefix from A and a suffix from B (section 2.2), and
//     exp(z) is unchanged by word reversal.  Hence  inverse_k[w_1..w_k] = (-1)^k sig_k[w_k..w_1]:
//     a signed permutation, no arithmetic;
//   * multiplication on the left in place, out[r] <- a[r / group] [x] out[r], which continues a
//     signature that was computed earlier over the data that followed (section 5.5, "keeping the
//     signature up-to-date": the `initial` argument).
#include "sig_internal.h"

namespace sig {
namespace {

// One thread per word and row; a thread whose word is not after its reversal moves the pair, so the
// kernel also works in place.
template <typename T>
__global__ void __launch_bounds__(256)
sig_invert_kernel(Shape sh, const T *in, T *out)
{
    const uint32_t S = uint32_t(sh.S);
    const uint32_t d = uint32_t(sh.d);
    const int N = sh.N;
    for (int64_t r = blockIdx.y; r < sh.B; r += gridDim.y) {
        const T *ip = in + r * int64_t(S);
        T *op = out + r * int64_t(S);
        for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < S; i += gridDim.x * blockDim.x) {
            int k = 1;
            while (k < N && i >= uint32_t(sh.off[k + 1])) ++k;
            const uint32_t base = uint32_t(sh.off[k]);
            uint32_t rest = i - base, rev = 0;
            for (int j = 0; j < k; ++j) {
                rev = rev * d + rest % d;
                rest /= d;
            }
            const uint32_t j = base + rev;
            if (j < i) continue;   // the thread of word j moves this pair
            const T u = ip[i], v = ip[j];
            const bool odd = (k & 1) != 0;
            op[i] = odd ? -v : v;
            if (j != i) op[j] = odd ? -u : u;
        }
    }
}

// One workgroup per row; levels highest first, so that a level is overwritten only after every
// product that reads it has been formed (level k needs levels below k of the right factor, and of
// level k itself only the word being written).
template <typename T>
__global__ void __launch_bounds__(256)
sig_left_mul_inplace_kernel(Shape sh, const T *__restrict__ a, int64_t group, T *out)
{
    const uint32_t d = uint32_t(sh.d);
    const int N = sh.N;
    for (int64_t r = blockIdx.x; r < sh.B; r += gridDim.x) {
        const T *ap = a + (r / group) * sh.S;
        T *bp = out + r * sh.S;
        for (int k = N; k >= 1; --k) {
            const uint32_t n_k = uint32_t(sh.pw[k]), off_k = uint32_t(sh.off[k]);
            for (uint32_t idx = threadIdx.x; idx < n_k; idx += blockDim.x) {
                T acc = ap[off_k + idx] + bp[off_k + idx];
                uint32_t prefix = idx, suffix = 0, scale = 1;
                for (int j = k - 1; j >= 1; --j) {
                    const uint32_t letter = prefix % d;
                    prefix /= d;
                    suffix += letter * scale;
                    scale *= d;
                    acc += ap[uint32_t(sh.off[j]) + prefix] * bp[uint32_t(sh.off[k - j]) + suffix];
                }
                bp[off_k + idx] = acc;
            }
            __syncthreads();
        }
    }
}

// Running product along the chunk ends of a stream-mode output [paths][n_inc][S], in place: with e_c the last row
// of chunk c (chunks of chunk_len rows, the last one shorter), row e_c <- row e_{c-1} [x] row e_c for c = 1, 2, ..
// in turn.  Coming in, row e_c holds the signature of chunk c alone; going out, that of the path up to and
// including chunk c (Chen's identity, eq. "grouplike").  One workgroup per path; the product as in the kernel above.
template <typename T>
__global__ void __launch_bounds__(256)
sig_chunk_prefix_kernel(Shape sh, int64_t paths, int64_t n_inc, int64_t chunk_len, T *out)
{
    const uint32_t d = uint32_t(sh.d);
    const int N = sh.N;
    for (int64_t p = blockIdx.x; p < paths; p += gridDim.x) {
        T *rows = out + p * n_inc * sh.S;
        int64_t prev = (chunk_len < n_inc ? chunk_len : n_inc) - 1;
        for (int64_t start = chunk_len; start < n_inc; start += chunk_len) {
            const int64_t end = (start + chunk_len < n_inc ? start + chunk_len : n_inc) - 1;
            const T *ap = rows + prev * sh.S;
            T *bp = rows + end * sh.S;
            for (int k = N; k >= 1; --k) {
                const uint32_t n_k = uint32_t(sh.pw[k]), off_k = uint32_t(sh.off[k]);
                for (uint32_t idx = threadIdx.x; idx < n_k; idx += blockDim.x) {
                    T acc = ap[off_k + idx] + bp[off_k + idx];
                    uint32_t prefix = idx, suffix = 0, scale = 1;
                    for (int j = k - 1; j >= 1; --j) {
                        const uint32_t letter = prefix % d;
                        prefix /= d;
                        suffix += letter * scale;
                        scale *= d;
                        acc += ap[uint32_t(sh.off[j]) + prefix] * bp[uint32_t(sh.off[k - j]) + suffix];
                    }
                    bp[off_k + idx] = acc;
                }
                __syncthreads();   // also makes this row visible to the threads that read it as the next left factor
            }
            prev = end;
        }
    }
}

// The same with the running product kept in LDS (signatures of at most kPrefixLdsWords scalars): the chain from one
// chunk end to the next then holds no trip to memory (the next right factor is fetched while the current product is
// formed) and one barrier pair per product: the product is formed in place over the left factor, levels highest
// first, which needs no barrier between levels because a level reads only lower levels of the left factor and, of
// its own level, only the word it then overwrites.
constexpr int kPrefixPerThread = 32;
constexpr int kPrefixLdsWords = 256 * kPrefixPerThread;

template <typename T>
__global__ void __launch_bounds__(256)
sig_chunk_prefix_lds_kernel(Shape sh, int64_t paths, int64_t n_inc, int64_t chunk_len, T *out)
{
    extern __shared__ __align__(16) unsigned char prefix_smem[];
    const uint32_t S = uint32_t(sh.S), d = uint32_t(sh.d);
    const int N = sh.N;
    T *A = reinterpret_cast<T *>(prefix_smem);   // the product so far
    T *R = A + S;                                // the right factor: the signature of the current chunk alone
    const uint32_t tid = threadIdx.x;
    for (int64_t p = blockIdx.x; p < paths; p += gridDim.x) {
        T *rows = out + p * n_inc * sh.S;
        const int64_t first_end = (chunk_len < n_inc ? chunk_len : n_inc) - 1;
        for (uint32_t i = tid; i < S; i += 256) A[i] = rows[first_end * sh.S + i];
        T next[kPrefixPerThread];
        auto fetch = [&](int64_t start) {
            if (start >= n_inc) return;
            const T *src = rows + ((start + chunk_len < n_inc ? start + chunk_len : n_inc) - 1) * sh.S;
#pragma unroll
            for (int j = 0; j < kPrefixPerThread; ++j)
                if (tid + 256u * j < S) next[j] = src[tid + 256u * j];
        };
        fetch(chunk_len);
        for (int64_t start = chunk_len; start < n_inc; start += chunk_len) {
            T *dst = rows + ((start + chunk_len < n_inc ? start + chunk_len : n_inc) - 1) * sh.S;
#pragma unroll
            for (int j = 0; j < kPrefixPerThread; ++j)
                if (tid + 256u * j < S) R[tid + 256u * j] = next[j];
            fetch(start + chunk_len);
            __syncthreads();
            for (int k = N; k >= 1; --k) {
                const uint32_t n_k = uint32_t(sh.pw[k]), off_k = uint32_t(sh.off[k]);
                for (uint32_t idx = tid; idx < n_k; idx += 256) {
                    T acc = A[off_k + idx] + R[off_k + idx];
                    uint32_t prefix = idx, suffix = 0, scale = 1;
                    for (int j = k - 1; j >= 1; --j) {
                        const uint32_t letter = prefix % d;
                        prefix /= d;
                        suffix += letter * scale;
                        scale *= d;
                        acc += A[uint32_t(sh.off[j]) + prefix] * R[uint32_t(sh.off[k - j]) + suffix];
                    }
                    A[off_k + idx] = acc;
                    dst[off_k + idx] = acc;
                }
            }
            __syncthreads();
        }
    }
}

template <typename T>
hipError_t launch_chunk_prefix(const Shape &sh, int64_t paths, int64_t n_inc, int64_t chunk_len, T *out, hipStream_t st)
{
    const unsigned grid = unsigned(paths < (int64_t(1) << 20) ? paths : (int64_t(1) << 20));
    const size_t lds = 2 * size_t(sh.S) * sizeof(T);
    if (sh.S <= kPrefixLdsWords && lds <= 64 * 1024) {
        hipLaunchKernelGGL((sig_chunk_prefix_lds_kernel<T>), dim3(grid), dim3(256), lds, st, sh, paths, n_inc, chunk_len, out);
        return hipGetLastError();
    }
    hipLaunchKernelGGL((sig_chunk_prefix_kernel<T>), dim3(grid), dim3(256), 0, st, sh, paths, n_inc, chunk_len, out);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_invert(const Shape &sh, const T *in, T *out, hipStream_t st)
{
    const unsigned bx = unsigned((sh.S + 255) / 256 < 4096 ? (sh.S + 255) / 256 : 4096);
    const unsigned by = unsigned(sh.B < 65535 ? sh.B : 65535);
    hipLaunchKernelGGL((sig_invert_kernel<T>), dim3(bx, by), dim3(256), 0, st, sh, in, out);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_left_mul(const Shape &sh, const T *a, int64_t group, T *out, hipStream_t st)
{
    const unsigned grid = unsigned(sh.B < (int64_t(1) << 20) ? sh.B : (int64_t(1) << 20));
    hipLaunchKernelGGL((sig_left_mul_inplace_kernel<T>), dim3(grid), dim3(256), 0, st, sh, a, group, out);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_invert_f32(const Shape &sh, const float *in, float *out, hipStream_t st) { return launch_invert(sh, in, out, st); }
hipError_t launch_invert_f64(const Shape &sh, const double *in, double *out, hipStream_t st) { return launch_invert(sh, in, out, st); }
hipError_t launch_chunk_prefix_f32(const Shape &sh, int64_t paths, int64_t n_inc, int64_t chunk_len, float *out, hipStream_t st)
{
    return launch_chunk_prefix(sh, paths, n_inc, chunk_len, out, st);
}
hipError_t launch_chunk_prefix_f64(const Shape &sh, int64_t paths, int64_t n_inc, int64_t chunk_len, double *out, hipStream_t st)
{
    return launch_chunk_prefix(sh, paths, n_inc, chunk_len, out, st);
}
hipError_t launch_left_mul_f32(const Shape &sh, const float *a, int64_t group, float *out, hipStream_t st)
{
    return launch_left_mul(sh, a, group, out, st);
}
hipError_t launch_left_mul_f64(const Shape &sh, const double *a, int64_t group, double *out, hipStream_t st)
{
    return launch_left_mul(sh, a, group, out, st);
}

}  // namespace sig
