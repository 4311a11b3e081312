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
// formed) and two barriers per product.  A product is written to a buffer of its own (two buffers take turns as
// left factor and result), so its levels need no barrier between them.
// A workgroup barrier that orders the LDS traffic only: __syncthreads() would also wait for the global loads and
// stores in flight (the next right factor on its way in, the last product on its way out), which is the latency
// this kernel is built to keep off the chain.
__device__ __forceinline__ void prefix_lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// n / d for n < 2^16 and 1 <= d < 2^16 with magic = ceil(2^32 / d) kept in 32 bits: the excess
// n (magic d - 2^32) / (d 2^32) stays below n / 2^32 < 1 / d, so it never carries into the quotient.  For d = 1 the
// magic number is 2^32, which 32 bits hold as 0: the quotient is n itself (one channel, or a signature of one scalar).
__device__ __forceinline__ uint32_t prefix_div(uint32_t n, uint32_t magic) { return magic != 0 ? __umulhi(n, magic) : n; }

constexpr int kPrefixPerThread = 32;
constexpr int kPrefixLdsWords = 256 * kPrefixPerThread;

template <typename T, int THREADS>
__global__ void __launch_bounds__(THREADS)
sig_chunk_prefix_lds_kernel(Shape sh, int64_t paths, int64_t n_inc, int64_t chunk_len, T *out)
{
    extern __shared__ __align__(16) unsigned char prefix_smem[];
    const uint32_t S = uint32_t(sh.S), d = uint32_t(sh.d);
    const int N = sh.N;
    const uint32_t magic = uint32_t(((uint64_t(1) << 32) + d - 1) / d);   // level sizes here stay below 2^16
    // the level tables where a run-time index costs an LDS read (indexing the kernel argument would go through scratch)
    __shared__ uint32_t lv_off[SIG_MAX_DEPTH + 2], lv_size[SIG_MAX_DEPTH + 2];
    if (threadIdx.x >= 1 && threadIdx.x <= uint32_t(N) + 1) {   // level t: d^t words after d + .. + d^(t-1) others
        uint32_t size = d, before = 0;
        for (uint32_t t = 1; t < threadIdx.x; ++t) {
            before += size;
            size *= d;
        }
        lv_off[threadIdx.x] = before;
        lv_size[threadIdx.x] = size;
    }
    __syncthreads();
    T *A = reinterpret_cast<T *>(prefix_smem);   // the product so far,
    T *C = A + S;                                // the product being formed (the two swap after every product),
    T *R = C + S;                                // the right factor: the signature of the current chunk alone
    const uint32_t tid = threadIdx.x;
    for (int64_t p = blockIdx.x; p < paths; p += gridDim.x) {
        T *rows = out + p * n_inc * sh.S;
        const int64_t first_end = (chunk_len < n_inc ? chunk_len : n_inc) - 1;
        for (uint32_t i = tid; i < S; i += THREADS) A[i] = rows[first_end * sh.S + i];
        constexpr int kPerThread = kPrefixLdsWords / THREADS;
        T next[kPerThread];
        auto fetch = [&](int64_t start) {
            if (start >= n_inc) return;
            const T *src = rows + ((start + chunk_len < n_inc ? start + chunk_len : n_inc) - 1) * sh.S;
#pragma unroll
            for (int j = 0; j < kPerThread; ++j)   // unconditional, on a clamped index: the loads stay in flight together
                if (uint32_t(THREADS) * j < S) next[j] = src[tid + uint32_t(THREADS) * j < S ? tid + uint32_t(THREADS) * j : S - 1];
        };
        fetch(chunk_len);
        for (int64_t start = chunk_len; start < n_inc; start += chunk_len) {
            T *dst = rows + ((start + chunk_len < n_inc ? start + chunk_len : n_inc) - 1) * sh.S;
#pragma unroll
            for (int j = 0; j < kPerThread; ++j)
                if (tid + uint32_t(THREADS) * j < S) R[tid + uint32_t(THREADS) * j] = next[j];
            fetch(start + chunk_len);
            prefix_lds_barrier();
            for (int k = N; k >= 1; --k) {
                const uint32_t n_k = lv_size[k], off_k = lv_off[k];
                for (uint32_t idx = tid; idx < n_k; idx += THREADS) {
                    T acc = A[off_k + idx] + R[off_k + idx];
                    uint32_t prefix = idx, suffix = 0, scale = 1;
                    for (int j = k - 1; j >= 1; --j) {
                        const uint32_t q = prefix_div(prefix, magic);
                        const uint32_t letter = prefix - q * d;
                        prefix = q;
                        suffix += letter * scale;
                        scale *= d;
                        acc += A[lv_off[j] + prefix] * R[lv_off[k - j] + suffix];
                    }
                    C[off_k + idx] = acc;
                    dst[off_k + idx] = acc;
                }
            }
            prefix_lds_barrier();
            T *swap = A;
            A = C;
            C = swap;
        }
        __syncthreads();   // the next path's first row overwrites a buffer that may still be read
    }
}

// The same with every chunk signature of the path brought into LDS at once (one trip to memory for the whole chain):
// for paths whose chunk signatures fit together.
template <typename T>
__global__ void __launch_bounds__(256)
sig_chunk_prefix_all_kernel(Shape sh, int64_t paths, int64_t n_inc, int64_t chunk_len, int n_chunks, T *out)
{
    extern __shared__ __align__(16) unsigned char prefix_smem[];
    const uint32_t S = uint32_t(sh.S), d = uint32_t(sh.d);
    const int N = sh.N;
    const uint32_t magic = uint32_t(((uint64_t(1) << 32) + d - 1) / d);   // level sizes here stay below 2^16
    // the level tables where a run-time index costs an LDS read (indexing the kernel argument would go through scratch)
    __shared__ uint32_t lv_off[SIG_MAX_DEPTH + 2], lv_size[SIG_MAX_DEPTH + 2];
    if (threadIdx.x >= 1 && threadIdx.x <= uint32_t(N) + 1) {   // level t: d^t words after d + .. + d^(t-1) others
        uint32_t size = d, before = 0;
        for (uint32_t t = 1; t < threadIdx.x; ++t) {
            before += size;
            size *= d;
        }
        lv_off[threadIdx.x] = before;
        lv_size[threadIdx.x] = size;
    }
    __syncthreads();
    T *all = reinterpret_cast<T *>(prefix_smem);   // chunk c at all + c * S, one spare signature behind them: the
                                                   // product so far and the product being formed take turns in chunk
                                                   // 0's place and the spare, so the levels of a product need no barrier
    const uint32_t tid = threadIdx.x;
    for (int64_t p = blockIdx.x; p < paths; p += gridDim.x) {
        T *rows = out + p * n_inc * sh.S;
        {
            // scalar e of the chunk signatures laid end to end is scalar i of chunk c; eight loads in flight per thread
            // (every one of them unconditional, on a clamped index: a load under a branch would be waited for there)
            const uint32_t total = uint32_t(n_chunks) * S;
            const uint32_t magic_s = uint32_t(((uint64_t(1) << 32) + S - 1) / S);   // total < 2^16
            for (uint32_t e0 = tid; e0 < total; e0 += 256 * 8) {
                T v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const uint32_t e = e0 + 256u * j < total ? e0 + 256u * j : total - 1;
                    const uint32_t c = prefix_div(e, magic_s), i = e - c * S;
                    const int64_t end = ((int64_t(c) + 1) * chunk_len < n_inc ? (int64_t(c) + 1) * chunk_len : n_inc) - 1;
                    v[j] = rows[end * sh.S + i];
                }
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (e0 + 256u * j < total) all[e0 + 256u * j] = v[j];
            }
        }
        __syncthreads();
        T *A = all, *C = all + uint32_t(n_chunks) * S;
        for (int c = 1; c < n_chunks; ++c) {
            const T *R = all + uint32_t(c) * S;
            T *dst = rows + (((c + 1) * chunk_len < n_inc ? (c + 1) * chunk_len : n_inc) - 1) * sh.S;
            for (int k = N; k >= 1; --k) {
                const uint32_t n_k = lv_size[k], off_k = lv_off[k];
                for (uint32_t idx = tid; idx < n_k; idx += 256) {
                    T acc = A[off_k + idx] + R[off_k + idx];
                    uint32_t prefix = idx, suffix = 0, scale = 1;
                    for (int j = k - 1; j >= 1; --j) {
                        const uint32_t q = prefix_div(prefix, magic);
                        const uint32_t letter = prefix - q * d;
                        prefix = q;
                        suffix += letter * scale;
                        scale *= d;
                        acc += A[lv_off[j] + prefix] * R[lv_off[k - j] + suffix];
                    }
                    C[off_k + idx] = acc;
                    dst[off_k + idx] = acc;
                }
            }
            prefix_lds_barrier();
            T *swap = A;
            A = C;
            C = swap;
        }
        __syncthreads();   // the next path's loads overwrite the chunk signatures
    }
}



// The same for signatures of at most 1024 scalars, with everything that does not depend on the data taken out of the
// chain: a thread owns up to four words, and which scalars of the two factors make up each of them (N - 1 pairs of
// LDS indices per word, pointing at a zero kept behind every signature where a word has fewer terms) is worked out
// once, into registers.  A product is then one batch of independent LDS reads and multiply-adds: one LDS latency
// instead of one per term.  NT = N - 1.
constexpr int kPrefixSmallWords = 1024;

template <typename T, int NT>
__global__ void __launch_bounds__(256)
sig_chunk_prefix_small_kernel(Shape sh, int64_t paths, int64_t n_inc, int64_t chunk_len, int n_chunks, T *out)
{
    constexpr int W = kPrefixSmallWords / 256;
    extern __shared__ __align__(16) unsigned char prefix_smem[];
    const uint32_t S = uint32_t(sh.S), d = uint32_t(sh.d);
    const uint32_t row = S + 1;                        // a signature and a zero behind it
    T *X = reinterpret_cast<T *>(prefix_smem);         // chunk c at X + c * row, one spare row behind them: the product
                                                       // so far and the product being formed take turns in chunk 0's
                                                       // place and the spare
    const uint32_t tid = threadIdx.x;
    const uint32_t magic = uint32_t(((uint64_t(1) << 32) + d - 1) / d);
    const uint32_t magic_s = uint32_t(((uint64_t(1) << 32) + S - 1) / S);
    uint32_t own[W], term[W][NT > 0 ? NT : 1];
#pragma unroll
    for (int w = 0; w < W; ++w) {
        const uint32_t i = tid + 256u * w;
        own[w] = i < S ? i : S;
        uint32_t k = 1, before = 0, size = d;
        while (i < S && i >= before + size) {   // the level of word i
            before += size;
            size *= d;
            ++k;
        }
        // peel letters off the end of the word: prefix w_1..w_j (level j) and suffix w_{j+1}..w_k (level k - j)
        uint32_t prefix = i - before, suffix = 0, scale = 1, suf_size = 1, suf_off = 0;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            uint32_t entry = (S << 16) | S;   // no such term: zero times zero
            if (i < S && uint32_t(t) + 1 < k) {
                const uint32_t q = prefix_div(prefix, magic);
                suffix += (prefix - q * d) * scale;
                prefix = q;
                scale *= d;
                suf_size *= d;                      // d^(t+1); suf_off is the offset of level t + 1
                uint32_t pre_off = 0, pre_size = d;   // offset of level k - 1 - t
                for (uint32_t l = 1; l + 1 + uint32_t(t) < k; ++l) {
                    pre_off += pre_size;
                    pre_size *= d;
                }
                entry = ((pre_off + prefix) << 16) | (suf_off + suffix);
                suf_off += suf_size;
            }
            term[w][t] = entry;
        }
    }
    for (int64_t p = blockIdx.x; p < paths; p += gridDim.x) {
        T *rows = out + p * n_inc * sh.S;
        const uint32_t total = uint32_t(n_chunks) * S;
        for (uint32_t e0 = tid; e0 < total; e0 += 256 * 8) {
            T v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {   // unconditional loads on a clamped index: all in flight together
                const uint32_t e = e0 + 256u * j < total ? e0 + 256u * j : total - 1;
                const uint32_t c = prefix_div(e, magic_s), i = e - c * S;
                const int64_t end = ((int64_t(c) + 1) * chunk_len < n_inc ? (int64_t(c) + 1) * chunk_len : n_inc) - 1;
                v[j] = rows[end * sh.S + i];
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t e = e0 + 256u * j;
                if (e < total) {
                    const uint32_t c = prefix_div(e, magic_s);
                    X[c * row + (e - c * S)] = v[j];
                }
            }
        }
        if (tid <= uint32_t(n_chunks)) X[tid * row + S] = T(0);
        __syncthreads();
        T *A = X, *C = X + uint32_t(n_chunks) * row;
        for (int c = 1; c < n_chunks; ++c) {
            const T *R = X + uint32_t(c) * row;
            T *dst = rows + (((int64_t(c) + 1) * chunk_len < n_inc ? (int64_t(c) + 1) * chunk_len : n_inc) - 1) * sh.S;
            T acc[W];
#pragma unroll
            for (int w = 0; w < W; ++w) acc[w] = A[own[w]] + R[own[w]];
#pragma unroll
            for (int w = 0; w < W; ++w)
#pragma unroll
                for (int t = 0; t < NT; ++t) acc[w] += A[term[w][t] >> 16] * R[term[w][t] & 0xffffu];
#pragma unroll
            for (int w = 0; w < W; ++w)
                if (tid + 256u * w < S) {
                    C[own[w]] = acc[w];
                    dst[own[w]] = acc[w];
                }
            prefix_lds_barrier();
            T *swap = A;
            A = C;
            C = swap;
        }
        __syncthreads();   // the next path's loads overwrite the chunk signatures
    }
}

template <typename T>
hipError_t launch_chunk_prefix_small(const Shape &sh, int64_t paths, int64_t n_inc, int64_t chunk_len, int n_chunks, T *out,
                                     unsigned grid, size_t lds, hipStream_t st)
{
    switch (sh.N) {
#define SIG_PREFIX_SMALL_CASE(n)                                                                                        \
    case n:                                                                                                             \
        hipLaunchKernelGGL((sig_chunk_prefix_small_kernel<T, n - 1>), dim3(grid), dim3(256), lds, st, sh, paths, n_inc,    \
                           chunk_len, n_chunks, out);                                                                   \
        return hipGetLastError();
        SIG_PREFIX_SMALL_CASE(1)
        SIG_PREFIX_SMALL_CASE(2)
        SIG_PREFIX_SMALL_CASE(3)
        SIG_PREFIX_SMALL_CASE(4)
        SIG_PREFIX_SMALL_CASE(5)
        SIG_PREFIX_SMALL_CASE(6)
        SIG_PREFIX_SMALL_CASE(7)
        SIG_PREFIX_SMALL_CASE(8)
        SIG_PREFIX_SMALL_CASE(9)
#undef SIG_PREFIX_SMALL_CASE
    }
    return hipErrorNotSupported;
}

template <typename T>
hipError_t launch_chunk_prefix(const Shape &sh, int64_t paths, int64_t n_inc, int64_t chunk_len, T *out, hipStream_t st)
{
    const unsigned grid = unsigned(paths < (int64_t(1) << 20) ? paths : (int64_t(1) << 20));
    const int64_t n_chunks = (n_inc + chunk_len - 1) / chunk_len;
    const size_t lds_small = size_t(n_chunks + 1) * size_t(sh.S + 1) * sizeof(T);
    if (sh.S <= kPrefixSmallWords && sh.N <= 9 && sh.d <= 64 && n_chunks <= 255 && n_chunks * sh.S < 65536 && lds_small <= 60 * 1024)
        return launch_chunk_prefix_small(sh, paths, n_inc, chunk_len, int(n_chunks), out, grid, lds_small, st);
    const size_t lds_all = size_t(n_chunks + 1) * size_t(sh.S) * sizeof(T);
    if (n_chunks <= 64 && lds_all <= 60 * 1024) {
        hipLaunchKernelGGL((sig_chunk_prefix_all_kernel<T>), dim3(grid), dim3(256), lds_all, st, sh, paths, n_inc, chunk_len,
                           int(n_chunks), out);
        return hipGetLastError();
    }
    const size_t lds = 3 * size_t(sh.S) * sizeof(T);
    if (sh.S <= kPrefixLdsWords && lds <= 64 * 1024) {
        // a product is about N multiply-adds per scalar, instruction-bound: 16 wavefronts for the larger signatures
        if (sh.S >= 1024)
            hipLaunchKernelGGL((sig_chunk_prefix_lds_kernel<T, 1024>), dim3(grid), dim3(1024), lds, st, sh, paths, n_inc, chunk_len, out);
        else
            hipLaunchKernelGGL((sig_chunk_prefix_lds_kernel<T, 256>), dim3(grid), dim3(256), lds, st, sh, paths, n_inc, chunk_len, out);
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
