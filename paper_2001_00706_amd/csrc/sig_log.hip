// Logarithm of signatures in the truncated tensor algebra and the logsignature in the basis of paper
// appendix A.2.4 (sections 2.3 and 4.3).
//
// log: with x the signature without its constant term,  log(1 + x) = sum_{m=1..N} c_m x^{[x] m},
// c_m = (-1)^{m+1} / m, evaluated by Horner's rule from the inside out:
//     R_N = c_N x,   R_m = c_m x + x [x] R_{m+1},   log = R_1.
// R_m is needed at levels 1..N-m+1 only (a product of m or more factors has no lower levels to feed), so
// the top level is computed once.  A product x [x] R reads strictly lower levels of R, so R lives in `out`
// and is updated in place, levels highest first, with a workgroup barrier between levels; one workgroup
// per signature.
//
// logsignature: psi(log(Sig)) is the vector of coefficients of the Lyndon words (appendix A.2.4): a gather
// with an index table that `sig_lyndon_indices` computes on the host.
#include "sig_internal.h"

#include <vector>

namespace sig {
namespace {

template <typename T>
__global__ void __launch_bounds__(256)
sig_log_kernel(Shape sh, const T *__restrict__ in, T *__restrict__ out)
{
    const uint32_t d = uint32_t(sh.d);
    const int N = sh.N;
    for (int64_t r = blockIdx.x; r < sh.B; r += gridDim.x) {
        const T *x = in + r * sh.S;
        T *R = out + r * sh.S;
        for (int m = N; m >= 1; --m) {
            const T c = (m & 1 ? T(1) : T(-1)) / T(m);
            for (int k = N - m + 1; k >= 1; --k) {
                const uint32_t n_k = uint32_t(sh.pw[k]), off_k = uint32_t(sh.off[k]);
                for (uint32_t idx = threadIdx.x; idx < n_k; idx += blockDim.x) {
                    T acc = c * x[off_k + idx];
                    // splits of the word into a prefix of x (j letters) and a suffix of R (k - j letters)
                    uint32_t prefix = idx, suffix = 0, scale = 1;
                    for (int j = k - 1; j >= 1; --j) {
                        const uint32_t letter = prefix % d;
                        prefix /= d;
                        suffix += letter * scale;
                        scale *= d;
                        acc += x[uint32_t(sh.off[j]) + prefix] * R[uint32_t(sh.off[k - j]) + suffix];
                    }
                    R[off_k + idx] = acc;
                }
                __syncthreads();
            }
        }
    }
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
    hipLaunchKernelGGL((sig_log_kernel<T>), dim3(grid), dim3(256), 0, st, sh, in, out);
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
