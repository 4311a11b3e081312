// Group product of two batches of truncated signatures, out[b] = a[b] [x] b[b]
// (paper section 2.2:  (A [x] B)_k = sum_{j=0..k} A_j (x) B_{k-j},  A_0 = B_0 = 1; by Chen's
// identity, eq. "grouplike", this joins the signatures of two adjacent intervals, section 5.5).
//
// One thread per output word w = w_1..w_k:
//     out_k[w] = a_k[w] + b_k[w] + sum_{j=1..k-1} a_j[w_1..w_j] * b_{k-j}[w_{j+1}..w_k].
// Consecutive threads share the prefix (one broadcast read of a) and walk consecutive suffixes
// (coalesced reads of b), so the kernel runs at memory speed: 3 S scalars per path.
#include "sig_internal.h"

namespace sig {
namespace {

template <typename T>
__global__ void __launch_bounds__(256)
sig_combine_kernel(Shape sh, const T *__restrict__ a, const T *__restrict__ b, T *__restrict__ out)
{
    const uint32_t S = uint32_t(sh.S);
    const int N = sh.N;
    for (int64_t p = blockIdx.y; p < sh.B; p += gridDim.y) {
        const T *ap = a + p * int64_t(S);
        const T *bp = b + p * int64_t(S);
        T *op = out + p * int64_t(S);
        for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < S; i += gridDim.x * blockDim.x) {
            int k = 1;
            while (k < N && i >= uint32_t(sh.off[k + 1])) ++k;
            const uint32_t idx = i - uint32_t(sh.off[k]);
            T acc = ap[i] + bp[i];
            for (int j = 1; j < k; ++j) {
                const uint32_t tail = uint32_t(sh.pw[k - j]);  // d^(k-j) words of length k-j
                acc += ap[uint32_t(sh.off[j]) + idx / tail] * bp[uint32_t(sh.off[k - j]) + idx % tail];
            }
            op[i] = acc;
        }
    }
}

template <typename T>
hipError_t launch_combine(const Shape &sh, const T *a, const T *b, T *out, hipStream_t st)
{
    const unsigned bx = unsigned((sh.S + 255) / 256 < 4096 ? (sh.S + 255) / 256 : 4096);
    const unsigned by = unsigned(sh.B < 65535 ? sh.B : 65535);
    hipLaunchKernelGGL(sig_combine_kernel<T>, dim3(bx, by), dim3(256), 0, st, sh, a, b, out);
    return hipGetLastError();
}

}  // namespace

bool combine_supported(const Shape &sh) { return sh.S < (int64_t(1) << 31); }

hipError_t launch_combine_f32(const Shape &sh, const float *a, const float *b, float *out, hipStream_t st)
{
    return launch_combine<float>(sh, a, b, out, st);
}

hipError_t launch_combine_f64(const Shape &sh, const double *a, const double *b, double *out, hipStream_t st)
{
    return launch_combine<double>(sh, a, b, out, st);
}

}  // namespace sig
