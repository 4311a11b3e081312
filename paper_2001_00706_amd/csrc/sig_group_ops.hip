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
hipError_t launch_left_mul_f32(const Shape &sh, const float *a, int64_t group, float *out, hipStream_t st)
{
    return launch_left_mul(sh, a, group, out, st);
}
hipError_t launch_left_mul_f64(const Shape &sh, const double *a, int64_t group, double *out, hipStream_t st)
{
    return launch_left_mul(sh, a, group, out, st);
}

}  // namespace sig
