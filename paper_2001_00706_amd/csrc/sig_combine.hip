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

// Where product p finds its operands: with p = q * n_inner + i (i < n_inner), operand a starts at
// a + q * a_outer + i * a_inner scalars, likewise b and out.  Packed operands: n_inner = everything, inner = S.
struct Strides {
    int64_t a, b, out;                    // inner strides
    int64_t n_inner;                      // products per outer step
    int64_t a_outer, b_outer, out_outer;  // outer strides
};

// D: the channel count when it is one of the common ones (division by a constant is a multiply
// and a shift), 0 for any other d (division by the runtime value).
template <typename T, int D>
__global__ void __launch_bounds__(256)
sig_combine_kernel(Shape sh, Strides rs, const T *__restrict__ a, const T *__restrict__ b, T *__restrict__ out)
{
    const uint32_t S = uint32_t(sh.S);
    const int N = sh.N;
    const uint32_t d = D > 0 ? uint32_t(D) : uint32_t(sh.d);
    for (int64_t p = blockIdx.y; p < sh.B; p += gridDim.y) {
        const int64_t q = p / rs.n_inner, r = p - q * rs.n_inner;
        const T *ap = a + q * rs.a_outer + r * rs.a;
        const T *bp = b + q * rs.b_outer + r * rs.b;
        T *op = out + q * rs.out_outer + r * rs.out;
        for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < S; i += gridDim.x * blockDim.x) {
            int k = 1;
            while (k < N && i >= uint32_t(sh.off[k + 1])) ++k;
            const uint32_t idx = i - uint32_t(sh.off[k]);
            T acc = ap[i] + bp[i];
            // peel letters off the end of the word: prefix w_1..w_j and suffix w_{j+1}..w_k, j = k-1 .. 1
            uint32_t prefix = idx, suffix = 0, scale = 1;
            for (int j = k - 1; j >= 1; --j) {
                const uint32_t letter = prefix % d;
                prefix /= d;
                suffix += letter * scale;
                scale *= d;
                acc += ap[uint32_t(sh.off[j]) + prefix] * bp[uint32_t(sh.off[k - j]) + suffix];
            }
            op[i] = acc;
        }
    }
}

// Four consecutive words per thread, for channel counts that are multiples of 4 (then every level
// size and offset is a multiple of 4 too): the four words differ only in their last letter, so each
// term is one broadcast scalar of `a` times four consecutive scalars of `b`, and all traffic moves
// in 4-scalar vectors.
template <typename T, int D>
__global__ void __launch_bounds__(256)
sig_combine_vec4_kernel(Shape sh, Strides rs, const T *__restrict__ a, const T *__restrict__ b, T *__restrict__ out)
{
    static_assert(D % 4 == 0, "vector path needs d to be a multiple of 4");
    typedef T T4 __attribute__((ext_vector_type(4)));
    const uint32_t S4 = uint32_t(sh.S) / 4;
    const int N = sh.N;
    for (int64_t p = blockIdx.y; p < sh.B; p += gridDim.y) {
        const int64_t q = p / rs.n_inner, r = p - q * rs.n_inner;
        const T *ap = a + q * rs.a_outer + r * rs.a;
        const T *bp = b + q * rs.b_outer + r * rs.b;
        T *op = out + q * rs.out_outer + r * rs.out;
        for (uint32_t v = blockIdx.x * blockDim.x + threadIdx.x; v < S4; v += gridDim.x * blockDim.x) {
            const uint32_t i = 4 * v;
            int k = 1;
            while (k < N && i >= uint32_t(sh.off[k + 1])) ++k;
            const uint32_t idx = i - uint32_t(sh.off[k]);
            T4 acc = *reinterpret_cast<const T4 *>(ap + i) + *reinterpret_cast<const T4 *>(bp + i);
            uint32_t prefix = idx, suffix = 0, scale = 1;
            for (int j = k - 1; j >= 1; --j) {
                const uint32_t letter = prefix % D;   // for j = k-1 this is the (4-aligned) last letter
                prefix /= D;
                suffix += letter * scale;
                scale *= D;
                acc += ap[uint32_t(sh.off[j]) + prefix] *
                       *reinterpret_cast<const T4 *>(bp + uint32_t(sh.off[k - j]) + suffix);
            }
            *reinterpret_cast<T4 *>(op + i) = acc;
        }
    }
}

template <typename T>
hipError_t launch_combine(const Shape &sh, const T *a, const T *b, T *out, hipStream_t st, const int64_t *strides)
{
    // strides: {a, b, out} or {a, b, out, n_inner, a_outer, b_outer, out_outer} (flagged by a negative first entry
    // being impossible: the caller passes the count in strides[3] as 0 when there is no outer level)
    const int64_t whole = int64_t(1) << 62;
    Strides rs = {sh.S, sh.S, sh.S, whole, 0, 0, 0};
    if (strides != nullptr) {
        rs.a = strides[0];
        rs.b = strides[1];
        rs.out = strides[2];
        if (strides[3] > 0) {
            rs.n_inner = strides[3];
            rs.a_outer = strides[4];
            rs.b_outer = strides[5];
            rs.out_outer = strides[6];
        }
    }
    const unsigned bx = unsigned((sh.S + 255) / 256 < 4096 ? (sh.S + 255) / 256 : 4096);
    const unsigned by = unsigned(sh.B < 65535 ? sh.B : 65535);
    const dim3 grid(bx, by), block(256);
    const bool aligned = (reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b) | reinterpret_cast<uintptr_t>(out)) %
                                 (4 * sizeof(T)) == 0 &&
                         (rs.a | rs.b | rs.out | rs.a_outer | rs.b_outer | rs.out_outer) % 4 == 0;
    if (aligned && (sh.d == 4 || sh.d == 8 || sh.d == 16)) {
        const dim3 grid4(unsigned((sh.S / 4 + 255) / 256 < 4096 ? (sh.S / 4 + 255) / 256 : 4096), by);
        if (sh.d == 4) hipLaunchKernelGGL((sig_combine_vec4_kernel<T, 4>), grid4, block, 0, st, sh, rs, a, b, out);
        if (sh.d == 8) hipLaunchKernelGGL((sig_combine_vec4_kernel<T, 8>), grid4, block, 0, st, sh, rs, a, b, out);
        if (sh.d == 16) hipLaunchKernelGGL((sig_combine_vec4_kernel<T, 16>), grid4, block, 0, st, sh, rs, a, b, out);
        return hipGetLastError();
    }
    switch (sh.d) {
        case 2: hipLaunchKernelGGL((sig_combine_kernel<T, 2>), grid, block, 0, st, sh, rs, a, b, out); break;
        case 3: hipLaunchKernelGGL((sig_combine_kernel<T, 3>), grid, block, 0, st, sh, rs, a, b, out); break;
        case 4: hipLaunchKernelGGL((sig_combine_kernel<T, 4>), grid, block, 0, st, sh, rs, a, b, out); break;
        case 5: hipLaunchKernelGGL((sig_combine_kernel<T, 5>), grid, block, 0, st, sh, rs, a, b, out); break;
        case 6: hipLaunchKernelGGL((sig_combine_kernel<T, 6>), grid, block, 0, st, sh, rs, a, b, out); break;
        case 7: hipLaunchKernelGGL((sig_combine_kernel<T, 7>), grid, block, 0, st, sh, rs, a, b, out); break;
        case 8: hipLaunchKernelGGL((sig_combine_kernel<T, 8>), grid, block, 0, st, sh, rs, a, b, out); break;
        case 16: hipLaunchKernelGGL((sig_combine_kernel<T, 16>), grid, block, 0, st, sh, rs, a, b, out); break;
        default: hipLaunchKernelGGL((sig_combine_kernel<T, 0>), grid, block, 0, st, sh, rs, a, b, out); break;
    }
    return hipGetLastError();
}

}  // namespace

bool combine_supported(const Shape &sh) { return sh.S < (int64_t(1) << 31); }

hipError_t launch_combine_f32(const Shape &sh, const float *a, const float *b, float *out, hipStream_t st,
                              const int64_t *strides)
{
    return launch_combine<float>(sh, a, b, out, st, strides);
}

hipError_t launch_combine_f64(const Shape &sh, const double *a, const double *b, double *out, hipStream_t st,
                              const int64_t *strides)
{
    return launch_combine<double>(sh, a, b, out, st, strides);
}

}  // namespace sig
