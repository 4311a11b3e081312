// Matrix-core kernel family (fp32), d = 4 channels, depth N = 4..6, final mode.
//
// One wavefront scans one path and keeps the whole truncated tensor-algebra element in
// registers.  Every stage of the Horner scheme of the fused multiply-exponentiate
// (paper section 4.1, eq. "fusedterm"),
//     T^(i)[w_1..w_i] = T^(i-1)[w_1..w_{i-1}] * z[w_i]/(k-i+1) + A_i[w_1..w_i],
// is a batch of 4x4 outer products plus an addend, which is exactly what
// v_mfma_f32_4x4x1_16b_f32 computes: 16 independent blocks, D_b[i][j] = a_b[i]*b_b[j] + C_b[i][j].
// The accumulation of the top level over the increments, A_N += T^(N-1) (x) z, is a dense
// contraction over the increment index carried out one rank-1 slice at a time, because
// each slice's left factor depends on the state the previous slice produced.
//
// Register layout (lane = 16*w_1 + 4*w_2 + q, 0 <= q < 4):
//   level 1..3 ("low levels", plain VALU, one scalar per lane, replicated where the level
//       has fewer than 64 words):   A_1[w_1], A_2[w_1 w_2], A_3[w_1 w_2 q]   (q = w_3)
//   level k >= 4 (matrix cores): 4^(k-4) groups of 4 registers; group g holds the words
//       whose letters w_3..w_{k-2} spell g in base 4; register r of the group is letter
//       w_{k-1} = r; lane q is the last letter w_k = q; the block index (lane / 4) is w_1 w_2.
// With this layout the D registers of a level-k stage are, as they stand, the A operand of
// the level-(k+1) stage (register r of group g feeds group 4g + r), and the B operand is
// always z[lane & 3] times a reciprocal, so no data ever moves between lanes.
//
// Levels are updated highest first; the temporaries T^(i) of a higher target level are
// formed from the old A_i before A_i itself is overwritten, so the update is in place.
#include "sig_internal.h"

namespace sig {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int kTile = 256;  // increments staged in LDS at a time

__device__ __forceinline__ f4 outer4(float a, float b, f4 c)
{
    // 16 blocks of D[i][j] = a[i] * b[j] + C[i][j]; lane 4*blk + i supplies a[i], lane 4*blk + j supplies b[j];
    // register i of lane 4*blk + j receives D[i][j]
    return __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, c, 0, 0, 0);
}

template <int N>
struct State {
    float A1 = 0.0f, A2 = 0.0f, A3 = 0.0f;
    f4 A4[1];
    f4 A5[N >= 5 ? 4 : 1];
    f4 A6[N >= 6 ? 16 : 1];
};

// One fused multiply-exponentiate A <- A [x] exp(z).  zA, zB, zC = z[w_1], z[w_2], z[q] of this lane.
template <int N>
__device__ __forceinline__ void fused_step(State<N> &S, float zA, float zB, float zC)
{
    float t1[N + 1], t2[N + 1], t3[N + 1];
#pragma unroll
    for (int k = 2; k <= N; ++k) t1[k] = __builtin_fmaf(zA, 1.0f / k, S.A1);
#pragma unroll
    for (int k = 2; k <= N; ++k) t2[k] = __builtin_fmaf(t1[k], zB * (1.0f / (k - 1)), S.A2);
#pragma unroll
    for (int k = 3; k <= N; ++k) t3[k] = __builtin_fmaf(t2[k], zC * (1.0f / (k - 2)), S.A3);

    f4 t4[N + 1];
#pragma unroll
    for (int k = N; k >= 4; --k) t4[k] = outer4(t3[k], zC * (1.0f / (k - 3)), S.A4[0]);

    if constexpr (N >= 5) {
        f4 t5[N + 1][4];
#pragma unroll
        for (int k = N; k >= 5; --k)
#pragma unroll
            for (int g = 0; g < 4; ++g) t5[k][g] = outer4(t4[k][g], zC * (1.0f / (k - 4)), S.A5[g]);
        if constexpr (N >= 6) {
#pragma unroll
            for (int g = 0; g < 16; ++g) S.A6[g] = outer4(t5[6][g >> 2][g & 3], zC, S.A6[g]);
        }
#pragma unroll
        for (int g = 0; g < 4; ++g) S.A5[g] = t5[5][g];
    }
    S.A4[0] = t4[4];
    S.A3 = t3[3];
    S.A2 = t2[2];
    S.A1 += zA;
}

template <int N>
__global__ void __launch_bounds__(64)
sig_mfma_d4_kernel(const float *__restrict__ path, float *__restrict__ out, int64_t L, int64_t n_inc, int basepoint)
{
    static_assert(N >= 4 && N <= 6, "depths served by this kernel");
    __shared__ float inc[kTile * 4];

    const int lane = threadIdx.x;
    const int w1 = lane >> 4, w2 = (lane >> 2) & 3, q = lane & 3;
    const int64_t b = blockIdx.x;
    const float *x = path + b * L * 4;

    State<N> S;
    S.A4[0] = (f4){0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int g = 0; g < (N >= 5 ? 4 : 1); ++g) S.A5[g] = (f4){0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int g = 0; g < (N >= 6 ? 16 : 1); ++g) S.A6[g] = (f4){0.0f, 0.0f, 0.0f, 0.0f};

    for (int64_t t0 = 0; t0 < n_inc; t0 += kTile) {
        const int nt = int(n_inc - t0 < kTile ? n_inc - t0 : kTile);
        __syncthreads();
        for (int i = lane; i < nt * 4; i += 64) {
            const int64_t s = t0 + (i >> 2);
            const int c = i & 3;
            float hi, lo;
            if (basepoint) {
                hi = x[s * 4 + c];
                lo = s == 0 ? 0.0f : x[(s - 1) * 4 + c];
            } else {
                hi = x[(s + 1) * 4 + c];
                lo = x[s * 4 + c];
            }
            inc[i] = hi - lo;
        }
        __syncthreads();
        float zA = inc[w1], zB = inc[w2], zC = inc[q];
        for (int s = 0; s < nt; ++s) {
            const int sn = s + 1 < nt ? s + 1 : s;
            const float nA = inc[sn * 4 + w1], nB = inc[sn * 4 + w2], nC = inc[sn * 4 + q];
            fused_step<N>(S, zA, zB, zC);
            zA = nA;
            zB = nB;
            zC = nC;
        }
    }

    // store: levels concatenated, each in lexicographic word order
    constexpr int64_t S_total = (N == 4 ? 340 : N == 5 ? 1364 : 5460);
    float *o = out + b * S_total;
    if ((lane & 15) == 0) o[w1] = S.A1;
    if (q == 0) o[4 + (lane >> 2)] = S.A2;
    o[20 + lane] = S.A3;
    const int blk = lane >> 2;
#pragma unroll
    for (int r = 0; r < 4; ++r) o[84 + blk * 16 + r * 4 + q] = S.A4[0][r];
    if constexpr (N >= 5) {
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int r = 0; r < 4; ++r) o[340 + blk * 64 + g * 16 + r * 4 + q] = S.A5[g][r];
    }
    if constexpr (N >= 6) {
#pragma unroll
        for (int g = 0; g < 16; ++g)
#pragma unroll
            for (int r = 0; r < 4; ++r) o[1364 + blk * 256 + g * 16 + r * 4 + q] = S.A6[g][r];
    }
}

}  // namespace

const char *mfma_kernel_name(const Shape &sh)
{
    if (sh.d == 4 && sh.N >= 4 && sh.N <= 6 && !sh.stream && sh.B <= 0x7fffffff) return "mfma_d4";
    return nullptr;
}

hipError_t launch_mfma_f32(const Shape &sh, const float *path, float *out, hipStream_t st)
{
    if (mfma_kernel_name(sh) == nullptr) return hipErrorNotSupported;
    const dim3 grid(static_cast<unsigned>(sh.B)), block(64);
    switch (sh.N) {
        case 4: hipLaunchKernelGGL(sig_mfma_d4_kernel<4>, grid, block, 0, st, path, out, sh.L, sh.n_inc, sh.basepoint); break;
        case 5: hipLaunchKernelGGL(sig_mfma_d4_kernel<5>, grid, block, 0, st, path, out, sh.L, sh.n_inc, sh.basepoint); break;
        case 6: hipLaunchKernelGGL(sig_mfma_d4_kernel<6>, grid, block, 0, st, path, out, sh.L, sh.n_inc, sh.basepoint); break;
        default: return hipErrorNotSupported;
    }
    return hipGetLastError();
}

}  // namespace sig
