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
//
// A single wavefront issues in order, and on this chip vector and matrix-core instructions of
// one wavefront do not overlap (alternating them is slower than running them in blocks), so a
// step is laid out as one block of vector work followed by one block of outer products, and the
// vector block is kept short: the scaled increments z/m come ready-made from an LDS table that
// is filled once per tile of increments.
#include "sig_internal.h"

namespace sig {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

// Scalars in a depth-N signature over 4 channels, and the offset of each level.
template <int N>
constexpr int kChannels = (N == 4 ? 340 : N == 5 ? 1364 : 5460);
constexpr int kOff4 = 84, kOff5 = 340, kOff6 = 1364;

// Increments staged in LDS at a time.  Each staged increment takes 4*(N-1) floats (z/1 .. z/(N-1)).
template <int N>
constexpr int kTile = (N == 6 ? 256 : 64);

template <int N>
constexpr int kLdsFloats = (kTile<N> * 4 * (N - 1) > kChannels<N> ? kTile<N> * 4 * (N - 1) : kChannels<N>);

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

// This lane's view of one staged increment: z[w_1], z[w_2]/m and z[q]/m.
template <int N>
struct Row {
    float zA;
    float zB[N];  // zB[m] = z[w_2]/m, m = 1..N-1
    float zC[N];  // zC[m] = z[q]/m,   m = 1..N-2
};

// `tab` points at one increment's scaled copies in LDS: tab[(m-1)*4 + c] = z[c]/m, m = 1..N-1.
template <int N>
__device__ __forceinline__ Row<N> load_row(const float *tab, int w1, int w2, int q)
{
    Row<N> R;
    R.zA = tab[w1];
#pragma unroll
    for (int m = 1; m <= N - 1; ++m) R.zB[m] = tab[(m - 1) * 4 + w2];
#pragma unroll
    for (int m = 1; m <= N - 2; ++m) R.zC[m] = tab[(m - 1) * 4 + q];
    return R;
}

// One fused multiply-exponentiate A <- A [x] exp(z).
template <int N>
__device__ __forceinline__ void fused_step(State<N> &S, const Row<N> &R)
{
    const float zA = R.zA;
    const float *zB = R.zB, *zC = R.zC;

    // low levels, one scalar per lane
    float t1[N + 1], t2[N + 1], t3[N + 1];
#pragma unroll
    for (int k = 2; k <= N; ++k) t1[k] = __builtin_fmaf(zA, 1.0f / k, S.A1);
#pragma unroll
    for (int k = 2; k <= N; ++k) t2[k] = __builtin_fmaf(t1[k], zB[k - 1], S.A2);
#pragma unroll
    for (int k = 3; k <= N; ++k) t3[k] = __builtin_fmaf(t2[k], zC[k - 2], S.A3);

    // levels 4.., outer products on the matrix cores; higher targets first, so that each A_i is
    // read by every stage that needs its old value before it is overwritten
    f4 t4[N + 1];
#pragma unroll
    for (int k = N; k >= 5; --k) t4[k] = outer4(t3[k], zC[k - 3], S.A4[0]);
    S.A4[0] = outer4(t3[4], zC[1], S.A4[0]);
    if constexpr (N >= 5) {
        f4 t5[4];
        if constexpr (N >= 6) {
#pragma unroll
            for (int g = 0; g < 4; ++g) t5[g] = outer4(t4[6][g], zC[2], S.A5[g]);
        }
#pragma unroll
        for (int g = 0; g < 4; ++g) S.A5[g] = outer4(t4[5][g], zC[1], S.A5[g]);
        if constexpr (N >= 6) {
#pragma unroll
            for (int g = 0; g < 16; ++g) S.A6[g] = outer4(t5[g >> 2][g & 3], zC[1], S.A6[g]);
        }
    }
    S.A3 = t3[3];
    S.A2 = t2[2];
    S.A1 += zA;
}

// Where word number i of a level (lexicographic) is parked in LDS on its way to `out`.  The
// registers of one store hold 4 consecutive words per lane quad and the quads are 4^(k-2) words
// apart, which would put all 16 quads on the same banks; XOR-ing the quad number into bits 2..5
// spreads them while keeping every aligned group of 4 words contiguous for the 16-byte read-back.
__device__ __forceinline__ int park4(int i) { return i ^ ((((i >> 4) >> 2) & 3) << 2); }
__device__ __forceinline__ int park5(int i) { return i ^ ((i >> 6) << 2); }
__device__ __forceinline__ int park6(int i) { return i ^ ((i >> 8) << 2); }

template <int N>
__global__ void __launch_bounds__(64)
sig_mfma_d4_kernel(const float *__restrict__ path, float *__restrict__ out, int64_t L, int64_t n_inc, int basepoint)
{
    static_assert(N >= 4 && N <= 6, "depths served by this kernel");
    __shared__ __align__(16) float lds[kLdsFloats<N>];

    const int lane = threadIdx.x;
    const int w1 = lane >> 4, w2 = (lane >> 2) & 3, q = lane & 3;
    const int64_t b = blockIdx.x;
    const f4 *x4 = reinterpret_cast<const f4 *>(path) + b * L;  // point l of this path

    State<N> S;
    S.A4[0] = (f4){0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int g = 0; g < (N >= 5 ? 4 : 1); ++g) S.A5[g] = (f4){0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int g = 0; g < (N >= 6 ? 16 : 1); ++g) S.A6[g] = (f4){0.0f, 0.0f, 0.0f, 0.0f};

    constexpr int kRow = 4 * (N - 1);  // floats per staged increment
    for (int64_t t0 = 0; t0 < n_inc; t0 += kTile<N>) {
        const int nt = int(n_inc - t0 < kTile<N> ? n_inc - t0 : kTile<N>);
        __syncthreads();
        // every lane fetches its points of the tile with independent 16-byte loads (all in
        // flight together: one memory round trip per tile), then differences, scales and stages
        constexpr int kPer = kTile<N> / 64;
        f4 hi[kPer], lo[kPer];
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const int i = lane + 64 * j;
            const int64_t s = t0 + i;  // increment number
            hi[j] = lo[j] = (f4){0.0f, 0.0f, 0.0f, 0.0f};
            if (i < nt) {
                const int64_t p_hi = basepoint ? s : s + 1;
                hi[j] = x4[p_hi];
                if (p_hi > 0) lo[j] = x4[p_hi - 1];
            }
        }
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const int i = lane + 64 * j;
            if (i < nt) {
                const f4 z = hi[j] - lo[j];
                f4 *row = reinterpret_cast<f4 *>(lds + i * kRow);
                row[0] = z;
#pragma unroll
                for (int m = 2; m <= N - 1; ++m) row[m - 1] = z * (1.0f / m);
            }
        }
        __syncthreads();
        // two increments per trip; the rows of the next two are fetched from LDS while the
        // current ones are being folded in, so the scan never waits for the LDS latency
        Row<N> r0 = load_row<N>(lds, w1, w2, q);
        Row<N> r1 = load_row<N>(lds + (nt > 1 ? kRow : 0), w1, w2, q);
        int s = 0;
        for (; s + 1 < nt; s += 2) {
            const int s2 = s + 2 < nt ? s + 2 : nt - 1, s3 = s + 3 < nt ? s + 3 : nt - 1;
            const Row<N> n0 = load_row<N>(lds + s2 * kRow, w1, w2, q);
            __builtin_amdgcn_sched_barrier(0);
            fused_step<N>(S, r0);
            const Row<N> n1 = load_row<N>(lds + s3 * kRow, w1, w2, q);
            __builtin_amdgcn_sched_barrier(0);
            fused_step<N>(S, r1);
            r0 = n0;
            r1 = n1;
        }
        if (s < nt) fused_step<N>(S, r0);
    }

    // park the state in LDS in word order, then copy it out 16 bytes per lane, fully coalesced
    __syncthreads();
    if ((lane & 15) == 0) lds[w1] = S.A1;
    if (q == 0) lds[4 + (lane >> 2)] = S.A2;
    lds[20 + lane] = S.A3;
    const int blk = lane >> 2;
#pragma unroll
    for (int r = 0; r < 4; ++r) lds[kOff4 + park4(blk * 16 + r * 4 + q)] = S.A4[0][r];
    if constexpr (N >= 5) {
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int r = 0; r < 4; ++r) lds[kOff5 + park5(blk * 64 + g * 16 + r * 4 + q)] = S.A5[g][r];
    }
    if constexpr (N >= 6) {
#pragma unroll
        for (int g = 0; g < 16; ++g)
#pragma unroll
            for (int r = 0; r < 4; ++r) lds[kOff6 + park6(blk * 256 + g * 16 + r * 4 + q)] = S.A6[g][r];
    }
    __syncthreads();
    f4 *o4 = reinterpret_cast<f4 *>(out + b * kChannels<N>);
    if (lane < kOff4 / 4) o4[lane] = *reinterpret_cast<const f4 *>(lds + lane * 4);
    o4[kOff4 / 4 + lane] = *reinterpret_cast<const f4 *>(lds + kOff4 + park4(lane * 4));
    if constexpr (N >= 5) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            o4[kOff5 / 4 + j * 64 + lane] = *reinterpret_cast<const f4 *>(lds + kOff5 + park5((j * 64 + lane) * 4));
    }
    if constexpr (N >= 6) {
#pragma unroll
        for (int j = 0; j < 16; ++j)
            o4[kOff6 / 4 + j * 64 + lane] = *reinterpret_cast<const f4 *>(lds + kOff6 + park6((j * 64 + lane) * 4));
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
