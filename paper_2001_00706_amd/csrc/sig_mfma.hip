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
//   level 2, 3 (plain VALU, one scalar per lane, level 2 replicated over q):
//       A_2[w_1 w_2], A_3[w_1 w_2 q]   (q = w_3)
//   level k >= 4 (matrix cores): 4^(k-4) groups of 4 registers; group g holds the words
//       whose letters w_3..w_{k-2} spell g in base 4; register r of the group is letter
//       w_{k-1} = r; lane q is the last letter w_k = q; the block index (lane / 4) is w_1 w_2.
// With this layout the D registers of a level-k stage are, as they stand, the A operand of
// the level-(k+1) stage (register r of group g feeds group 4g + r), and the B operand is
// always z[lane & 3] times a reciprocal, so no data ever moves between lanes.
//
// Level 1 is not carried at all: A_1 after s increments is the displacement x_s - x_first, so the
// innermost Horner terms z/k + A_1 of all target levels are tabulated, with the scaled increments
// z/m, when a tile of points is staged in LDS.
//
// Levels are updated highest first; the temporaries T^(i) of a higher target level are
// formed from the old A_i before A_i itself is overwritten, so the update is in place.
//
// A lone wavefront on a SIMD issues in order and its vector and matrix-core instructions do not
// overlap (alternating them is slower than running them in blocks), so the kernel is bound by
// its instruction count: a step is 9 vector FMAs, 5 LDS reads and 27 outer products at N = 6.
#include "sig_internal.h"
#include "sig_mfma_common.h"

namespace sig {
namespace {

// Scalars in a depth-N signature over 4 channels, and the offset of each level.
template <int N>
constexpr int kChannels = (N == 4 ? 340 : N == 5 ? 1364 : 5460);
constexpr int kOff4 = 84, kOff5 = 340, kOff6 = 1364;

// One staged increment is 64 floats (in a row of 68): for each channel c, 8 floats t1[c][k-2] = z[c]/k + A_1[c]
// (k = 2..N, padded) at c*8, then 8 floats zs[c][m-1] = z[c]/m (m = 1..N-1, padded) at 32 + c*8.
constexpr int kRow = 68;  // 64 used + 4 of padding: rows land on different LDS banks when 64 lanes write one row each
constexpr int kTile = 64;  // increments staged in LDS at a time (one per lane)

template <int N>
constexpr int kLdsFloats = (kTile * kRow > kChannels<N> ? kTile * kRow : kChannels<N>);

template <int N>
struct State {
    float A2 = 0.0f, A3 = 0.0f;
    f4 A4[1];
    f4 A5[N >= 5 ? 4 : 1];
    f4 A6[N >= 6 ? 16 : 1];
};

// This lane's view of one staged increment.
template <int N>
struct Row {
    float t1[N + 1];  // t1[k] = z[w_1]/k + A_1[w_1], k = 2..N
    float zB[N];      // zB[m] = z[w_2]/m, m = 1..N-1
    float zC[N];      // zC[m] = z[q]/m,   m = 1..N-2
};

template <int N>
__device__ __forceinline__ Row<N> load_row(const float *row, int w1, int w2, int q)
{
    Row<N> R;
#pragma unroll
    for (int k = 2; k <= N; ++k) R.t1[k] = row[w1 * 8 + (k - 2)];
#pragma unroll
    for (int m = 1; m <= N - 1; ++m) R.zB[m] = row[32 + w2 * 8 + (m - 1)];
#pragma unroll
    for (int m = 1; m <= N - 2; ++m) R.zC[m] = row[32 + q * 8 + (m - 1)];
    return R;
}

// One fused multiply-exponentiate A <- A [x] exp(z) on levels 2..N.
template <int N>
__device__ __forceinline__ void fused_step(State<N> &S, const Row<N> &R)
{
    // levels 2 and 3, one scalar per lane
    float t2[N + 1], t3[N + 1];
#pragma unroll
    for (int k = 2; k <= N; ++k) t2[k] = __builtin_fmaf(R.t1[k], R.zB[k - 1], S.A2);
#pragma unroll
    for (int k = 3; k <= N; ++k) t3[k] = __builtin_fmaf(t2[k], R.zC[k - 2], S.A3);
    S.A3 = t3[3];
    S.A2 = t2[2];

    // levels 4..N: outer products on the matrix cores; higher targets first, so that each A_i is
    // read by every stage that needs its old value before it is overwritten
    f4 t4[N + 1];
#pragma unroll
    for (int k = N; k >= 5; --k) t4[k] = outer4(t3[k], R.zC[k - 3], S.A4[0]);
    S.A4[0] = outer4(t3[4], R.zC[1], S.A4[0]);
    if constexpr (N >= 5) {
        f4 t5[4];
        if constexpr (N >= 6) {
#pragma unroll
            for (int g = 0; g < 4; ++g) t5[g] = outer4(t4[6][g], R.zC[2], S.A5[g]);
        }
#pragma unroll
        for (int g = 0; g < 4; ++g) S.A5[g] = outer4(t4[5][g], R.zC[1], S.A5[g]);
        if constexpr (N >= 6) {
#pragma unroll
            for (int g = 0; g < 16; ++g) S.A6[g] = outer4(t5[g >> 2][g & 3], R.zC[1], S.A6[g]);
        }
    }
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
sig_mfma_d4_kernel(const float *__restrict__ path, float *__restrict__ out, int64_t L, int64_t n_inc_total, int basepoint,
                   const float *__restrict__ bpv, int chunks, int64_t chunk_len)
{
    static_assert(N >= 4 && N <= 6, "depths served by this kernel");
    __shared__ __align__(16) float lds[kLdsFloats<N>];

    const int lane = threadIdx.x;
    const int w1 = lane >> 4, w2 = (lane >> 2) & 3, q = lane & 3;
    const int64_t b = blockIdx.x;   // output row: a path, or one chunk of a path
    const ChunkView cv = chunk_view(b, chunks, chunk_len, n_inc_total);
    const int64_t n_inc = cv.n;
    const f4 *x4 = reinterpret_cast<const f4 *>(path) + cv.path * L;  // point l of this path
    const f4 zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
    // the point before the first increment: the path's first point, or the basepoint (the origin unless given),
    // or the point a later chunk starts from
    const f4 x_base = bpv != nullptr ? reinterpret_cast<const f4 *>(bpv)[cv.path] : zero4;
    const int64_t i_first = basepoint ? cv.inc0 - 1 : cv.inc0;
    const f4 x_first = n_inc == 0 ? zero4 : i_first >= 0 ? x4[i_first] : x_base;

    State<N> S;
    S.A4[0] = zero4;
#pragma unroll
    for (int g = 0; g < (N >= 5 ? 4 : 1); ++g) S.A5[g] = zero4;
#pragma unroll
    for (int g = 0; g < (N >= 6 ? 16 : 1); ++g) S.A6[g] = zero4;

    // the two points around increment number s (zeros past the end of the path); the points of a
    // tile are fetched while the tile before it is being scanned
    f4 p_hi, p_lo;
    auto fetch_points = [&](int64_t s) {
        p_hi = p_lo = zero4;
        if (s < n_inc) {
            const int64_t i_hi = cv.inc0 + (basepoint ? s : s + 1);
            p_hi = x4[i_hi];
            p_lo = i_hi > 0 ? x4[i_hi - 1] : x_base;
        }
    };
    fetch_points(lane);

    for (int64_t t0 = 0; t0 < n_inc; t0 += kTile) {
        const int nt = int(n_inc - t0 < kTile ? n_inc - t0 : kTile);
        __syncthreads();
        if (lane < nt) {
            // lane i stages increment t0 + i: z = hi - lo, and A_1 before it = lo - x_first
            const f4 z = p_hi - p_lo;
            const f4 a1 = p_lo - x_first;
            float *row = lds + lane * kRow;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                f4 lo4, hi4 = zero4, zlo, zhi = zero4;
                lo4[0] = __builtin_fmaf(z[c], 1.0f / 2, a1[c]);
                lo4[1] = __builtin_fmaf(z[c], 1.0f / 3, a1[c]);
                lo4[2] = __builtin_fmaf(z[c], 1.0f / 4, a1[c]);
                lo4[3] = __builtin_fmaf(z[c], 1.0f / 5, a1[c]);
                hi4[0] = __builtin_fmaf(z[c], 1.0f / 6, a1[c]);
                zlo[0] = z[c];
                zlo[1] = z[c] * (1.0f / 2);
                zlo[2] = z[c] * (1.0f / 3);
                zlo[3] = z[c] * (1.0f / 4);
                zhi[0] = z[c] * (1.0f / 5);
                f4 *r4 = reinterpret_cast<f4 *>(row + c * 8);
                r4[0] = lo4;
                r4[1] = hi4;
                r4[8] = zlo;
                r4[9] = zhi;
            }
        }
        __syncthreads();
        fetch_points(t0 + kTile + lane);
        // four increments per trip: their rows are fetched from LDS together, so the LDS latency
        // is paid once per trip and no register is copied between trips
        int s = 0;
        for (; s + 4 <= nt; s += 4) {
            Row<N> R[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) R[i] = load_row<N>(lds + (s + i) * kRow, w1, w2, q);
#pragma unroll
            for (int i = 0; i < 4; ++i) fused_step<N>(S, R[i]);
        }
        for (; s < nt; ++s) fused_step<N>(S, load_row<N>(lds + s * kRow, w1, w2, q));
    }

    // level 1 is the total displacement
    const f4 a1 = n_inc == 0 ? zero4 : x4[i_first + n_inc] - x_first;

    // park the state in LDS in word order, then copy it out 16 bytes per lane, fully coalesced
    __syncthreads();
    if (lane == 0) *reinterpret_cast<f4 *>(lds) = a1;
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
    if (sh.d != 4 || sh.stream || sh.B > 0x7fffffff) return nullptr;
    return (sh.N >= 4 && sh.N <= 6) ? "mfma_d4" : nullptr;
}

hipError_t launch_mfma_f32(const Shape &sh, const float *path, float *out, hipStream_t st)
{
    if (mfma_kernel_name(sh) == nullptr) return hipErrorNotSupported;
    const dim3 grid(static_cast<unsigned>(sh.B)), block(64);
    const float *bpv = static_cast<const float *>(sh.basepoint_value);
    switch (sh.N) {
        case 4: hipLaunchKernelGGL(sig_mfma_d4_kernel<4>, grid, block, 0, st, path, out, sh.L, sh.n_inc, sh.basepoint, bpv, sh.chunks, sh.chunk_len); break;
        case 5: hipLaunchKernelGGL(sig_mfma_d4_kernel<5>, grid, block, 0, st, path, out, sh.L, sh.n_inc, sh.basepoint, bpv, sh.chunks, sh.chunk_len); break;
        case 6: hipLaunchKernelGGL(sig_mfma_d4_kernel<6>, grid, block, 0, st, path, out, sh.L, sh.n_inc, sh.basepoint, bpv, sh.chunks, sh.chunk_len); break;
        default: return hipErrorNotSupported;
    }
    return hipGetLastError();
}

}  // namespace sig
