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
#include "sig_mfma_common.h"

namespace sig {
namespace {

// Scalars in a depth-N signature over 4 channels, and the offset of each level.
template <int N>
constexpr int kChannels = (N == 4 ? 340 : N == 5 ? 1364 : 5460);
constexpr int kOff4 = 84, kOff5 = 340, kOff6 = 1364;

// Increments staged in LDS at a time.  Each staged increment takes 4*(N-1) floats (z/1 .. z/(N-1)).
template <int N>
constexpr int kTile = (N == 6 ? 256 : 64);

template <int N>
constexpr int kLdsFloats = (kTile<N> * 4 * (N - 1) > kChannels<N> ? kTile<N> * 4 * (N - 1) : kChannels<N>);

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

// Levels 1..3 of one fused multiply-exponentiate A <- A [x] exp(z), one scalar per lane, and
// the level-3 Horner terms t3[k] = T_k^(3) of the higher targets k = 4..N.
template <int N>
__device__ __forceinline__ void low_levels(State<N> &S, const Row<N> &R, float (&t3)[N + 1])
{
    float t1[N + 1], t2[N + 1];
#pragma unroll
    for (int k = 2; k <= N; ++k) t1[k] = __builtin_fmaf(R.zA, 1.0f / k, S.A1);
#pragma unroll
    for (int k = 2; k <= N; ++k) t2[k] = __builtin_fmaf(t1[k], R.zB[k - 1], S.A2);
#pragma unroll
    for (int k = 3; k <= N; ++k) t3[k] = __builtin_fmaf(t2[k], R.zC[k - 2], S.A3);
    S.A3 = t3[3];
    S.A2 = t2[2];
    S.A1 += R.zA;
}

// Levels 4..N: outer products on the matrix cores; higher targets first, so that each A_i is
// read by every stage that needs its old value before it is overwritten.  zC[m] = z[q]/m.
template <int N>
__device__ __forceinline__ void high_levels(State<N> &S, const float (&t3)[N + 1], const float *zC)
{
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
}

// One fused multiply-exponentiate A <- A [x] exp(z).
template <int N>
__device__ __forceinline__ void fused_step(State<N> &S, const Row<N> &R)
{
    float t3[N + 1];
    low_levels<N>(S, R, t3);
    high_levels<N>(S, t3, R.zC);
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

// ---------------------------------------------------------------------------------------------
// Two wavefronts per path.
//
// A lone wavefront on a SIMD issues roughly one instruction every 8 clocks whatever its kind, so
// the one-wavefront kernel above is bound by its instruction count, not by the matrix cores.  Here
// the work of a path is cut along its only one-way dependency: wavefront 1 (the producer) folds
// each increment into levels 1..3 and hands the level-3 Horner terms t3[k], k = 4..N, over
// through LDS; wavefront 0 (the consumer) owns levels 4..N and does nothing but outer products.
// Nothing flows back, so the producer simply runs one chunk of increments ahead.  Both
// wavefronts run the same loop with one workgroup barrier per trip, hence cannot fall out of step.
constexpr int kChunk = 4;      // increments per hand-over
constexpr int kPairTile = 64;  // increments per staged LDS tile; two tiles are used alternately

template <int N>
struct PairLds {
    static constexpr int kRow = 4 * (N - 1);                    // floats per staged increment
    static constexpr int kTab = 2 * kPairTile * kRow;           // two tiles of scaled increments
    static constexpr int kRec = N - 3;                          // floats per lane handed over per increment
    static constexpr int kXchg = 2 * kChunk * 64 * kRec;        // two chunks of hand-over records
    static constexpr int kFloats = (kTab + kXchg > kChannels<N> ? kTab + kXchg : kChannels<N>);
};

// Producer side of one chunk: `rows` points at the chunk's first staged increment, `rec` at this
// lane's slot of the chunk's first hand-over record.  FULL: the chunk has all kChunk increments.
template <int N, bool FULL>
__device__ __forceinline__ void produce_chunk(State<N> &S, const float *rows, float *rec, int ns, int w1, int w2, int q)
{
    constexpr int kRow = 4 * (N - 1), kRec = N - 3;
    Row<N> R[kChunk];
#pragma unroll
    for (int i = 0; i < kChunk; ++i) R[i] = load_row<N>(rows + (FULL || i < ns ? i : 0) * kRow, w1, w2, q);
#pragma unroll
    for (int i = 0; i < kChunk; ++i) {
        if (FULL || i < ns) {
            float t3[N + 1];
            low_levels<N>(S, R[i], t3);
#pragma unroll
            for (int k = 4; k <= N; ++k) rec[i * 64 * kRec + (k - 4)] = t3[k];
        }
    }
}

// Consumer side of one chunk.
template <int N, bool FULL>
__device__ __forceinline__ void consume_chunk(State<N> &S, const float *rows, const float *rec, int ns, int q)
{
    constexpr int kRow = 4 * (N - 1), kRec = N - 3;
    float t3[kChunk][N + 1], zC[kChunk][N];
#pragma unroll
    for (int i = 0; i < kChunk; ++i) {
        const int ii = FULL || i < ns ? i : 0;
#pragma unroll
        for (int k = 4; k <= N; ++k) t3[i][k] = rec[ii * 64 * kRec + (k - 4)];
#pragma unroll
        for (int m = 1; m <= N - 3; ++m) zC[i][m] = rows[ii * kRow + (m - 1) * 4 + q];
    }
#pragma unroll
    for (int i = 0; i < kChunk; ++i)
        if (FULL || i < ns) high_levels<N>(S, t3[i], zC[i]);
}

template <int N>
__global__ void __launch_bounds__(128)
sig_mfma_d4_pair_kernel(const float *__restrict__ path, float *__restrict__ out, int64_t L, int64_t n_inc, int basepoint)
{
    static_assert(N >= 5 && N <= 6, "depths served by this kernel");
    using Lds = PairLds<N>;
    constexpr int kRow = Lds::kRow, kRec = Lds::kRec;
    __shared__ __align__(16) float lds[Lds::kFloats];
    float *tab = lds;
    float *xchg = lds + Lds::kTab;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const bool producer = __builtin_amdgcn_readfirstlane(tid >> 6) == 1;
    const int w1 = lane >> 4, w2 = (lane >> 2) & 3, q = lane & 3;
    const int64_t b = blockIdx.x;
    const f4 *x4 = reinterpret_cast<const f4 *>(path) + b * L;  // point l of this path

    State<N> S;
    S.A4[0] = (f4){0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int g = 0; g < 4; ++g) S.A5[g] = (f4){0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int g = 0; g < (N >= 6 ? 16 : 1); ++g) S.A6[g] = (f4){0.0f, 0.0f, 0.0f, 0.0f};

    // producer: the two points around increment number s (zeros past the end of the path)
    f4 p_hi = (f4){0.0f, 0.0f, 0.0f, 0.0f}, p_lo = p_hi;
    auto fetch_points = [&](int64_t s) {
        p_hi = p_lo = (f4){0.0f, 0.0f, 0.0f, 0.0f};
        if (s < n_inc) {
            const int64_t i_hi = basepoint ? s : s + 1;
            p_hi = x4[i_hi];
            if (i_hi > 0) p_lo = x4[i_hi - 1];
        }
    };
    if (producer) fetch_points(lane);

    const int64_t n_chunks = (n_inc + kChunk - 1) / kChunk;
    for (int64_t c = 0; c <= n_chunks; ++c) {
        if (producer) {
            if (c < n_chunks) {
                const int64_t s0 = c * kChunk;
                const int in_tile = int(s0 % kPairTile);
                float *tile = tab + int((s0 / kPairTile) & 1) * (kPairTile * kRow);
                if (in_tile == 0) {
                    // stage this tile from the points fetched one tile ago, then fetch the next tile's
                    if (s0 + lane < n_inc) {
                        const f4 z = p_hi - p_lo;
                        f4 *row = reinterpret_cast<f4 *>(tile + lane * kRow);
                        row[0] = z;
#pragma unroll
                        for (int m = 2; m <= N - 1; ++m) row[m - 1] = z * (1.0f / m);
                    }
                    fetch_points(s0 + kPairTile + lane);
                }
                const int ns = int(n_inc - s0 < kChunk ? n_inc - s0 : kChunk);
                float *rec = xchg + (int(c & 1) * kChunk * 64 + lane) * kRec;
                if (ns == kChunk) {
                    produce_chunk<N, true>(S, tile + in_tile * kRow, rec, kChunk, w1, w2, q);
                } else {
                    produce_chunk<N, false>(S, tile + in_tile * kRow, rec, ns, w1, w2, q);
                }
            }
        } else {
            if (c > 0) {
                const int64_t s0 = (c - 1) * kChunk;
                const int in_tile = int(s0 % kPairTile);
                const float *tile = tab + int((s0 / kPairTile) & 1) * (kPairTile * kRow);
                const int ns = int(n_inc - s0 < kChunk ? n_inc - s0 : kChunk);
                const float *rec = xchg + (int((c - 1) & 1) * kChunk * 64 + lane) * kRec;
                if (ns == kChunk) {
                    consume_chunk<N, true>(S, tile + in_tile * kRow, rec, kChunk, q);
                } else {
                    consume_chunk<N, false>(S, tile + in_tile * kRow, rec, ns, q);
                }
            }
        }
        __syncthreads();
    }

    // park the state in LDS in word order (levels 1..3 from the producer, the rest from the
    // consumer), then both wavefronts copy it out 16 bytes per lane
    const int blk = lane >> 2;
    if (producer) {
        if ((lane & 15) == 0) lds[w1] = S.A1;
        if (q == 0) lds[4 + (lane >> 2)] = S.A2;
        lds[20 + lane] = S.A3;
    } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) lds[kOff4 + park4(blk * 16 + r * 4 + q)] = S.A4[0][r];
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int r = 0; r < 4; ++r) lds[kOff5 + park5(blk * 64 + g * 16 + r * 4 + q)] = S.A5[g][r];
        if constexpr (N >= 6) {
#pragma unroll
            for (int g = 0; g < 16; ++g)
#pragma unroll
                for (int r = 0; r < 4; ++r) lds[kOff6 + park6(blk * 256 + g * 16 + r * 4 + q)] = S.A6[g][r];
        }
    }
    __syncthreads();
    f4 *o4 = reinterpret_cast<f4 *>(out + b * kChannels<N>);
    for (int j = tid; j < kChannels<N> / 4; j += 128) {
        const int i = 4 * j;
        const int at = i < kOff4 ? i : i < kOff5 ? kOff4 + park4(i - kOff4) : i < kOff6 ? kOff5 + park5(i - kOff5) : kOff6 + park6(i - kOff6);
        o4[j] = *reinterpret_cast<const f4 *>(lds + at);
    }
}

}  // namespace

const char *mfma_kernel_name(const Shape &sh, bool pair)
{
    if (sh.d != 4 || sh.stream || sh.B > 0x7fffffff) return nullptr;
    if (pair) return (sh.N == 5 || sh.N == 6) ? "mfma_d4_pair" : nullptr;
    return (sh.N >= 4 && sh.N <= 6) ? "mfma_d4" : nullptr;
}

hipError_t launch_mfma_f32(const Shape &sh, bool pair, const float *path, float *out, hipStream_t st)
{
    if (mfma_kernel_name(sh, pair) == nullptr) return hipErrorNotSupported;
    const dim3 grid(static_cast<unsigned>(sh.B));
    if (pair) {
        const dim3 block(128);
        if (sh.N == 5) hipLaunchKernelGGL(sig_mfma_d4_pair_kernel<5>, grid, block, 0, st, path, out, sh.L, sh.n_inc, sh.basepoint);
        else hipLaunchKernelGGL(sig_mfma_d4_pair_kernel<6>, grid, block, 0, st, path, out, sh.L, sh.n_inc, sh.basepoint);
        return hipGetLastError();
    }
    const dim3 block(64);
    switch (sh.N) {
        case 4: hipLaunchKernelGGL(sig_mfma_d4_kernel<4>, grid, block, 0, st, path, out, sh.L, sh.n_inc, sh.basepoint); break;
        case 5: hipLaunchKernelGGL(sig_mfma_d4_kernel<5>, grid, block, 0, st, path, out, sh.L, sh.n_inc, sh.basepoint); break;
        case 6: hipLaunchKernelGGL(sig_mfma_d4_kernel<6>, grid, block, 0, st, path, out, sh.L, sh.n_inc, sh.basepoint); break;
        default: return hipErrorNotSupported;
    }
    return hipGetLastError();
}

}  // namespace sig
