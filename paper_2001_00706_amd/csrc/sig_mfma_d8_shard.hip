// Matrix-core kernel family (fp32), d = 8 channels, depth N = 4..6, final mode, 64 independent
// wavefronts per path.
//
// Small batches of wide, deep signatures (e.g. 32 paths of 8 channels at depth 5) are bound by the
// chain of dependent increments, not by arithmetic: the only way to use the chip is to cut one path
// into many independent pieces.  The words that start with a given two-letter prefix f = f_1 f_2,
// together with f_1 and f_1 f_2 themselves, are closed under the fused multiply-exponentiate (paper
// section 4.1, eq. "fusedterm"), so each of the 64 prefixes gets a wavefront of its own that scans all
// the increments and writes its own slice of every level.
//
// Register layout of shard f (lane = 8*w_3 + w_4; as a matrix-core lane: block = lane/4, q = lane%4):
//   A_1[f_1], A_2[f_1 f_2]      the same scalar in every lane
//   A_3[f w_3], A_4[f w_3 w_4]  one scalar per lane (A_3 replicated over w_4)
//   A_5[f w_3 w_4 w_5]          2 groups (w_5 / 4) of 4 registers
//   A_6[f w_3 .. w_6]           16 groups (w_5/4, w_5%4, w_6/4) of 4 registers
// A level-k stage for k >= 5 is a batch of 4x4 outer products (v_mfma_f32_4x4x1_16b_f32): the left
// operand a[i] sits in lane 4*block + i, i.e. letter w_{k-1} % 4 with the block carrying the letters
// before it; the right operand is z[4*g + j] for the half g of the new letter.  Result register r, lane
// q hold (w_{k-1}%4, w_k%4), which is again a left operand for the next level.  The top level swaps
// the operands, so that a lane ends up with 4 consecutive words.
#include "sig_internal.h"
#include "sig_mfma_common.h"

namespace sig {
namespace {

constexpr int kD8 = 8;
constexpr int kTile8 = 64;  // increments staged in LDS at a time
constexpr int kCol8 = kTile8 + 4;   // floats between two columns of the staged table: 16-byte aligned, and the
                                    // 16-byte reads of eight different columns fall into different LDS banks

__host__ __device__ constexpr int level_off8(int k)  // offset of level k (1-based) in a d = 8 signature
{
    int off = 0, p = 1;
    for (int j = 1; j < k; ++j) {
        p *= kD8;
        off += p;
    }
    return off;
}

template <int N>
struct State8 {
    float A4 = 0.0f;
    f4 A5[2];
    f4 A6[N >= 6 ? 16 : 1];
};

// Levels 1..3 of a shard do not wait for the levels above them, and inside the shard they are running sums:
//   A_1[f_1] before increment s is a coordinate of the path itself,
//   A_2[f] = sum over earlier increments of T_2^(1) z[f_2],    T_k^(1) = z[f_1]/k + A_1,
//   A_3[f w_3] = sum over earlier increments of T_3^(2) z[w_3], T_k^(2) = T_k^(1) z[f_2]/(k-1) + A_2.
// So a whole tile of increments is handled at once, and what the sequential part of the scan needs from the low
// levels, T_k^(3)[w_3] = T_k^(2) z[w_3]/(k-2) + A_3[w_3] for k = 4..N, is tabulated in LDS next to the increment.
// Every one of the 64 shards of a path would otherwise repeat that arithmetic in each lane at each increment.
//
// The table is built in two steps.  First a lane per increment: z, T^(1), the prefix sum of level 2 over the
// wavefront, T_k^(2); z and the T_k^(2) (scaled) go to LDS.  Then a lane per (letter w_3, run of eight increments):
// the eight terms of A_3[f w_3] of the run are accumulated in registers (one multiply-add each), the run totals are
// summed over the eight runs of the letter with three lane moves, and the lane writes the table entries of its eight
// increments.  (One lane per increment for all eight letters costs eight prefix sums over the wavefront, six
// dependent lane moves each, per tile: two and a half times the instructions.)
//
// Columns of the table: z[0..7], then T_k^(3)[0..7] / (k - 3) for k = 4..N, then T_3^(2) and T_k^(2) / ((k-2)(k-3))
// for k = 4..N (read by the second step only); kTile8 increments per column.
template <int N>
constexpr int kRow8 = kD8 * (N - 2);
template <int N>
constexpr int kCols8 = kRow8<N> + (N - 2);

// DPP move that leaves 0 in the lanes of the rows (of 16 lanes) not named in ROWS and in lanes whose source lies
// outside their row.
template <int CTRL, int ROWS>
__device__ __forceinline__ float dpp_or_zero(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROWS, 0xf, false));
}

// The same with a choice of banks (groups of four lanes inside a row) that receive the moved value.
template <int CTRL, int BANKS>
__device__ __forceinline__ float dpp_banks_or_zero(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, BANKS, false));
}

// Inclusive prefix sum over the 64 lanes (lane i receives v_0 + .. + v_i): doubling steps inside each row of 16
// lanes (a shift past the start of the row brings 0), then the row totals passed on to the rows after them.
__device__ __forceinline__ float wave_inclusive_scan(float v)
{
    v += dpp_or_zero<0x111, 0xf>(v);   // row_shr:1
    v += dpp_or_zero<0x112, 0xf>(v);   // row_shr:2
    v += dpp_or_zero<0x114, 0xf>(v);   // row_shr:4
    v += dpp_or_zero<0x118, 0xf>(v);   // row_shr:8
    v += dpp_or_zero<0x142, 0xa>(v);   // row_bcast:15 into rows 1 and 3: the last lane of the row before
    v += dpp_or_zero<0x143, 0xc>(v);   // row_bcast:31 into rows 2 and 3: lane 31
    return v;
}

// Exclusive prefix sum (lane i receives v_0 + .. + v_{i-1}) and, in `total`, the sum over all lanes.
__device__ __forceinline__ float wave_exclusive_scan(float v, float &total)
{
    const float incl = wave_inclusive_scan(v);
    total = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, incl), 63));
    return incl - v;
}

// Element i (the same in every lane) of the 8 floats (a, b).
__device__ __forceinline__ float pick8(f4 a, f4 b, int i)
{
    const f4 h = (i & 4) ? b : a;
    const float lo = (i & 1) ? h[1] : h[0], hi = (i & 1) ? h[3] : h[2];
    return (i & 2) ? hi : lo;
}

// One fused multiply-exponentiate restricted to the words of this shard, levels 4..N, needs from the table of
// its increment z[w_4], z[q], z[4 + q] and t3[k] = T_k^(3)[w_3] / (k - 3) for k = 4..N (the divisor of the next
// Horner step is folded into the table).  The table is stored column by column (kTile8 increments per column, kCol8 floats apart),
// so one 16-byte LDS read brings a column's entries of four consecutive increments.
template <int N>
struct Row8 {
    float z4, zlo, zhi;
    float t3[N + 1];
};

template <int N>
struct Rows8 {   // four consecutive increments
    f4 z4, zlo, zhi;
    f4 t3[N + 1];
};

template <int N>
__device__ __forceinline__ Rows8<N> load_rows8(const float *tab, int s, int w3, int w4, int q)   // s a multiple of 4
{
    Rows8<N> R;
    R.z4 = *reinterpret_cast<const f4 *>(tab + w4 * kCol8 + s);
    R.zlo = *reinterpret_cast<const f4 *>(tab + q * kCol8 + s);
    R.zhi = *reinterpret_cast<const f4 *>(tab + (4 + q) * kCol8 + s);
#pragma unroll
    for (int k = 4; k <= N; ++k) R.t3[k] = *reinterpret_cast<const f4 *>(tab + (kD8 * (k - 3) + w3) * kCol8 + s);
    return R;
}

template <int N>
__device__ __forceinline__ Row8<N> pick_row8(const Rows8<N> &V, int i)
{
    Row8<N> R;
    R.z4 = V.z4[i];
    R.zlo = V.zlo[i];
    R.zhi = V.zhi[i];
#pragma unroll
    for (int k = 4; k <= N; ++k) R.t3[k] = V.t3[k][i];
    return R;
}

template <int N>
__device__ __forceinline__ void step8(State8<N> &S, const Row8<N> &R)
{
    float t4[N + 1];
#pragma unroll
    for (int k = 4; k <= N; ++k) t4[k] = __builtin_fmaf(R.t3[k], R.z4, S.A4);

    if constexpr (N >= 5) {
        if constexpr (N >= 6) {
            // T_6^(5), then the level-6 update (top level: operands swapped)
            f4 t5[2];
            t5[0] = outer4(t4[6], R.zlo * 0.5f, S.A5[0]);
            t5[1] = outer4(t4[6], R.zhi * 0.5f, S.A5[1]);
#pragma unroll
            for (int g5 = 0; g5 < 2; ++g5)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    S.A6[(g5 * 4 + r) * 2 + 0] = outer4(R.zlo, t5[g5][r], S.A6[(g5 * 4 + r) * 2 + 0]);
                    S.A6[(g5 * 4 + r) * 2 + 1] = outer4(R.zhi, t5[g5][r], S.A6[(g5 * 4 + r) * 2 + 1]);
                }
            S.A5[0] = outer4(t4[5], R.zlo, S.A5[0]);
            S.A5[1] = outer4(t4[5], R.zhi, S.A5[1]);
        } else {
            S.A5[0] = outer4(R.zlo, t4[5], S.A5[0]);  // top level: operands swapped
            S.A5[1] = outer4(R.zhi, t4[5], S.A5[1]);
        }
    }
    S.A4 = t4[4];
}

typedef unsigned int u4 __attribute__((ext_vector_type(4)));

template <int N>
__global__ void __launch_bounds__(64)
sig_mfma_d8_shard_kernel(const float *__restrict__ path, float *__restrict__ out, int64_t L, int64_t n_inc_total,
                         int basepoint, const float *__restrict__ bpv, int chunks, int64_t chunk_len)
{
    static_assert(N >= 4 && N <= 6, "depths served by this kernel");
    constexpr int kRow = kRow8<N>;
    constexpr int kS = level_off8(N + 1);
    __shared__ __align__(16) float lds[kCol8 * kCols8<N>];

    const int lane = threadIdx.x;
    const int w3 = lane >> 3, w4 = lane & 7, q = lane & 3;
    const int seg = lane & 7;   // while a table is built: this lane's run of eight increments, for the letter w3
    const int64_t b = blockIdx.x >> 6;   // output row: a path, or one chunk of a path
    const int f1 = (blockIdx.x >> 3) & 7, f2 = blockIdx.x & 7;
    const ChunkView cv = chunk_view(b, chunks, chunk_len, n_inc_total);
    const int64_t n_inc = cv.n;
    const f4 *x4 = reinterpret_cast<const f4 *>(path) + cv.path * L * 2;  // 2 pieces of 16 bytes per point
    float *o = out + b * kS;
    const f4 zero4 = {0.0f, 0.0f, 0.0f, 0.0f};

    State8<N> S;
    S.A5[0] = S.A5[1] = zero4;
#pragma unroll
    for (int g = 0; g < (N >= 6 ? 16 : 1); ++g) S.A6[g] = zero4;

    // the point the scan starts from: the chunk's first point, or the basepoint (the origin unless given)
    f4 base0 = zero4, base1 = zero4;
    if (bpv != nullptr) {
        base0 = reinterpret_cast<const f4 *>(bpv)[cv.path * 2];
        base1 = reinterpret_cast<const f4 *>(bpv)[cv.path * 2 + 1];
    }
    const int64_t i_first = basepoint ? cv.inc0 - 1 : cv.inc0;
    float x_first = 0.0f, x_last = 0.0f;   // coordinate f_1 of the first and last point of the scan
    if (n_inc > 0) {
        x_first = i_first >= 0 ? pick8(x4[i_first * 2], x4[i_first * 2 + 1], f1) : pick8(base0, base1, f1);
        x_last = pick8(x4[(i_first + n_inc) * 2], x4[(i_first + n_inc) * 2 + 1], f1);
    }
    float A2 = 0.0f;   // A_2[f] before the current tile
    float A3 = 0.0f;   // A_3[f w3] before the current tile

    // the two points around increment number s (zeros past the end of the scan); the points of a
    // tile are fetched while the tile before it is being scanned
    struct Points {
        f4 hi0, hi1, lo0, lo1;
    };
    auto fetch_points = [&](int64_t s) {
        Points P;
        P.hi0 = P.hi1 = P.lo0 = P.lo1 = zero4;
        if (s < n_inc) {
            const int64_t i_hi = cv.inc0 + (basepoint ? s : s + 1);
            P.hi0 = x4[i_hi * 2];
            P.hi1 = x4[i_hi * 2 + 1];
            if (i_hi > 0) {
                P.lo0 = x4[(i_hi - 1) * 2];
                P.lo1 = x4[(i_hi - 1) * 2 + 1];
            } else {
                P.lo0 = base0;
                P.lo1 = base1;
            }
        }
        return P;
    };
    Points P0 = fetch_points(lane);

    for (int64_t t0 = 0; t0 < n_inc; t0 += kTile8) {
        const int nt = int(n_inc - t0 < kTile8 ? n_inc - t0 : kTile8);
        __syncthreads();
        {
            // first step, lane r = increment t0 + r; lanes past the end of the scan carry zero increments, which
            // add nothing to the running sums (their table entries are never read)
            const f4 z0 = P0.hi0 - P0.lo0, z1 = P0.hi1 - P0.lo1;
            const float zf1 = pick8(z0, z1, f1), zf2 = pick8(z0, z1, f2);
            const float a1 = lane < nt ? pick8(P0.lo0, P0.lo1, f1) - x_first : 0.0f;   // A_1[f_1] before this increment
            float t1[N + 1], t2[N + 1];
#pragma unroll
            for (int k = 2; k <= N; ++k) t1[k] = __builtin_fmaf(zf1, 1.0f / k, a1);
            float sum2;
            const float a2 = A2 + wave_exclusive_scan(t1[2] * zf2, sum2);
            A2 += sum2;
#pragma unroll
            for (int k = 3; k <= N; ++k) t2[k] = __builtin_fmaf(t1[k], zf2 * (1.0f / (k - 1)), a2);
#pragma unroll
            for (int w = 0; w < kD8; ++w) lds[w * kCol8 + lane] = w < 4 ? z0[w & 3] : z1[w & 3];
            lds[kRow * kCol8 + lane] = t2[3];
#pragma unroll
            for (int k = 4; k <= N; ++k) lds[(kRow + k - 3) * kCol8 + lane] = t2[k] * (1.0f / ((k - 2) * (k - 3)));
        }
        __syncthreads();
        {
            // second step, lane (w3, seg): increments 8 seg .. 8 seg + 7 of the tile, letter w3
            const float *zc = lds + w3 * kCol8 + 8 * seg, *tc = lds + kRow * kCol8 + 8 * seg;
            const f4 za = *reinterpret_cast<const f4 *>(zc), zb = *reinterpret_cast<const f4 *>(zc + 4);
            const f4 ta = *reinterpret_cast<const f4 *>(tc), tb = *reinterpret_cast<const f4 *>(tc + 4);
            float zz[8], p[8];   // p[j]: the terms of A_3[f w3] of the run up to and with increment j
#pragma unroll
            for (int j = 0; j < 8; ++j) zz[j] = j < 4 ? za[j & 3] : zb[j & 3];
            p[0] = ta[0] * zz[0];
#pragma unroll
            for (int j = 1; j < 8; ++j) p[j] = __builtin_fmaf(j < 4 ? ta[j & 3] : tb[j & 3], zz[j], p[j - 1]);
            // totals of the runs before this one (the eight runs of a letter sit in eight consecutive lanes)
            float incl = p[7], moved;
            moved = dpp_or_zero<0x111, 0xf>(incl);   // row_shr:1
            incl += seg >= 1 ? moved : 0.0f;
            moved = dpp_or_zero<0x112, 0xf>(incl);   // row_shr:2
            incl += seg >= 2 ? moved : 0.0f;
            incl += dpp_banks_or_zero<0x114, 0xa>(incl);   // row_shr:4 into the upper half of each group of eight
            const float total = __builtin_bit_cast(
                float, __builtin_amdgcn_ds_bpermute(4 * (lane | 7), __builtin_bit_cast(int, incl)));
            const float before = A3 + (incl - p[7]);
            A3 += total;
            float a3[8];   // A_3[f w3] before increment j of the run
            a3[0] = before;
#pragma unroll
            for (int j = 1; j < 8; ++j) a3[j] = before + p[j - 1];
#pragma unroll
            for (int k = 4; k <= N; ++k) {
                const float *uc = lds + (kRow + k - 3) * kCol8 + 8 * seg;
                const f4 ua = *reinterpret_cast<const f4 *>(uc), ub = *reinterpret_cast<const f4 *>(uc + 4);
                f4 ea, eb;   // T_k^(3)[w3] / (k - 3)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    ea[j] = __builtin_fmaf(ua[j], zz[j], k == 4 ? a3[j] : a3[j] * (1.0f / (k - 3)));
                    eb[j] = __builtin_fmaf(ub[j], zz[4 + j], k == 4 ? a3[4 + j] : a3[4 + j] * (1.0f / (k - 3)));
                }
                float *ec = lds + (kD8 * (k - 3) + w3) * kCol8 + 8 * seg;
                *reinterpret_cast<f4 *>(ec) = ea;
                *reinterpret_cast<f4 *>(ec + 4) = eb;
            }
        }
        __syncthreads();
        P0 = fetch_points(t0 + kTile8 + lane);
        // The tile is walked in rounds of four increments, the next four fetched from LDS while these are folded in
        // (two sets of registers taking turns, so that nothing is copied).  The rows past the end of the scan hold
        // zero increments, which leave the state as it is (T z + A with z = 0), so the last round needs no shorter
        // variant.
        const int nr = (nt + 3) & ~3;
        int s = 0;
        Rows8<N> V0 = load_rows8<N>(lds, 0, w3, w4, q);
        for (; s + 12 <= nr; s += 8) {
            const Rows8<N> V1 = load_rows8<N>(lds, s + 4, w3, w4, q);
            __builtin_amdgcn_sched_barrier(0);   // the reads are issued before the arithmetic they hide behind
#pragma unroll
            for (int i = 0; i < 4; ++i) step8<N>(S, pick_row8<N>(V0, i));
            V0 = load_rows8<N>(lds, s + 8, w3, w4, q);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 4; ++i) step8<N>(S, pick_row8<N>(V1, i));
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) step8<N>(S, pick_row8<N>(V0, i));
        s += 4;
        if (s < nr) {
            const Rows8<N> V1 = load_rows8<N>(lds, s, w3, w4, q);
#pragma unroll
            for (int i = 0; i < 4; ++i) step8<N>(S, pick_row8<N>(V1, i));
        }
    }
    // store this shard's slice of every level
    const int f = f1 * 8 + f2;
    if (f2 == 0 && lane == 0) o[f1] = x_last - x_first;   // level 1 is the total displacement
    if (lane == 0) o[level_off8(2) + f] = A2;
    if (w4 == 0) o[level_off8(3) + f * 8 + w3] = A3;
    o[level_off8(4) + f * 64 + lane] = S.A4;
    if constexpr (N == 5) {
        // register r, lane (block, q) of group g: word 8*(lane/4 * 4 + q) + 4*g + r of the 512-word slice
        f4 *o5 = reinterpret_cast<f4 *>(o + level_off8(5) + f * 512);
#pragma unroll
        for (int g = 0; g < 2; ++g) o5[lane * 2 + g] = S.A5[g];
    }
    if constexpr (N == 6) {
        // level 5 in chaining orientation: register r = w_4 % 4, lane q = w_5 % 4
        float *o5 = o + level_off8(5) + f * 512;
#pragma unroll
        for (int g = 0; g < 2; ++g)
#pragma unroll
            for (int r = 0; r < 4; ++r) o5[(w3 * 8 + 4 * ((lane >> 2) & 1) + r) * 8 + 4 * g + q] = S.A5[g][r];
        // level 6 (swapped): group (g5, r5, g6), register r = w_6 % 4, lane q = w_5 % 4
        f4 *o6 = reinterpret_cast<f4 *>(o + level_off8(6) + f * 4096);
#pragma unroll
        for (int g5 = 0; g5 < 2; ++g5)
#pragma unroll
            for (int r5 = 0; r5 < 4; ++r5)
#pragma unroll
                for (int g6 = 0; g6 < 2; ++g6) {
                    const int w4v = 4 * ((lane >> 2) & 1) + r5, w5v = 4 * g5 + q;
                    o6[(((w3 * 8 + w4v) * 8 + w5v) * 8 + 4 * g6) / 4] = S.A6[(g5 * 4 + r5) * 2 + g6];
                }
    }
}

template <int N>
hipError_t launch8(const Shape &sh, const float *path, float *out, hipStream_t st)
{
    hipLaunchKernelGGL(sig_mfma_d8_shard_kernel<N>, dim3(static_cast<unsigned>(sh.B * 64)), dim3(64), 0, st, path, out,
                       sh.L, sh.n_inc, sh.basepoint, static_cast<const float *>(sh.basepoint_value), sh.chunks, sh.chunk_len);
    return hipGetLastError();
}

}  // namespace

const char *mfma_d8_kernel_name(const Shape &sh)
{
    if (sh.d != 8 || sh.N < 4 || sh.N > 6 || sh.stream || sh.B > 0x1ffffff) return nullptr;
    return "mfma_d8_shard";
}

hipError_t launch_mfma_d8_f32(const Shape &sh, const float *path, float *out, hipStream_t st)
{
    if (mfma_d8_kernel_name(sh) == nullptr) return hipErrorNotSupported;
    switch (sh.N) {
        case 4: return launch8<4>(sh, path, out, st);
        case 5: return launch8<5>(sh, path, out, st);
        case 6: return launch8<6>(sh, path, out, st);
    }
    return hipErrorNotSupported;
}

}  // namespace sig
