// Matrix-core kernel family (fp32), d = 4 channels, depth N = 4..7, final and stream mode,
// four wavefronts per path with no communication between them.
//
// The words that start with a given first letter f, together with the one-letter word f itself,
// are closed under the fused multiply-exponentiate (paper section 4.1, eq. "fusedterm"): the
// new coefficient of a word depends only on the old coefficients of its prefixes.  So a path is
// cut into four shards by first letter, one wavefront each, and every shard scans all the
// increments on its own; each writes its own slice of every level, and the slices tile the output.
// This gives a batch of B paths 4B wavefronts, which is what stream mode needs: there every
// prefix signature is written out (section 5.5, "expanding intervals"), the kernel is bound by
// HBM writes, and one wavefront per path cannot issue stores fast enough.
//
// Register layout of shard f (lane = 16*w_2 + 4*w_3 + q):
//   A_1[f]                 the same scalar in every lane
//   A_2[f w_2], A_3[f w_2 w_3], A_4[f w_2 w_3 q]      one scalar per lane (replicated where needed)
//   A_k, k >= 5            4^(k-5) groups of 4 registers: group g spells letters w_4..w_{k-2},
//                          register r is letter w_{k-1}, lane q is letter w_k, block (lane/4) is w_2 w_3
// Levels 1..4 are plain vector FMAs; from level 5 on each Horner stage is a batch of 4x4 outer
// products on the matrix cores whose result registers are, as they stand, the left operand of the
// next stage.  The top level feeds no further stage, so its outer product is taken with the two
// operands swapped: register r is then the LAST letter w_N and lane q the letter before it, a lane
// holds 4 consecutive words, and a wavefront store covers 1 KB of contiguous output with no
// shuffling at all.  Lower matrix-core levels (only present for N >= 6) are stored word by word, as
// they sit in the registers (the four lanes of a quad write 16 contiguous bytes per instruction).  The 21 words of levels 1..3 go out in one store
// instruction: every lane writes one of them (several lanes the same word with the same value).
#include "sig_internal.h"
#include "sig_mfma_common.h"

namespace sig {
namespace {

// offsets of levels 1..8 in a d = 4 signature
constexpr int kLevelOff[9] = {0, 0, 4, 20, 84, 340, 1364, 5460, 21844};

template <int N>
constexpr int kTileShard = 64;  // increments staged in LDS at a time

template <int N>
struct ShardState {
    float A1 = 0.0f, A2 = 0.0f, A3 = 0.0f, A4 = 0.0f;
    f4 A5[1];
    f4 A6[N >= 6 ? 4 : 1];
    f4 A7[N >= 7 ? 16 : 1];
};

// This lane's view of one staged increment.
template <int N>
struct ShardRow {
    float zf;      // z[f]
    float zB[N];   // zB[m] = z[w_2]/m, m = 1..N-1
    float zC[N];   // zC[m] = z[w_3]/m, m = 1..N-2
    float zQ[N];   // zQ[m] = z[q]/m,   m = 1..N-3
};

// `tab` points at one increment's scaled copies in LDS: tab[(m-1)*4 + c] = z[c]/m, m = 1..N-1.
template <int N>
__device__ __forceinline__ ShardRow<N> load_shard_row(const float *tab, int f, int w2, int w3, int q)
{
    ShardRow<N> R;
    R.zf = tab[f];
#pragma unroll
    for (int m = 1; m <= N - 1; ++m) R.zB[m] = tab[(m - 1) * 4 + w2];
#pragma unroll
    for (int m = 1; m <= N - 2; ++m) R.zC[m] = tab[(m - 1) * 4 + w3];
#pragma unroll
    for (int m = 1; m <= N - 3; ++m) R.zQ[m] = tab[(m - 1) * 4 + q];
    return R;
}

// One fused multiply-exponentiate restricted to the words of this shard.
template <int N>
__device__ __forceinline__ void shard_step(ShardState<N> &S, const ShardRow<N> &R)
{
    float t1[N + 1], t2[N + 1], t3[N + 1], t4[N + 1];
#pragma unroll
    for (int k = 2; k <= N; ++k) t1[k] = __builtin_fmaf(R.zf, 1.0f / k, S.A1);
#pragma unroll
    for (int k = 2; k <= N; ++k) t2[k] = __builtin_fmaf(t1[k], R.zB[k - 1], S.A2);
#pragma unroll
    for (int k = 3; k <= N; ++k) t3[k] = __builtin_fmaf(t2[k], R.zC[k - 2], S.A3);
#pragma unroll
    for (int k = 4; k <= N; ++k) t4[k] = __builtin_fmaf(t3[k], R.zQ[k - 3], S.A4);

    // levels 5.., higher targets first so that every stage reads the old A_i
    if constexpr (N >= 5) {
        f4 t5[N + 1];
#pragma unroll
        for (int k = N; k >= 6; --k) t5[k] = outer4(t4[k], R.zQ[k - 4], S.A5[0]);
        if constexpr (N == 5) S.A5[0] = outer4(R.zQ[1], t4[5], S.A5[0]);  // top level: operands swapped
        else S.A5[0] = outer4(t4[5], R.zQ[1], S.A5[0]);
        if constexpr (N >= 6) {
            f4 t6[4];
            if constexpr (N >= 7) {
#pragma unroll
                for (int g = 0; g < 4; ++g) t6[g] = outer4(t5[7][g], R.zQ[2], S.A6[g]);
            }
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                if constexpr (N == 6) S.A6[g] = outer4(R.zQ[1], t5[6][g], S.A6[g]);  // top level: swapped
                else S.A6[g] = outer4(t5[6][g], R.zQ[1], S.A6[g]);
            }
            if constexpr (N >= 7) {
#pragma unroll
                for (int g = 0; g < 16; ++g) S.A7[g] = outer4(R.zQ[1], t6[g >> 2][g & 3], S.A7[g]);  // top: swapped
            }
        }
    }
    S.A4 = t4[4];
    S.A3 = t3[3];
    S.A2 = t2[2];
    S.A1 += R.zf;
}

// Per-lane constants of the stores, all in bytes from the start of a signature.
struct StorePlan {
    int low_off;             // the word of levels 1..3 this lane writes
    unsigned m1, m2, m3;     // all-ones for the level that word belongs to, zero otherwise
    int off4;                // this lane's word of level 4
    int off5, off6, off7;    // this lane's first 16 bytes of levels 5, 6 (group 0), 7 (group 0)
};

template <int N>
__device__ __forceinline__ StorePlan make_store_plan(int f, int lane)
{
    // levels 1..3: lanes 1, 17, 33, 49 carry A_2[f w_2]; lane 5 carries A_1[f]; every other lane
    // carries A_3[f w_2 w_3] (the lanes of a quad hold the same value and write it to the same word)
    StorePlan p;
    const bool is2 = (lane & 15) == 1, is1 = lane == 5;
    p.m1 = is1 ? ~0u : 0u;
    p.m2 = is2 ? ~0u : 0u;
    p.m3 = (is1 || is2) ? 0u : ~0u;
    p.low_off = 4 * (is2 ? kLevelOff[2] + 4 * f + (lane >> 4) : is1 ? f : kLevelOff[3] + 16 * f + (lane >> 2));
    p.off4 = 4 * (kLevelOff[4] + 64 * f + lane);
    // level k >= 5 occupies G = 4^(k-5) groups per block; group g of block blk starts at word (blk*G + g)*16,
    // and inside a group lane q holds words 4q..4q+3
    const int blk = lane >> 2, q = lane & 3;
    p.off5 = 4 * (kLevelOff[5] + 256 * f) + 16 * lane;
    p.off6 = 4 * (kLevelOff[6] + 1024 * f) + 16 * (blk * 16 + q);
    p.off7 = 4 * (kLevelOff[7] + 4096 * f) + 16 * (blk * 64 + q);
    return p;
}

typedef unsigned int u4 __attribute__((ext_vector_type(4)));

// Writes this shard's slice of every level of one signature.  The signature starts `row_bytes`
// into the buffer described by `rsrc` (a wave-uniform scalar), so the stores need no per-lane
// address arithmetic; stores beyond the descriptor's range would be dropped by the hardware.
template <int N>
__device__ __forceinline__ void store_shard(const ShardState<N> &S, __amdgpu_buffer_rsrc_t rsrc, int row_bytes,
                                            const StorePlan &p, int lane)
{
    const unsigned low = (__builtin_bit_cast(unsigned, S.A1) & p.m1) | (__builtin_bit_cast(unsigned, S.A2) & p.m2) |
                         (__builtin_bit_cast(unsigned, S.A3) & p.m3);
    __builtin_amdgcn_raw_buffer_store_b32(low, rsrc, p.low_off, row_bytes, 0);
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, S.A4), rsrc, p.off4, row_bytes, 0);
    // A level below the top one goes out as it sits in the registers (register r = letter w_{k-1}, lane q = letter
    // w_k): four one-word stores, 16 r - 12 q bytes from where 16 bytes of four consecutive words would start; the
    // four lanes of a quad write 16 contiguous bytes per instruction.  Transposed in the lane quads (DPP moves on copies of the accumulators) and stored 16 bytes per
    // lane, the first prefix signature of a round of four increments came out, now and then, with one register of
    // the transposed level wrong in lanes 12..15 of every row of 16 lanes, once a SIMD held more than one wavefront
    // (more than 128 paths; depth 6 and 7, stream mode, where every increment ends in a store; the state itself
    // stayed right).  Final mode, with one store after the scan, never showed it and takes the same route.
    const int back = 12 * (lane & 3);
    auto store_word = [&](float word, int offset) {
        // through a vector register: handed the element of an accumulator tuple directly, the compiler stored element 0
        // of the tuple four times
        asm volatile("" : "+v"(word));
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, word), rsrc, offset, row_bytes, 0);
    };
    if constexpr (N >= 5) {
        if constexpr (N >= 6) {
#pragma unroll
            for (int r = 0; r < 4; ++r) store_word(S.A5[0][r], p.off5 - back + 16 * r);
        } else {
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u4, S.A5[0]), rsrc, p.off5, row_bytes, 0);
        }
    }
    if constexpr (N >= 6) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            if constexpr (N >= 7) {
#pragma unroll
                for (int r = 0; r < 4; ++r) store_word(S.A6[g][r], p.off6 + 64 * g - back + 16 * r);
            } else {
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u4, S.A6[g]), rsrc, p.off6 + 64 * g, row_bytes, 0);
            }
        }
    }
    if constexpr (N >= 7) {
#pragma unroll
        for (int g = 0; g < 16; ++g)
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u4, S.A7[g]), rsrc, p.off7 + 64 * g, row_bytes, 0);
    }
}

// Buffer descriptor for `bytes` bytes at `base` (raw buffer, no swizzle, 32-bit offsets).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(float *base, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(base, 0, int(bytes), 0x00020000);
}

template <int N, bool STREAM>
__global__ void __launch_bounds__(64)
sig_mfma_d4_shard_kernel(const float *__restrict__ path, float *__restrict__ out, int64_t L, int64_t n_inc_total,
                         int basepoint, const float *__restrict__ bpv, int chunks, int64_t chunk_len)
{
    static_assert(N >= 4 && N <= 7, "depths served by this kernel");
    constexpr int kRow = 4 * (N - 1);  // floats per staged increment
    constexpr int kTile = kTileShard<N>;
    constexpr int kS = kLevelOff[N + 1];
    __shared__ __align__(16) float lds[kTile * kRow];

    const int lane = threadIdx.x;
    const int w2 = lane >> 4, w3 = (lane >> 2) & 3, q = lane & 3;
    // Workgroups are handed to the chip's 8 XCDs (each with its own L2) round-robin by number.  The four shards
    // of a path write interleaved pieces of the same output rows, pieces that do not end on cache-line boundaries,
    // so they are kept on one XCD, where the L2 merges them into whole lines: inside every run of 32 workgroups
    // (8 paths x 4 shards) the XCD number picks the path and the rest picks the shard.
    int64_t b;   // output row: a path, or one chunk of a path
    int f;       // first letter
    {
        const unsigned id = blockIdx.x, full = gridDim.x & ~31u;
        if (id < full) {
            const unsigned slot = id >> 3;
            b = int64_t(slot >> 2) * 8 + (id & 7);
            f = int(slot & 3);
        } else {
            b = id >> 2;
            f = int(id & 3);
        }
    }
    const ChunkView cv = chunk_view(b, chunks, chunk_len, n_inc_total);
    const int64_t n_inc = cv.n;
    const f4 *x4 = reinterpret_cast<const f4 *>(path) + cv.path * L;  // point l of this path
    float *o = out + b * (STREAM ? n_inc * kS : int64_t(kS));

    const StorePlan plan = make_store_plan<N>(f, lane);

    ShardState<N> S;
    S.A5[0] = (f4){0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int g = 0; g < (N >= 6 ? 4 : 1); ++g) S.A6[g] = (f4){0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int g = 0; g < (N >= 7 ? 16 : 1); ++g) S.A7[g] = (f4){0.0f, 0.0f, 0.0f, 0.0f};

    // the two points around increment number s (zeros past the end of the path); the points of
    // a tile are fetched while the tile before it is being scanned
    f4 p_hi, p_lo;
    auto fetch_points = [&](int64_t s) {
        p_hi = p_lo = (f4){0.0f, 0.0f, 0.0f, 0.0f};
        if (s < n_inc) {
            const int64_t i_hi = cv.inc0 + (basepoint ? s : s + 1);
            p_hi = x4[i_hi];
            if (i_hi > 0) p_lo = x4[i_hi - 1];
            else if (bpv != nullptr) p_lo = reinterpret_cast<const f4 *>(bpv)[cv.path];
        }
    };
    fetch_points(lane);

    for (int64_t t0 = 0; t0 < n_inc; t0 += kTile) {
        const int nt = int(n_inc - t0 < kTile ? n_inc - t0 : kTile);
        __syncthreads();
        if (lane < nt) {
            const f4 z = p_hi - p_lo;
            f4 *row = reinterpret_cast<f4 *>(lds + lane * kRow);
            row[0] = z;
#pragma unroll
            for (int m = 2; m <= N - 1; ++m) row[m - 1] = z * (1.0f / m);
        }
        __syncthreads();
        fetch_points(t0 + kTile + lane);
        // stream mode: one descriptor per tile of prefix signatures (a tile is at most 64 * 87376 bytes)
        const __amdgpu_buffer_rsrc_t rsrc = make_rsrc(o + (STREAM ? t0 * kS : 0), unsigned(STREAM ? nt : 1) * kS * 4u);
        int s = 0;
        for (; s + 4 <= nt; s += 4) {
            ShardRow<N> R[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) R[i] = load_shard_row<N>(lds + (s + i) * kRow, f, w2, w3, q);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                shard_step<N>(S, R[i]);
                if constexpr (STREAM) store_shard<N>(S, rsrc, (s + i) * kS * 4, plan, lane);
            }
        }
        for (; s < nt; ++s) {
            shard_step<N>(S, load_shard_row<N>(lds + s * kRow, f, w2, w3, q));
            if constexpr (STREAM) store_shard<N>(S, rsrc, s * kS * 4, plan, lane);
        }
    }
    if constexpr (!STREAM) store_shard<N>(S, make_rsrc(o, kS * 4u), 0, plan, lane);
}


// ---- stream mode for N <= 6: one workgroup of four wavefronts (the four first-letter shards) per path ----
//
// A stream-mode launch is a pure HBM write stream, and what the memory system rewards is long runs of whole
// 128-byte lines written by one wavefront.  The shards' own slices of a prefix signature are short and end inside
// lines, so here they are first assembled in LDS, in output order, kRowsPerFlush prefix signatures at a time (two
// such buffers take turns), and after a barrier the four wavefronts copy the assembled run to `out`: each takes a
// contiguous quarter of it, cut at 128-byte boundaries of the output address, 16 bytes per lane.
template <int N>
constexpr int kRowsPerFlush = N == 4 ? 16 : N == 5 ? 4 : 1;   // about 21.8 KB per buffer at every depth

template <int N>
__device__ __forceinline__ void lds_store_shard(const ShardState<N> &S, char *row, const StorePlan &p, int lane)
{
    const unsigned low = (__builtin_bit_cast(unsigned, S.A1) & p.m1) | (__builtin_bit_cast(unsigned, S.A2) & p.m2) |
                         (__builtin_bit_cast(unsigned, S.A3) & p.m3);
    *reinterpret_cast<unsigned *>(row + p.low_off) = low;
    *reinterpret_cast<float *>(row + p.off4) = S.A4;
    if constexpr (N == 5) *reinterpret_cast<f4 *>(row + p.off5) = S.A5[0];
    if constexpr (N >= 6) {
        // level 5 as it sits in the registers (register r = letter w_4, lane q = letter w_5), a word per register
#pragma unroll
        for (int r = 0; r < 4; ++r) *reinterpret_cast<float *>(row + p.off5 - 12 * (lane & 3) + 16 * r) = S.A5[0][r];
    }
    if constexpr (N >= 6) {
#pragma unroll
        for (int g = 0; g < 4; ++g) *reinterpret_cast<f4 *>(row + p.off6 + 64 * g) = S.A6[g];
    }
}

template <int N>
__global__ void __launch_bounds__(256)
sig_mfma_d4_stream_kernel(const float *__restrict__ path, float *__restrict__ out, int64_t L, int64_t n_inc, int basepoint,
                          const float *__restrict__ bpv)
{
    static_assert(N >= 4 && N <= 6, "depths served by this kernel");
    constexpr int kRow = 4 * (N - 1);   // floats per staged increment
    constexpr int kTile = 128;          // increments staged at a time
    constexpr int kS = kLevelOff[N + 1];
    constexpr int kFlush = kRowsPerFlush<N>;
    __shared__ __align__(16) float tab[kTile * kRow];
    __shared__ __align__(16) float rows[2][kFlush * kS];

    const int tid = threadIdx.x, lane = tid & 63;
    const int f = __builtin_amdgcn_readfirstlane(tid >> 6);       // wavefront number = first letter (a scalar)
    const int w2 = lane >> 4, w3 = (lane >> 2) & 3, q = lane & 3;
    const int64_t b = blockIdx.x;
    const f4 *x4 = reinterpret_cast<const f4 *>(path) + b * L;
    char *o = reinterpret_cast<char *>(out + b * n_inc * kS);
    const StorePlan plan = make_store_plan<N>(f, lane);

    ShardState<N> S;
    S.A5[0] = (f4){0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int g = 0; g < (N >= 6 ? 4 : 1); ++g) S.A6[g] = (f4){0.0f, 0.0f, 0.0f, 0.0f};

    f4 p_hi, p_lo;
    auto fetch_points = [&](int64_t s) {
        p_hi = p_lo = (f4){0.0f, 0.0f, 0.0f, 0.0f};
        if (s < n_inc) {
            const int64_t i_hi = basepoint ? s : s + 1;
            p_hi = x4[i_hi];
            if (i_hi > 0) p_lo = x4[i_hi - 1];
            else if (bpv != nullptr) p_lo = reinterpret_cast<const f4 *>(bpv)[b];
        }
    };
    if (tid < kTile) fetch_points(tid);

    int fill = 0, cur = 0;     // prefix signatures assembled in rows[cur] so far
    int64_t flushed = 0;       // prefix signatures already copied to `out`
    // every wavefront of the workgroup takes the same trips through these loops, so the barriers below are met by all
    constexpr int kRunBytes = kFlush * kS * 4;                         // a full buffer
    constexpr int kPieces = (kRunBytes / 4 + 127 + 1023) / 1024;       // 1 KB pieces in a wavefront's share of it
    auto flush = [&]() {
        // a barrier that orders the LDS traffic only: __syncthreads() would also wait for the global stores of the
        // previous run to complete, and the scan would then advance at the latency of HBM writes
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
        char *run = o + flushed * (kS * 4);
        const int bytes = fill * (kS * 4), quarter = bytes / 4;
        const int mis = int(reinterpret_cast<uintptr_t>(run) & 127);
        // this wavefront's share [lo, hi) of the run, in bytes from its start, cut where the ADDRESS is a multiple of 128
        int lo = f == 0 ? 0 : ((mis + quarter * f) & ~127) - mis;
        int hi = f == 3 ? bytes : ((mis + quarter * (f + 1)) & ~127) - mis;
        lo = lo < 0 ? 0 : lo;
        hi = hi < 0 ? 0 : hi;
        const char *src = reinterpret_cast<const char *>(rows[cur]);
        f4 piece[kPieces];
#pragma unroll
        for (int j = 0; j < kPieces; ++j) {
            const int at = lo + lane * 16 + j * 1024;
            if (at < hi) piece[j] = *reinterpret_cast<const f4 *>(src + at);
        }
#pragma unroll
        for (int j = 0; j < kPieces; ++j) {
            const int at = lo + lane * 16 + j * 1024;
            if (at < hi) *reinterpret_cast<f4 *>(run + at) = piece[j];
        }
        flushed += fill;
        fill = 0;
        cur ^= 1;
    };

    for (int64_t t0 = 0; t0 < n_inc; t0 += kTile) {
        const int nt = int(n_inc - t0 < kTile ? n_inc - t0 : kTile);
        __syncthreads();
        if (tid < nt) {
            const f4 z = p_hi - p_lo;
            f4 *row = reinterpret_cast<f4 *>(tab + tid * kRow);
            row[0] = z;
#pragma unroll
            for (int m = 2; m <= N - 1; ++m) row[m - 1] = z * (1.0f / m);
        }
        __syncthreads();
        if (tid < kTile) fetch_points(t0 + kTile + tid);
        for (int s = 0; s < nt; s += 4) {
            const int m = nt - s < 4 ? nt - s : 4;
            ShardRow<N> R[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (i < m) R[i] = load_shard_row<N>(tab + (s + i) * kRow, f, w2, w3, q);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (i < m) {
                    shard_step<N>(S, R[i]);
                    lds_store_shard<N>(S, reinterpret_cast<char *>(rows[cur]) + fill * (kS * 4), plan, lane);
                    if (++fill == kFlush) flush();
                }
            }
        }
    }
    if (fill > 0) flush();
}

template <int N>
hipError_t launch_shard(const Shape &sh, const float *path, float *out, hipStream_t st)
{
    const dim3 grid(static_cast<unsigned>(sh.B * 4)), block(64);
    if (sh.stream) {
        hipLaunchKernelGGL((sig_mfma_d4_shard_kernel<N, true>), grid, block, 0, st, path, out, sh.L, sh.n_inc, sh.basepoint,
                           static_cast<const float *>(sh.basepoint_value), sh.chunks, sh.chunk_len);
    } else {
        hipLaunchKernelGGL((sig_mfma_d4_shard_kernel<N, false>), grid, block, 0, st, path, out, sh.L, sh.n_inc, sh.basepoint,
                           static_cast<const float *>(sh.basepoint_value), sh.chunks, sh.chunk_len);
    }
    return hipGetLastError();
}

}  // namespace

const char *mfma_shard_kernel_name(const Shape &sh)
{
    if (sh.d != 4 || sh.N < 4 || sh.N > 7 || sh.B > 0x1fffffff) return nullptr;
    return "mfma_d4_shard";
}

const char *mfma_stream_kernel_name(const Shape &sh)
{
    if (sh.d != 4 || sh.N < 4 || sh.N > 6 || !sh.stream || sh.chunks > 1 || sh.B > 0x7fffffff) return nullptr;
    return "mfma_d4_stream";
}

bool mfma_stream_preferred(const Shape &sh)
{
    // An output that fits the 256 MB last-level cache is absorbed there at more than 6 TB/s whatever the store
    // pattern, and four independent wavefronts per path get there fastest (B = 192, L = 256, N = 5: 6.4 TB/s).
    // Beyond it the writes go to HBM at the pace of the store pattern: pieces that end inside 128-byte lines
    // reach 3.7 TB/s at B = 1024, whole runs assembled in LDS 5.1 to 5.3 TB/s.
    constexpr int64_t kCacheBytes = 300 * 1000 * 1000;
    return mfma_stream_kernel_name(sh) != nullptr && sh.B * sh.n_inc * sh.S * 4 > kCacheBytes;
}

hipError_t launch_mfma_stream_f32(const Shape &sh, const float *path, float *out, hipStream_t st)
{
    if (mfma_stream_kernel_name(sh) == nullptr) return hipErrorNotSupported;
    const dim3 grid(static_cast<unsigned>(sh.B)), block(256);
    const float *bpv = static_cast<const float *>(sh.basepoint_value);
    switch (sh.N) {
        case 4: hipLaunchKernelGGL(sig_mfma_d4_stream_kernel<4>, grid, block, 0, st, path, out, sh.L, sh.n_inc, sh.basepoint, bpv); break;
        case 5: hipLaunchKernelGGL(sig_mfma_d4_stream_kernel<5>, grid, block, 0, st, path, out, sh.L, sh.n_inc, sh.basepoint, bpv); break;
        case 6: hipLaunchKernelGGL(sig_mfma_d4_stream_kernel<6>, grid, block, 0, st, path, out, sh.L, sh.n_inc, sh.basepoint, bpv); break;
        default: return hipErrorNotSupported;
    }
    return hipGetLastError();
}

hipError_t launch_mfma_shard_f32(const Shape &sh, const float *path, float *out, hipStream_t st)
{
    if (mfma_shard_kernel_name(sh) == nullptr) return hipErrorNotSupported;
    switch (sh.N) {
        case 4: return launch_shard<4>(sh, path, out, st);
        case 5: return launch_shard<5>(sh, path, out, st);
        case 6: return launch_shard<6>(sh, path, out, st);
        case 7: return launch_shard<7>(sh, path, out, st);
    }
    return hipErrorNotSupported;
}

}  // namespace sig
