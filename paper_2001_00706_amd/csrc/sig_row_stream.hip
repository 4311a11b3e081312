// Stream-mode kernel family for channel counts without a matrix-core stream kernel (d = 2..16 except where noted
// below), fp32 and fp64: one wavefront scans a few rows (paths, or chunks of paths) and writes every prefix signature
// as whole rows of consecutive scalars.
//
// Arithmetic as in the prefix-tree family (paper section 4.1, eq. "fusedterm": the new coefficient of a word needs the
// coefficients of that word's prefixes only): a lane stands for a word u of P letters, carries the coefficients of u
// and of its prefixes, and owns the U = N - P levels below u (d scalars, or d + d^2).  What differs is the shape: P
// is the largest number of letters with d^P <= 64, so that the words of one row fill a wavefront (or a whole number
// of rows does), an increment costs a few dozen instructions, and nothing is ever exchanged between wavefronts:
// workgroups are single wavefronts and there is no workgroup barrier that waits for anything but the LDS.
//
// Stores are what stream mode is made of.  A lane's words of the top level are d^U scalars in a row, so stored from
// registers every instruction would touch 64 different lines.  Instead the wavefront assembles the signature in LDS,
// in flat word order, and copies it out lane after lane: 256 bytes in a row per store instruction.  The LDS index is
// skewed by one word per lane block of even length, which puts the lanes' blocks into different banks.
//
// The kernel serves every row layout of sig_internal.h: plain stream mode, the two passes of a stream scan cut into
// chunks (chunk signatures to the chunk ends; chunks rescanned from the row before them), and final mode (packed
// rows, chunked or not), where it is the fastest family for the shapes that leave one level below a lane's word:
// 128 points, d = 8, N = 3: 19 us against 47 on the prefix-tree kernel at 32 paths, 30 against 56 at 4096.
#include <type_traits>

#include "sig_internal.h"

namespace sig {
namespace {

constexpr int kRsTile = 32;   // increments staged in LDS at a time

__host__ __device__ constexpr int64_t rs_off(int d, int k)   // offset of level k (1-based) in a flat element
{
    int64_t off = 0, p = 1;
    for (int j = 1; j < k; ++j) {
        p *= d;
        off += p;
    }
    return off;
}

__host__ __device__ constexpr int rs_letters(int d, int n)   // largest P <= n - 1 with d^P <= 64
{
    int p = 0;
    int64_t w = 1;
    while (p < n - 1 && w * d <= 64) {
        w *= d;
        ++p;
    }
    return p;
}

template <typename T, int D, int N>
struct RowShape {
    static constexpr int P = rs_letters(D, N);
    static constexpr int U = N - P;
    static constexpr int kWords = int(rs_off(D, P + 1) - rs_off(D, P));   // d^P lanes per row
    static constexpr int R = 64 / kWords;                                  // rows per wavefront
    static constexpr int64_t kS = rs_off(D, N + 1);
    static constexpr int kBlock = U == 1 ? D : D * D;                      // a lane's run of top-level scalars
    static constexpr bool kSkew = kBlock % 2 == 0;
    static constexpr int64_t kStageRow = kS + (kSkew ? kS / kBlock : 0) + 1;
    static constexpr int64_t kLdsBytes = (R * kStageRow + R * kRsTile * D) * int64_t(sizeof(T));
    // one or two levels below a lane's word (two only up to 8 channels: beyond, a wavefront would carry several rows of
    // 90 and more scalars per lane, and the prefix-tree kernel is the faster one), at most 10 rows per wavefront, LDS in
    // bounds
    static constexpr bool kServed = N >= 2 && P >= 1 && (U == 1 || (U == 2 && D <= 8)) && R <= 10 && kLdsBytes <= 60 * 1024;
};

template <typename T, int D, int N>
__host__ __device__ constexpr int64_t rs_skew(int64_t i)
{
    return RowShape<T, D, N>::kSkew ? i + i / RowShape<T, D, N>::kBlock : i;
}

// A workgroup barrier that orders the LDS traffic only (a workgroup is one wavefront here, so this is an ordering
// point for the compiler and the LDS counter, not a wait for other wavefronts): __syncthreads() would also wait for
// the global stores issued before it, and the scan would advance at the latency of those writes.
__device__ __forceinline__ void rs_lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ float rs_fma(float a, float b, float c) { return __builtin_fmaf(a, b, c); }
__device__ __forceinline__ double rs_fma(double a, double b, double c) { return __builtin_fma(a, b, c); }

template <typename T, int D, int N>
__global__ void __launch_bounds__(64)
sig_row_stream_kernel(Shape sh, const T *__restrict__ path, T *__restrict__ out)
{
    using RS = RowShape<T, D, N>;
    constexpr int P = RS::P, U = RS::U, R = RS::R, kWords = RS::kWords;
    constexpr int H2 = U >= 2 ? D * D : 1;
    constexpr int64_t kS = RS::kS, kStageRow = RS::kStageRow;
    __shared__ T zt[R * kRsTile * D];
    __shared__ T stage[R * kStageRow];
    __shared__ int64_t row_x[R];       // per row of this wavefront: its path,
    __shared__ int64_t row_inc0[R];    // number of its first increment inside the path,
    __shared__ int64_t row_first[R];   // output row of that increment,
    __shared__ int row_n[R];           // increments to fold in,
    __shared__ int row_write[R];       // and rows to write in stream mode

    const int lane = threadIdx.x;
    const int slot_raw = lane / kWords;
    const int slot = slot_raw < R ? slot_raw : R - 1;   // lanes beyond the last row idle along
    const int u = lane - slot_raw * kWords;
    const int64_t row0 = int64_t(blockIdx.x) * R;
    const bool live = slot_raw < R && row0 + slot < sh.B;

    if (lane < R) {
        int64_t x0 = 0, inc0 = 0, first = 0;
        int n = 0, wr = 0;
        if (row0 + lane < sh.B) {
            const ChunkView cv = chunk_view(row0 + lane, sh.chunks, sh.chunk_len, sh.n_inc);
            x0 = cv.path;
            inc0 = cv.inc0;
            // rows of a stream-mode output, or (plain final mode) one packed signature per row
            first = sh.stream || sh.rows_in_stream ? cv.path * sh.n_inc + cv.inc0 : row0 + lane - (int64_t(cv.n) - 1);
            n = int(cv.n);
            wr = !sh.stream ? 0 : sh.rows_in_stream ? (n > 0 ? n - 1 : 0) : n;
        }
        row_x[lane] = x0;
        row_inc0[lane] = inc0;
        row_first[lane] = first;
        row_n[lane] = n;
        row_write[lane] = wr;
    }
    rs_lds_barrier();
    int n_max = 0;
    int n_of[R], write_of[R];   // the same for every lane: kept in scalar registers
    int64_t first_of[R];
#pragma unroll
    for (int p = 0; p < R; ++p) {
        n_of[p] = __builtin_amdgcn_readfirstlane(row_n[p]);
        write_of[p] = __builtin_amdgcn_readfirstlane(row_write[p]);
        const int64_t f = row_first[p];
        first_of[p] = int64_t(uint64_t(uint32_t(__builtin_amdgcn_readfirstlane(int(uint64_t(f) & 0xffffffffu)))) |
                              (uint64_t(uint32_t(__builtin_amdgcn_readfirstlane(int(uint64_t(f) >> 32)))) << 32));
        n_max = n_of[p] > n_max ? n_of[p] : n_max;
    }

    int cl[P + 1];   // letters of this lane's word
    {
        int rest = u;
#pragma unroll
        for (int i = P; i >= 1; --i) {
            cl[i] = rest % D;
            rest /= D;
        }
    }
    T rk[N + 2];
#pragma unroll
    for (int m = 1; m <= N + 1; ++m) rk[m] = T(1) / T(m);

    T A[P + 1];   // coefficients of the prefixes of the word, and of the word itself (level P)
    T B1[D];      // words u c
    T B2[H2];     // words u c c'
#pragma unroll
    for (int i = 0; i <= P; ++i) A[i] = T(0);
#pragma unroll
    for (int c = 0; c < D; ++c) B1[c] = T(0);
#pragma unroll
    for (int c = 0; c < H2; ++c) B2[c] = T(0);

    // a chunk of a stream scan starts from the signature of everything before it, which the row before it holds
    if (sh.stream && sh.rows_in_stream && live && row_inc0[slot] > 0 && row_n[slot] > 0) {
        const T *o = out + (row_first[slot] - 1) * kS;
        int q = u;
#pragma unroll
        for (int i = P; i >= 1; --i) {
            A[i] = o[rs_off(D, i) + q];
            q /= D;
        }
#pragma unroll
        for (int c = 0; c < D; ++c) B1[c] = o[rs_off(D, P + 1) + u * D + c];
        if constexpr (U >= 2) {
#pragma unroll
            for (int c = 0; c < D * D; ++c) B2[c] = o[rs_off(D, P + 2) + u * (D * D) + c];
        }
    }

    // this lane's words into the staging row of its slot; a prefix is the first lane's below it
    T *my_stage = stage + slot * kStageRow;
    auto stage_words = [&]() {
        int q = u, width = 1;
#pragma unroll
        for (int i = P; i >= 1; --i) {
            if (u % width == 0) my_stage[rs_skew<T, D, N>(rs_off(D, i) + q)] = A[i];
            q /= D;
            width *= D;
        }
#pragma unroll
        for (int c = 0; c < D; ++c) my_stage[rs_skew<T, D, N>(rs_off(D, P + 1) + u * D + c)] = B1[c];
        if constexpr (U >= 2) {
#pragma unroll
            for (int c = 0; c < D * D; ++c) my_stage[rs_skew<T, D, N>(rs_off(D, P + 2) + u * (D * D) + c)] = B2[c];
        }
    };
    // row p of the staging area to output row `dst_row`, by the whole wavefront: 64 consecutive scalars per
    // instruction, the LDS reads of up to 16 of them in flight before the first store
    auto copy_out = [&](int p, int64_t dst_row) {
        T *dst = out + dst_row * kS;
        const T *src = stage + p * kStageRow;
        constexpr int kPieces = int((kS + 63) / 64), kBatch = 16;
#pragma unroll
        for (int j0 = 0; j0 < kPieces; j0 += kBatch) {
            T v[kBatch];
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {   // unconditional reads (index clamped in the last piece): none waits for a branch
                const int i = lane + 64 * (j0 + j);
                if (j0 + j < kPieces) v[j] = src[rs_skew<T, D, N>(64 * (j0 + j + 1) <= int(kS) || i < int(kS) ? i : int(kS) - 1)];
            }
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                const int i = lane + 64 * (j0 + j);
                if (j0 + j < kPieces && (64 * (j0 + j + 1) <= int(kS) || i < int(kS))) dst[i] = v[j];
            }
        }
    };

    // the rows of stream position `step` of every slot that has one: all LDS reads first, so that a wavefront with
    // several short rows waits for the LDS once per increment, not once per row
    constexpr int kPiecesAll = int((kS + 63) / 64);
    auto copy_step = [&](int step) {
        if constexpr (R > 1 && R * kPiecesAll <= 48) {
            T v[R][kPiecesAll];
#pragma unroll
            for (int p = 0; p < R; ++p)
#pragma unroll
                for (int j = 0; j < kPiecesAll; ++j) {
                    const int i = lane + 64 * j;
                    v[p][j] = stage[p * kStageRow + rs_skew<T, D, N>(64 * (j + 1) <= int(kS) || i < int(kS) ? i : int(kS) - 1)];
                }
#pragma unroll
            for (int p = 0; p < R; ++p)
                if (step < write_of[p]) {
                    T *dst = out + (first_of[p] + step) * kS;
#pragma unroll
                    for (int j = 0; j < kPiecesAll; ++j) {
                        const int i = lane + 64 * j;
                        if (64 * (j + 1) <= int(kS) || i < int(kS)) dst[i] = v[p][j];
                    }
                }
        } else {
#pragma unroll
            for (int p = 0; p < R; ++p)
                if (step < write_of[p]) copy_out(p, first_of[p] + step);
        }
    };

    const T *bpv = static_cast<const T *>(sh.basepoint_value);
    for (int t0 = 0; t0 < n_max; t0 += kRsTile) {
        rs_lds_barrier();   // the increments of the tile before are no longer needed
        // the tile's increments, R * kRsTile * D scalars, up to sixteen per lane at a time: every load is unconditional (on an
        // index clamped into the path) and issued before the first use, so a batch costs one trip to memory, not
        // one per scalar; rows past the end of the batch and increments past the end of a row add nothing
        constexpr int kStaged = R * kRsTile * D, kStageBatch = (kStaged + 63) / 64 < 16 ? (kStaged + 63) / 64 : 16;
#pragma unroll 1
        for (int e0 = 0; e0 < kStaged; e0 += 64 * kStageBatch) {
            T hi[kStageBatch], lo[kStageBatch];
            bool on[kStageBatch], first[kStageBatch];
#pragma unroll
            for (int j = 0; j < kStageBatch; ++j) {
                const int e = e0 + 64 * j + lane < kStaged ? e0 + 64 * j + lane : kStaged - 1;
                const int p = e / (kRsTile * D), i = (e / D) % kRsTile, c = e % D;
                on[j] = t0 + i < row_n[p];
                const T *x = path + row_x[p] * sh.L * D;
                const int64_t i_hi = on[j] ? row_inc0[p] + t0 + i + (sh.basepoint ? 0 : 1) : (sh.basepoint ? 0 : 1);
                first[j] = i_hi == 0;   // the increment from the basepoint
                hi[j] = x[i_hi * D + c];
                lo[j] = bpv != nullptr && first[j] ? bpv[row_x[p] * D + c] : x[(first[j] ? 0 : i_hi - 1) * D + c];
            }
#pragma unroll
            for (int j = 0; j < kStageBatch; ++j) {
                const int e = e0 + 64 * j + lane;
                if (e < kStaged) zt[e] = on[j] ? hi[j] - (first[j] && bpv == nullptr ? T(0) : lo[j]) : T(0);
            }
        }
        rs_lds_barrier();
        const int nt = n_max - t0 < kRsTile ? n_max - t0 : kRsTile;
        const T *zrow = zt + slot * kRsTile * D;
        for (int s = 0; s < nt; ++s, zrow += D) {
            // Horner terms along the word: Hn[k] = T^(k)_i for the level i just passed, k > i
            T Hn[N + 2];
            {
                const T zc = zrow[cl[1]];
#pragma unroll
                for (int k = 2; k <= N; ++k) Hn[k] = rs_fma(zc, rk[k], A[1]);
                A[1] += zc;
            }
#pragma unroll
            for (int i = 2; i <= P; ++i) {
                const T zc = zrow[cl[i]];
                const T a = A[i];
                A[i] = rs_fma(Hn[i], zc, a);
#pragma unroll
                for (int k = i + 1; k <= N; ++k) Hn[k] = rs_fma(Hn[k], zc * rk[k - i + 1], a);
            }
            T zu[D];
#pragma unroll
            for (int c = 0; c < D; ++c) zu[c] = zrow[c];
            if constexpr (U == 1) {
#pragma unroll
                for (int c = 0; c < D; ++c) B1[c] = rs_fma(Hn[P + 1], zu[c], B1[c]);
            } else {
#pragma unroll
                for (int c = 0; c < D; ++c) {
                    const T t1 = rs_fma(Hn[P + 2], zu[c] * rk[2], B1[c]);   // T^(N)_{P+1}[u c]
                    B1[c] = rs_fma(Hn[P + 1], zu[c], B1[c]);
#pragma unroll
                    for (int j = 0; j < D; ++j) B2[c * D + j] = rs_fma(t1, zu[j], B2[c * D + j]);
                }
            }
            if (sh.stream) {
                if (live) stage_words();
                rs_lds_barrier();
                copy_step(t0 + s);
                rs_lds_barrier();
            }
        }
    }

    // final mode: one signature per row, packed (the identity for a chunk without increments), or, for a chunk of a
    // stream scan, in the output row of its last increment
    if (!sh.stream) {
        if (live) stage_words();
        rs_lds_barrier();
#pragma unroll
        for (int p = 0; p < R; ++p)
            if (n_of[p] > 0 || (!sh.rows_in_stream && row0 + p < sh.B)) copy_out(p, first_of[p] + n_of[p] - 1);
    }
}

template <typename T, int D, int N>
hipError_t launch_row_stream_dn(const Shape &sh, const T *path, T *out, hipStream_t st)
{
    if constexpr (RowShape<T, D, N>::kServed) {
        const int64_t groups = (sh.B + RowShape<T, D, N>::R - 1) / RowShape<T, D, N>::R;
        if (groups > 0x7fffffff) return hipErrorNotSupported;
        hipLaunchKernelGGL((sig_row_stream_kernel<T, D, N>), dim3(unsigned(groups)), dim3(64), 0, st, sh, path, out);
        return hipGetLastError();
    } else {
        return hipErrorNotSupported;
    }
}

template <typename T, int D, int N>
constexpr bool row_stream_served() { return RowShape<T, D, N>::kServed; }

// (d, N) -> f<T, D, N>() over the instantiated range: d = 2..16, N = 2..8
template <typename T, int D, typename F>
auto dispatch_depth(int N, F &&f)
{
    switch (N) {
        case 2: return f(std::integral_constant<int, D>{}, std::integral_constant<int, 2>{});
        case 3: return f(std::integral_constant<int, D>{}, std::integral_constant<int, 3>{});
        case 4: return f(std::integral_constant<int, D>{}, std::integral_constant<int, 4>{});
        case 5: return f(std::integral_constant<int, D>{}, std::integral_constant<int, 5>{});
        case 6: return f(std::integral_constant<int, D>{}, std::integral_constant<int, 6>{});
        case 7: return f(std::integral_constant<int, D>{}, std::integral_constant<int, 7>{});
        case 8: return f(std::integral_constant<int, D>{}, std::integral_constant<int, 8>{});
    }
    return f(std::integral_constant<int, D>{}, std::integral_constant<int, 0>{});
}

template <typename T, typename F>
auto dispatch_shape(int d, int N, F &&f)
{
    switch (d) {
        case 2: return dispatch_depth<T, 2>(N, f);
        case 3: return dispatch_depth<T, 3>(N, f);
        case 4: return dispatch_depth<T, 4>(N, f);
        case 5: return dispatch_depth<T, 5>(N, f);
        case 6: return dispatch_depth<T, 6>(N, f);
        case 7: return dispatch_depth<T, 7>(N, f);
        case 8: return dispatch_depth<T, 8>(N, f);
        case 9: return dispatch_depth<T, 9>(N, f);
        case 10: return dispatch_depth<T, 10>(N, f);
        case 11: return dispatch_depth<T, 11>(N, f);
        case 12: return dispatch_depth<T, 12>(N, f);
        case 13: return dispatch_depth<T, 13>(N, f);
        case 14: return dispatch_depth<T, 14>(N, f);
        case 15: return dispatch_depth<T, 15>(N, f);
        case 16: return dispatch_depth<T, 16>(N, f);
    }
    return f(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{});
}

template <typename T>
bool row_stream_supported_t(const Shape &sh)
{
    if (sh.S >= (int64_t(1) << 31) || sh.n_inc >= (int64_t(1) << 31) - 64) return false;
    return dispatch_shape<T>(sh.d, sh.N, [](auto dc, auto nc) -> bool {
        constexpr int D = decltype(dc)::value, N = decltype(nc)::value;
        if constexpr (D >= 2 && N >= 2)
            return row_stream_served<T, D, N>();
        else
            return false;
    });
}

template <typename T>
hipError_t launch_row_stream_t(const Shape &sh, const T *path, T *out, hipStream_t st)
{
    if (!row_stream_supported_t<T>(sh)) return hipErrorNotSupported;
    return dispatch_shape<T>(sh.d, sh.N, [&](auto dc, auto nc) -> hipError_t {
        constexpr int D = decltype(dc)::value, N = decltype(nc)::value;
        if constexpr (D >= 2 && N >= 2)
            return launch_row_stream_dn<T, D, N>(sh, path, out, st);
        else
            return hipErrorNotSupported;
    });
}

}  // namespace

bool row_stream_one_level(const Shape &sh)
{
    return sh.d >= 2 && sh.d <= 64 && sh.N >= 2 && sh.N - rs_letters(sh.d, sh.N) == 1;
}

bool row_stream_supported(const Shape &sh, sig_dtype dtype)
{
    return dtype == SIG_F32 ? row_stream_supported_t<float>(sh) : row_stream_supported_t<double>(sh);
}

hipError_t launch_row_stream_f32(const Shape &sh, const float *path, float *out, hipStream_t st)
{
    return launch_row_stream_t<float>(sh, path, out, st);
}

hipError_t launch_row_stream_f64(const Shape &sh, const double *path, double *out, hipStream_t st)
{
    return launch_row_stream_t<double>(sh, path, out, st);
}

}  // namespace sig
