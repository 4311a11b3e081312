// Gradient of the signature with respect to the path for many channels (any d at N = 2..9, fp32 and
// fp64, final and stream mode): what serves more than 16 channels, where the prefix-tree gradient kernels have no
// instantiation (paper section 5.3, appendix C.1).
//
// The recurrences are those of sig_tree_backward_impl.h with one level below a thread's word and the channel count a
// run-time value.  A thread stands for a word u of N - 1 letters and a block of 16 (or 32) last letters j: it keeps the
// cotangents of the words u j in registers, carries the signature at the prefixes of u ("up": undoing the increment
// needs nothing else) and, for each prefix, the part of that prefix's cotangent that arrived through its own block
// ("down" is linear, so the parts may stay apart; a prefix's own cotangent goes to the first thread below it).
// Nothing is exchanged between threads except the one sum that ends an increment: its gradient is the sum of
// every thread's products for the letters of its block and of one scalar per letter of its word.
//   * The 64 lanes of a wavefront share their block of letters.  Their 16 x 64 products are summed over the lanes by a
//     butterfly that halves the number of values a lane still holds at every step (15 exchanges instead of 96), then
//     over the four rows of 16 lanes.
//   * A wavefront adds its sums and the scalars of its lanes' words into its own LDS row of the increment (lanes whose
//     words share a letter are summed first; nothing else writes to that row meanwhile); at the end of a tile the
//     rows of the workgroup's four
//     wavefronts are added in a fixed order and written to a workspace [path][workgroup][increment][d].
//   * A second kernel adds the workgroups' partial sums and turns gradients of increments into gradients of points.
#include "sig_internal.h"
#include "sig_lane_ops.h"

namespace sig {
namespace {

constexpr int kWbTile = 16;    // increments staged in LDS at a time

__device__ __forceinline__ float wb_fma(float a, float b, float c) { return __builtin_fmaf(a, b, c); }
__device__ __forceinline__ double wb_fma(double a, double b, double c) { return __builtin_fma(a, b, c); }

struct WbPlan {
    int block;                 // last letters per thread: 16 or 32
    int jblocks;               // ceil(d / block)
    int dpad;                  // jblocks * block
    int64_t words;             // d^(N-1)
    int64_t waves_per_block;   // wavefronts that cover the words once: ceil(words / 64)
    int64_t groups_per_path;   // workgroups of four wavefronts per path
};

// a[v], v = 0..15, summed over the 16 lanes of a row: lane l returns the total of value l % 16.  At every step a lane
// keeps the half of its values that its own lane-number bit selects and receives the partner's copies of them.
template <typename T>
__device__ __forceinline__ T row_transpose_sum(const T (&a)[16], int lane)
{
    const bool b3 = lane & 8, b2 = lane & 4, b1 = lane & 2, b0 = lane & 1;
    T s8[8], s4[4], s2[2];
#pragma unroll
    for (int v = 0; v < 8; ++v) s8[v] = (b3 ? a[v + 8] : a[v]) + neighbour<8>(b3 ? a[v] : a[v + 8]);
#pragma unroll
    for (int v = 0; v < 4; ++v) s4[v] = (b2 ? s8[v + 4] : s8[v]) + neighbour<4>(b2 ? s8[v] : s8[v + 4]);
#pragma unroll
    for (int v = 0; v < 2; ++v) s2[v] = (b1 ? s4[v + 2] : s4[v]) + neighbour<2>(b1 ? s4[v] : s4[v + 2]);
    return (b0 ? s2[1] : s2[0]) + neighbour<1>(b0 ? s2[0] : s2[1]);
}

// v summed over the four rows of 16 lanes, in every lane, with the two row swaps of this device (odd rows of one
// register against even rows of another; the upper two rows against the lower two) on two copies of the value.
struct WbPair {
    unsigned first, second;
};

__device__ __forceinline__ WbPair swap_rows_16(unsigned v)
{
    typedef unsigned u2 __attribute__((ext_vector_type(2)));
    const u2 r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    return {r[0], r[1]};   // as scalars: a bit cast of a vector element reads the vector's first one
}

__device__ __forceinline__ WbPair swap_rows_32(unsigned v)
{
    typedef unsigned u2 __attribute__((ext_vector_type(2)));
    const u2 r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return {r[0], r[1]};
}

__device__ __forceinline__ float rows_sum(float v)
{
    const WbPair r = swap_rows_16(__builtin_bit_cast(unsigned, v));
    const float s = __builtin_bit_cast(float, r.first) + __builtin_bit_cast(float, r.second);
    const WbPair q = swap_rows_32(__builtin_bit_cast(unsigned, s));
    return __builtin_bit_cast(float, q.first) + __builtin_bit_cast(float, q.second);
}

__device__ __forceinline__ double rows_sum(double v)
{
    const auto low = [](double x) { return unsigned(__builtin_bit_cast(unsigned long long, x)); };
    const auto high = [](double x) { return unsigned(__builtin_bit_cast(unsigned long long, x) >> 32); };
    const auto whole = [](unsigned lo, unsigned hi) { return __builtin_bit_cast(double, (unsigned long long)(hi) << 32 | lo); };
    const WbPair rl = swap_rows_16(low(v)), rh = swap_rows_16(high(v));
    const double s = whole(rl.first, rh.first) + whole(rl.second, rh.second);
    const WbPair ql = swap_rows_32(low(s)), qh = swap_rows_32(high(s));
    return whole(ql.first, qh.first) + whole(ql.second, qh.second);
}

template <typename T, int N, bool STREAM, int WB>   // WB: last letters per thread, 16 or 32
__global__ void __launch_bounds__(256)
sig_wide_backward_kernel(Shape sh, WbPlan pl, const T *__restrict__ path, const T *__restrict__ sig,
                         const T *__restrict__ gout, T *__restrict__ partial)
{
    constexpr int P = N - 1;
    extern __shared__ __align__(32) unsigned char wb_smem[];
    T *zt = reinterpret_cast<T *>(wb_smem);   // [kWbTile][dpad]: increments, zeros behind the d-th channel
    T *part = zt + kWbTile * pl.dpad;         // [kWbTile][4][dpad]: a wavefront's sums for an increment

    const int tid = threadIdx.x, lane = tid & 63, wave_in_group = tid >> 6;
    const int d = sh.d;
    const int64_t row = blockIdx.x / pl.groups_per_path, group = blockIdx.x % pl.groups_per_path;
    const int64_t wave = group * 4 + wave_in_group;
    const int jb_raw = int(wave / pl.waves_per_block);
    const int64_t u_raw = (wave % pl.waves_per_block) * 64 + lane;
    const bool live = jb_raw < pl.jblocks && u_raw < pl.words;
    const int64_t u = live ? u_raw : 0;   // idle threads shadow word 0 and contribute nothing
    const int jb = jb_raw < pl.jblocks ? jb_raw : 0;   // the same in every lane of a wavefront
    const int j0 = jb * WB;

    int cl[P + 1];        // letters of the word
    int64_t pre[P + 1];   // index of its prefix of i letters inside level i
    bool first[P + 1];    // whether this thread is the first one below that prefix
    {
        int64_t rest = u, width = 1;
#pragma unroll
        for (int i = P; i >= 1; --i) {
            pre[i] = rest;
            first[i] = live && jb == 0 && u % width == 0;
            cl[i] = int(rest % d);
            rest /= d;
            width *= d;
        }
    }
    // Words that share an earlier letter lie side by side, in runs of at least d words: where d >= 16 a row of 16 lanes
    // holds at most two such letters, that of its first lane and that of its last.
    bool with_first[P + 1], with_last[P + 1];   // whether letter i of this lane's word is the one or (else) the other
    int first_letter[P + 1], last_letter[P + 1];
    {
        int64_t rest_first = u_raw - (lane & 15), rest_last = rest_first + 15;
#pragma unroll
        for (int i = P; i >= 1; --i) {
            first_letter[i] = int(rest_first % d);
            last_letter[i] = int(rest_last % d);
            with_first[i] = live && cl[i] == first_letter[i];
            with_last[i] = live && !with_first[i] && cl[i] == last_letter[i];
            rest_first /= d;
            rest_last /= d;
        }
    }
    T rk[N + 2];
#pragma unroll
    for (int m = 1; m <= N + 1; ++m) rk[m] = T(1) / T(m);

    const int64_t per_row = STREAM ? sh.n_inc * sh.S : sh.S;
    const T *sg = sig + row * per_row;
    const T *go = gout + row * per_row;

    T Glo[P + 1], Gtop[WB];   // cotangents: this thread's part at its prefixes, whole at the words of its block
    T Alo[P + 1];                   // the signature at the prefixes
    {
        const T *g_last = STREAM ? go + (sh.n_inc - 1) * sh.S : go;
#pragma unroll
        for (int i = 1; i <= P; ++i) {
            Glo[i] = first[i] ? g_last[sh.off[i] + pre[i]] : T(0);
            Alo[i] = STREAM ? T(0) : sg[sh.off[i] + pre[i]];
        }
#pragma unroll
        for (int c = 0; c < WB; ++c) {
            const bool on = live && j0 + c < d;
            const T v = g_last[sh.off[N] + u * d + (on ? j0 + c : 0)];
            Gtop[c] = on ? v : T(0);
        }
    }

    T Alo_ahead[P + 1];   // stream mode: the signature before the next increment to be undone
#pragma unroll
    for (int i = 1; i <= P; ++i) Alo_ahead[i] = STREAM && sh.n_inc >= 2 ? sg[(sh.n_inc - 2) * sh.S + sh.off[i] + pre[i]] : T(0);

    const T *x = path + row * sh.L * d;
    const T *bpv = static_cast<const T *>(sh.basepoint_value);
    T *my_part = part + wave_in_group * pl.dpad;   // + increment * 4 * dpad
    T *pp = partial + (row * pl.groups_per_path + group) * sh.n_inc * d;

    for (int64_t t0 = ((sh.n_inc - 1) / kWbTile) * kWbTile; t0 >= 0; t0 -= kWbTile) {
        const int nt = int(sh.n_inc - t0 < kWbTile ? sh.n_inc - t0 : kWbTile);
        __syncthreads();   // the tile before has been written out
        for (int e = tid; e < kWbTile * pl.dpad; e += 256) {
            const int i = e / pl.dpad, c = e - i * pl.dpad;
            const bool on = i < nt && c < d;
            // unconditional loads on indices clamped into the path
            const int64_t i_hi = (on ? t0 + i : 0) + (sh.basepoint ? 0 : 1);
            const int cc = on ? c : 0;
            const T hi = x[i_hi * d + cc];
            const T lo_path = x[(i_hi > 0 ? i_hi - 1 : 0) * d + cc];
            const T lo = i_hi > 0 ? lo_path : (bpv != nullptr ? bpv[row * d + cc] : T(0));
            zt[e] = on ? hi - lo : T(0);
        }
        for (int e = tid; e < kWbTile * 4 * pl.dpad; e += 256) part[e] = T(0);
        __syncthreads();

        // an increment's values are read one step ahead of their use: the LDS atomic adds that end a step would
        // otherwise hold back the reads of the next one
        typedef T T4 __attribute__((ext_vector_type(4)));
        T zc_next[P + 1];
        T4 zb_next[WB / 4];
        auto read_step = [&](int i) {
            const T *zrow = zt + i * pl.dpad;
#pragma unroll
            for (int j = 1; j <= P; ++j) zc_next[j] = zrow[cl[j]];
#pragma unroll
            for (int q = 0; q < WB / 4; ++q) zb_next[q] = *reinterpret_cast<const T4 *>(zrow + j0 + 4 * q);
        };
        read_step(nt - 1);
        for (int i = nt - 1; i >= 0; --i) {
            const int64_t s = t0 + i;
            T zc[P + 1], zb[WB];
#pragma unroll
            for (int j = 1; j <= P; ++j) zc[j] = zc_next[j];
#pragma unroll
            for (int c = 0; c < WB; ++c) zb[c] = zb_next[c / 4][c % 4];
            read_step(i > 0 ? i - 1 : 0);
            T Glo_ahead[P + 1], Gtop_ahead[WB];
            if constexpr (STREAM) {
                // the signature after s increments is output entry s - 1 (the identity for s = 0): fetched an increment
                // ahead, like the row of the cotangent that is added at the end of this step, so that a trip to memory
                // is not part of every step of the chain
#pragma unroll
                for (int j = 1; j <= P; ++j) {
                    Alo[j] = s > 0 ? Alo_ahead[j] : T(0);
                    Alo_ahead[j] = sg[(s > 1 ? s - 2 : 0) * sh.S + sh.off[j] + pre[j]];
                }
                const T *g_row = go + (s > 0 ? s - 1 : 0) * sh.S;
#pragma unroll
                for (int j = 1; j <= P; ++j) Glo_ahead[j] = g_row[sh.off[j] + pre[j]];
#pragma unroll
                for (int c = 0; c < WB; ++c) Gtop_ahead[c] = g_row[sh.off[N] + u * d + (live && j0 + c < d ? j0 + c : 0)];
            }

            // ---- up: Hn[j][k] = T^(k)_j at this thread's word; the signature before the increment
            T Hn[P + 1][N + 2];
            T a_lo[P + 1];
            a_lo[1] = STREAM ? Alo[1] : Alo[1] - zc[1];
#pragma unroll
            for (int k = 2; k <= N; ++k) Hn[1][k] = wb_fma(zc[1], rk[k], a_lo[1]);
#pragma unroll
            for (int j = 2; j <= P; ++j) {
                a_lo[j] = STREAM ? Alo[j] : wb_fma(-Hn[j - 1][j], zc[j], Alo[j]);
#pragma unroll
                for (int k = j + 1; k <= N; ++k) Hn[j][k] = wb_fma(Hn[j - 1][k], zc[j] * rk[k - j + 1], a_lo[j]);
            }
            if constexpr (!STREAM) {
#pragma unroll
                for (int j = 1; j <= P; ++j) Alo[j] = a_lo[j];
            }

            // ---- down, top level: the words of this thread's block
            T dzb[WB];
            T Dc[N + 2];   // Dc[k] = this thread's part of D^(k)_j at its prefix of the level j being processed
#pragma unroll
            for (int k = 0; k <= N + 1; ++k) Dc[k] = T(0);
            {
                const T top_term = Hn[P][N];
                T acc = T(0);
#pragma unroll
                for (int c = 0; c < WB; ++c) {
                    dzb[c] = top_term * Gtop[c];
                    acc = wb_fma(Gtop[c], zb[c], acc);
                }
                Dc[N] = acc;
            }
            // ---- levels N-1 .. 1 along the word: one scalar per level, this thread's part only
            T chain[P + 1];
#pragma unroll
            for (int j = P; j >= 1; --j) {
                T contrib = j >= 2 ? Hn[j >= 2 ? j - 1 : 1][j] * Glo[j] : Glo[j];   // T^(k)_0 = 1
                T g_add = T(0);
#pragma unroll
                for (int k = j + 1; k <= N; ++k) {
                    const T tp = j >= 2 ? Hn[j >= 2 ? j - 1 : 1][k] * rk[k - j + 1] : rk[k - j + 1];
                    contrib = wb_fma(tp, Dc[k], contrib);
                    g_add += Dc[k];
                }
                if (j >= 2) {
#pragma unroll
                    for (int k = N; k >= j + 1; --k) Dc[k] = Dc[k] * (zc[j] * rk[k - j + 1]);
                    Dc[j] = Glo[j] * zc[j];
                }
                Glo[j] += g_add;
                chain[j] = contrib;
            }

            // ---- this wavefront's part of the increment's gradient
            T *acc_row = my_part + i * 4 * pl.dpad;
            // A float add in LDS takes about 3 clocks per active lane whether or not the lanes meet, a plain read or
            // write of 64 lanes about 6 in all: atomic adds are kept for the few lanes that may meet at an address,
            // everything else is brought to distinct lanes first and added by a read and a write.
            {
                T total = rows_sum(row_transpose_sum(*reinterpret_cast<const T(*)[16]>(&dzb[0]), lane));
                if constexpr (WB == 32) {   // the block's second half the same way; lanes 16 .. 31 add it
                    const T second = rows_sum(row_transpose_sum(*reinterpret_cast<const T(*)[16]>(&dzb[16]), lane));
                    total = lane & 16 ? second : total;
                }
                if (lane < WB) acc_row[j0 + lane] += total;
            }
            // earlier letters: a row's two sums, added by its first and its last lane (rows may share a letter)
#pragma unroll
            for (int j = 1; j < P; ++j) {
                const T of_first = group_sum<0, 4, T>(with_first[j] ? chain[j] : T(0));
                const T of_last = group_sum<0, 4, T>(with_last[j] ? chain[j] : T(0));
                const int pos = lane & 15;
                if (pos == 0 || pos == 15)
                    atomicAdd(acc_row + (pos == 0 ? first_letter[j] : last_letter[j]), pos == 0 ? of_first : of_last);
                if (live && !with_first[j] && !with_last[j]) atomicAdd(acc_row + cl[j], chain[j]);   // only where d < 16
            }
            // last letter: consecutive words have consecutive letters, lanes d apart share one
            {
                T mine = live ? chain[P] : T(0);
                const T own = mine;
                for (int k = d; k < 64 && pl.words > 1; k += d) {   // (a single word: a single live lane)
                    const T other = __shfl_down(own, unsigned(k));
                    mine += lane + k < 64 ? other : T(0);
                }
                if (live && lane < d) acc_row[cl[P]] += mine;
            }

            if constexpr (STREAM) {
                if (s > 0) {
#pragma unroll
                    for (int j = 1; j <= P; ++j) Glo[j] += first[j] ? Glo_ahead[j] : T(0);
#pragma unroll
                    for (int c = 0; c < WB; ++c) Gtop[c] += live && j0 + c < d ? Gtop_ahead[c] : T(0);
                }
            }
        }
        __syncthreads();
        for (int e = tid; e < nt * d; e += 256) {
            const int i = e / d, c = e - i * d;
            const T *q = part + i * 4 * pl.dpad + c;
            pp[(t0 + i) * d + c] = ((q[0] + q[pl.dpad]) + q[2 * pl.dpad]) + q[3 * pl.dpad];
        }
    }
}

// gpath[row][point] = (sum of the partial gradients of the increment the point ends) - (of the one it starts);
// a basepoint only starts increment 0.
template <typename T>
__global__ void __launch_bounds__(256)
sig_wide_backward_reduce_kernel(Shape sh, int64_t n_partials, const T *__restrict__ partial, T *__restrict__ gpath,
                                T *__restrict__ gbase)
{
    const int d = sh.d;
    const int64_t per_row = (sh.n_inc + 1) * d;   // one extra "increment" -1 / n_inc at the ends
    const int64_t total = sh.B * per_row;
    for (int64_t e = blockIdx.x * int64_t(blockDim.x) + threadIdx.x; e < total; e += int64_t(gridDim.x) * blockDim.x) {
        const int64_t row = e / per_row, rem = e - row * per_row;
        const int64_t j = rem / d;   // output slot j: ends increment j - 1, starts increment j
        const int c = int(rem - j * d);
        const T *pr = partial + row * n_partials * sh.n_inc * d;
        T ends = T(0), starts = T(0);
        for (int64_t g = 0; g < n_partials; ++g) {
            if (j >= 1) ends += pr[(g * sh.n_inc + (j - 1)) * d + c];
            if (j < sh.n_inc) starts += pr[(g * sh.n_inc + j) * d + c];
        }
        const T v = ends - starts;
        if (sh.basepoint) {
            // slot 0 is the basepoint, slot j >= 1 the point j - 1
            if (j == 0) {
                if (gbase != nullptr) gbase[row * d + c] = v;
            } else {
                gpath[(row * sh.L + (j - 1)) * d + c] = v;
            }
        } else {
            gpath[(row * sh.L + j) * d + c] = v;
        }
    }
}

bool wb_plan(const Shape &sh, size_t elem, WbPlan &pl)
{
    if (sh.N < 2 || sh.N > 9 || sh.d < 1 || sh.chunks > 1 || sh.S >= (int64_t(1) << 31) || sh.n_inc < 1) return false;
    // from depth 3 on, where the channels fill whole blocks of 32 letters, the larger block halves the share of everything a
    // thread does per word rather than per letter (the chain along the word, the sums of its scalars)
    // ... as long as that leaves a thousand workgroups: below, a wavefront's latency per increment is what counts
    pl.words = sh.pw[sh.N - 1];
    pl.waves_per_block = (pl.words + 63) / 64;
    pl.block = sh.N >= 3 && sh.N <= 4 && sh.d % 32 == 0 && sh.B * ((pl.waves_per_block * (sh.d / 32) + 3) / 4) >= 1024 ? 32 : 16;
    pl.jblocks = (sh.d + pl.block - 1) / pl.block;
    pl.dpad = pl.jblocks * pl.block;
    pl.groups_per_path = (pl.waves_per_block * pl.jblocks + 3) / 4;
    if (sh.B * pl.groups_per_path > 0x7fffffff) return false;
    return elem * size_t(5 * kWbTile) * size_t(pl.dpad) <= 64 * 1024;
}

template <typename T>
hipError_t launch_wb_t(const Shape &sh, const T *path, const T *sig, const T *gout, T *gpath, T *gbase, void *workspace,
                       int64_t workspace_bytes, hipStream_t st)
{
    WbPlan pl;
    if (!wb_plan(sh, sizeof(T), pl)) return hipErrorNotSupported;
    const int64_t need = sh.B * pl.groups_per_path * sh.n_inc * sh.d * int64_t(sizeof(T));
    if (workspace == nullptr || workspace_bytes < need) return hipErrorInvalidValue;
    T *partial = static_cast<T *>(workspace);
    const dim3 grid{unsigned(sh.B * pl.groups_per_path)}, block{256};
    const size_t lds = sizeof(T) * size_t(5 * kWbTile) * size_t(pl.dpad);
#define SIG_WB_LAUNCH_B(NN, BB)                                                                                                  \
    if (sh.stream)                                                                                                               \
        hipLaunchKernelGGL((sig_wide_backward_kernel<T, NN, true, BB>), grid, block, lds, st, sh, pl, path, sig, gout, partial); \
    else                                                                                                                         \
        hipLaunchKernelGGL((sig_wide_backward_kernel<T, NN, false, BB>), grid, block, lds, st, sh, pl, path, sig, gout, partial)
#define SIG_WB_LAUNCH(NN)          \
    if (pl.block == 32) {          \
        SIG_WB_LAUNCH_B(NN, 32);   \
    } else {                       \
        SIG_WB_LAUNCH_B(NN, 16);   \
    }
    switch (sh.N) {
        case 2: SIG_WB_LAUNCH(2); break;
        case 3: SIG_WB_LAUNCH(3); break;
        case 4: SIG_WB_LAUNCH(4); break;
        // deeper: blocks of 16 only
        case 5: SIG_WB_LAUNCH_B(5, 16); break;
        case 6: SIG_WB_LAUNCH_B(6, 16); break;
        case 7: SIG_WB_LAUNCH_B(7, 16); break;
        case 8: SIG_WB_LAUNCH_B(8, 16); break;
        case 9: SIG_WB_LAUNCH_B(9, 16); break;
        default: return hipErrorNotSupported;
    }
#undef SIG_WB_LAUNCH
#undef SIG_WB_LAUNCH_B
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    const int64_t total = sh.B * (sh.n_inc + 1) * sh.d;
    const unsigned rgrid = unsigned((total + 255) / 256 < 65536 ? (total + 255) / 256 : 65536);
    hipLaunchKernelGGL((sig_wide_backward_reduce_kernel<T>), dim3(rgrid), dim3(256), 0, st, sh, pl.groups_per_path, partial, gpath,
                       gbase);
    return hipGetLastError();
}

}  // namespace

bool wide_backward_supported(const Shape &sh, sig_dtype dtype)
{
    WbPlan pl;
    return wb_plan(sh, dtype == SIG_F32 ? sizeof(float) : sizeof(double), pl);
}

int64_t wide_backward_workspace_bytes(const Shape &sh, sig_dtype dtype)
{
    WbPlan pl;
    const size_t elem = dtype == SIG_F32 ? sizeof(float) : sizeof(double);
    if (!wb_plan(sh, elem, pl)) return -1;
    return sh.B * pl.groups_per_path * sh.n_inc * sh.d * int64_t(elem);
}

hipError_t launch_wide_backward_f32(const Shape &sh, const float *path, const float *sig, const float *gout, float *gpath,
                                    float *gbase, void *workspace, int64_t workspace_bytes, hipStream_t st)
{
    return launch_wb_t<float>(sh, path, sig, gout, gpath, gbase, workspace, workspace_bytes, st);
}

hipError_t launch_wide_backward_f64(const Shape &sh, const double *path, const double *sig, const double *gout, double *gpath,
                                    double *gbase, void *workspace, int64_t workspace_bytes, hipStream_t st)
{
    return launch_wb_t<double>(sh, path, sig, gout, gpath, gbase, workspace, workspace_bytes, st);
}

}  // namespace sig
