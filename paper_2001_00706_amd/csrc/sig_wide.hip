// Many channels (any d at N = 2 .. 9 up to 2^28 words of N - 1 letters; fp32 and fp64; final and stream mode): the kernel for d > 16, where
// the prefix-tree family has no instantiation (its channel count is a compile-time constant) and a signature is
// too large for the one-wavefront kernel.
//
// Arithmetic of the prefix-tree family (paper section 4.1, eq. "fusedterm": the new coefficient of a word needs the
// coefficients of that word's prefixes only) with the channel count a run-time value: a thread stands for a word u of
// N - 1 letters and a block of 16 (32, 64) last letters, carries the coefficients of u and of its prefixes (every thread below a
// prefix updates its own copy identically) and keeps the 16 top-level coefficients u j, j in its block, in
// registers.  Nothing is exchanged between threads, so the d^(N-1) * ceil(d / block) threads of a path may sit in any
// number of workgroups; paths with fewer than 256 threads share a workgroup.  The chain along the word is repeated
// by the ceil(d / block) threads of a word: a few multiply-adds against the block's 16 to 64.
#include "sig_internal.h"

namespace sig {
namespace {

constexpr int kWideTile = 32;    // increments staged in LDS at a time

__device__ __forceinline__ float wide_fma(float a, float b, float c) { return __builtin_fmaf(a, b, c); }
__device__ __forceinline__ double wide_fma(double a, double b, double c) { return __builtin_fma(a, b, c); }

struct WidePlan {
    int block;                // last letters per thread: 16, 32 or 64
    int jblocks;              // ceil(d / block)
    int dpad;                 // jblocks * block: floats per staged increment (zeros behind the d-th)
    int64_t threads;          // threads per path: d^(N-1) * jblocks
    int paths_per_group;      // paths sharing a workgroup (1 when a path has 256 threads or more)
    int64_t groups_per_path;  // workgroups per path (1 when paths share a workgroup)
};

template <typename T, int N, int WB>   // WB: last letters per thread, 16 or 32
__global__ void __launch_bounds__(256)
sig_wide_kernel(Shape sh, WidePlan pl, const T *__restrict__ path, T *__restrict__ out)
{
    constexpr int P = N - 1;
    extern __shared__ __align__(16) unsigned char wide_smem[];
    T *zt = reinterpret_cast<T *>(wide_smem);   // [paths_per_group][kWideTile][dpad]

    const int tid = threadIdx.x;
    const int d = sh.d;
    const bool shared_group = pl.threads < 256;
    const int slot_raw = shared_group ? tid / int(pl.threads) : 0;
    const int slot = slot_raw < pl.paths_per_group ? slot_raw : pl.paths_per_group - 1;   // threads beyond the last path idle along
    const int64_t t = shared_group ? tid - slot_raw * int(pl.threads) : int64_t(blockIdx.x % pl.groups_per_path) * 256 + tid;
    const int64_t row0 = shared_group ? int64_t(blockIdx.x) * pl.paths_per_group : int64_t(blockIdx.x / pl.groups_per_path);
    const int64_t row = row0 + slot;
    const bool live = t < pl.threads && slot_raw < pl.paths_per_group && row < sh.B;
    const int64_t u = (live ? t : 0) / pl.jblocks;          // the word of N - 1 letters
    const int jb = int((live ? t : 0) - u * pl.jblocks);    // the block of last letters
    const int j0 = jb * WB;

    int cl[P + 1];   // letters of the word
    {
        int64_t rest = u;
#pragma unroll
        for (int i = P; i >= 1; --i) {
            cl[i] = int(rest % d);
            rest /= d;
        }
    }
    T rk[N + 2];
#pragma unroll
    for (int m = 1; m <= N + 1; ++m) rk[m] = T(1) / T(m);

    T A[P + 1];             // coefficients of the prefixes of the word, and of the word itself (level N - 1)
    T top[WB];              // words u j, j = j0 .. j0 + WB - 1
#pragma unroll
    for (int i = 0; i <= P; ++i) A[i] = T(0);
#pragma unroll
    for (int c = 0; c < WB; ++c) top[c] = T(0);

    const T *bpv = static_cast<const T *>(sh.basepoint_value);
    // a row is a path or, in a chunked scan, a stretch of one: every row of a workgroup then walks chunk_len increments,
    // those past the end of a shorter stretch being zeros (which leave the state as it is)
    const int64_t n_inc = sh.chunks > 1 ? sh.chunk_len : sh.n_inc;
    // Stretches laid out inside a stream-mode output (Shape::rows_in_stream): in final mode a stretch writes its
    // signature to the row of its last increment; in stream mode it starts from the row before its first increment
    // and writes the rows of its increments but the last, which holds its final value already.
    const ChunkView mine = chunk_view(row < sh.B ? row : 0, sh.chunks, sh.chunk_len, sh.n_inc);
    T *stream_rows = out + (sh.rows_in_stream ? mine.path * sh.n_inc + mine.inc0 : row * sh.n_inc) * sh.S;
    const int64_t rows_to_write = sh.rows_in_stream ? mine.n - 1 : mine.n;
    // every block of 16 top-level scalars starts on a 16-byte boundary: signatures, levels and rows of d are whole
    // multiples of 16 bytes and so is the output's address
    constexpr int kPer16 = 16 / int(sizeof(T));
    const bool vec_ok = d % kPer16 == 0 && reinterpret_cast<uintptr_t>(out) % 16 == 0;

    // this thread's scalars of one signature; a prefix is written by the first thread below it
    auto store = [&](T *o) {
        if (jb == 0) {
            int64_t q = u, width = 1;
#pragma unroll
            for (int i = P; i >= 1; --i) {
                if (u % width == 0) o[sh.off[i] + q] = A[i];
                q /= d;
                width *= d;
            }
        }
        T *o_top = o + sh.off[N] + u * d + j0;
        if (vec_ok && j0 + WB <= d) {   // 16 bytes per store instead of one scalar
            constexpr int kVec = 16 / int(sizeof(T));
            typedef T TV __attribute__((ext_vector_type(kVec)));
#pragma unroll
            for (int c = 0; c < WB; c += kVec) {
                TV v;
#pragma unroll
                for (int k = 0; k < kVec; ++k) v[k] = top[c + k];
                *reinterpret_cast<TV *>(o_top + c) = v;
            }
        } else {
#pragma unroll
            for (int c = 0; c < WB; ++c)
                if (j0 + c < d) o_top[c] = top[c];
        }
    };

    if (sh.rows_in_stream && sh.stream && live && mine.inc0 > 0 && mine.n > 0) {
        const T *before = stream_rows - sh.S;   // the path's signature up to this stretch
        int64_t q = u;
#pragma unroll
        for (int i = P; i >= 1; --i) {
            A[i] = before[sh.off[i] + q];
            q /= d;
        }
#pragma unroll
        for (int c = 0; c < WB; ++c) top[c] = j0 + c < d ? before[sh.off[N] + u * d + j0 + c] : T(0);
    }

    const int row_floats = kWideTile * pl.dpad;
    for (int64_t t0 = 0; t0 < n_inc; t0 += kWideTile) {
        __syncthreads();
        // rows past the end of the batch, increments past the end of the path and the padding behind the last channel
        // add nothing; the loads are unconditional, on indices clamped into a path, and issued four scalars at a time
        // before the first use: a batch costs one trip to memory
        const int staged = pl.paths_per_group * row_floats;
        for (int e0 = 0; e0 < staged; e0 += 256 * 4) {
            T hi[4], lo[4];
            bool on[4], first[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (e0 + 256 * j >= staged) break;   // the same for every thread: nothing left to stage
                const int e = e0 + 256 * j + tid < staged ? e0 + 256 * j + tid : staged - 1;
                const int p = e / row_floats, r = e - p * row_floats, i = r / pl.dpad, c = r - i * pl.dpad;
                const ChunkView cv = chunk_view(row0 + p < sh.B ? row0 + p : 0, sh.chunks, sh.chunk_len, sh.n_inc);
                on[j] = row0 + p < sh.B && t0 + i < cv.n && c < d;
                const int64_t rp = cv.path;
                const T *x = path + rp * sh.L * d;
                const int cc = c < d ? c : 0;
                const int64_t i_hi = (on[j] ? cv.inc0 + t0 + i : 0) + (sh.basepoint ? 0 : 1);
                first[j] = i_hi == 0;   // the increment from the basepoint
                hi[j] = x[i_hi * d + cc];
                lo[j] = bpv != nullptr && first[j] ? bpv[rp * d + cc] : x[(first[j] ? 0 : i_hi - 1) * d + cc];
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int e = e0 + 256 * j + tid;
                if (e < staged) zt[e] = on[j] ? hi[j] - (first[j] && bpv == nullptr ? T(0) : lo[j]) : T(0);
            }
        }
        __syncthreads();
        const int nt = int(n_inc - t0 < kWideTile ? n_inc - t0 : kWideTile);
        const T *zrow = zt + slot * row_floats;
        for (int s = 0; s < nt; ++s, zrow += pl.dpad) {
            // Horner terms along the word: Hn[k] = T^(k)_i for the level i just passed, k > i
            T Hn[N + 2];
            {
                const T zc = zrow[cl[1]];
#pragma unroll
                for (int k = 2; k <= N; ++k) Hn[k] = wide_fma(zc, rk[k], A[1]);
                A[1] += zc;
            }
#pragma unroll
            for (int i = 2; i <= P; ++i) {
                const T zc = zrow[cl[i]];
                const T a = A[i];
                A[i] = wide_fma(Hn[i], zc, a);
#pragma unroll
                for (int k = i + 1; k <= N; ++k) Hn[k] = wide_fma(Hn[k], zc * rk[k - i + 1], a);
            }
#pragma unroll
            for (int c = 0; c < WB; c += kPer16) {   // the block's increments, 16 bytes per LDS read
                typedef T TZ __attribute__((ext_vector_type(kPer16)));
                const TZ zv = *reinterpret_cast<const TZ *>(zrow + j0 + c);
#pragma unroll
                for (int k = 0; k < kPer16; ++k) top[c + k] = wide_fma(Hn[N], zv[k], top[c + k]);
            }
            if (sh.stream && live && t0 + s < rows_to_write) store(stream_rows + (t0 + s) * sh.S);
        }
    }
    if (live && !sh.stream) {
        if (!sh.rows_in_stream)
            store(out + row * sh.S);
        else if (mine.n > 0)
            store(stream_rows + (mine.n - 1) * sh.S);
    }
}

bool wide_plan(const Shape &sh, WidePlan &pl)
{
    if (sh.N < 2 || sh.N > 9 || sh.d < 2 || (sh.chunks > 1 && sh.stream && !sh.rows_in_stream) || sh.S >= (int64_t(1) << 31)) return false;
    // From depth 3 on a thread also walks the chain along its word, about 12 multiply-adds' worth per increment: where the
    // channels fill whole blocks of 32 or 64 letters, the larger block halves or quarters the chain's share (1024 paths of
    // 128 points at d = 32, N = 3: 210 us against 337 with blocks of 16).
    pl.block = sh.N >= 3 && sh.N <= 4 && sh.d % 64 == 0 ? 64 : sh.N >= 3 && sh.N <= 4 && sh.d % 32 == 0 ? 32 : 16;
    pl.jblocks = (sh.d + pl.block - 1) / pl.block;
    pl.dpad = pl.jblocks * pl.block;
    pl.threads = sh.pw[sh.N - 1] * pl.jblocks;
    if (pl.threads > (int64_t(1) << 28)) return false;
    if (pl.threads >= 256) {
        pl.paths_per_group = 1;
        pl.groups_per_path = (pl.threads + 255) / 256;
    } else {
        const int fit = int(256 / pl.threads);
        pl.paths_per_group = fit < 16 ? fit : 16;
        pl.groups_per_path = 1;
    }
    return true;
}

template <typename T>
hipError_t launch_wide_t(const Shape &sh, const T *path, T *out, hipStream_t st)
{
    WidePlan pl;
    if (!wide_plan(sh, pl)) return hipErrorNotSupported;
    const size_t lds = size_t(pl.paths_per_group) * kWideTile * size_t(pl.dpad) * sizeof(T);
    if (lds > 64 * 1024) return hipErrorNotSupported;
    const int64_t groups = pl.threads >= 256 ? sh.B * pl.groups_per_path : (sh.B + pl.paths_per_group - 1) / pl.paths_per_group;
    if (groups > 0x7fffffff) return hipErrorNotSupported;
    const dim3 grid{unsigned(groups)}, block{256};
#define SIG_WIDE_LAUNCH(NN)                                                                                   \
    if (pl.block == 64)                                                                                       \
        hipLaunchKernelGGL((sig_wide_kernel<T, NN, 64>), grid, block, lds, st, sh, pl, path, out);            \
    else if (pl.block == 32)                                                                                  \
        hipLaunchKernelGGL((sig_wide_kernel<T, NN, 32>), grid, block, lds, st, sh, pl, path, out);            \
    else                                                                                                      \
        hipLaunchKernelGGL((sig_wide_kernel<T, NN, 16>), grid, block, lds, st, sh, pl, path, out)
    switch (sh.N) {
        case 2: SIG_WIDE_LAUNCH(2); break;
        case 3: SIG_WIDE_LAUNCH(3); break;
        case 4: SIG_WIDE_LAUNCH(4); break;
        // deeper: blocks of 16 only
        case 5: hipLaunchKernelGGL((sig_wide_kernel<T, 5, 16>), grid, block, lds, st, sh, pl, path, out); break;
        case 6: hipLaunchKernelGGL((sig_wide_kernel<T, 6, 16>), grid, block, lds, st, sh, pl, path, out); break;
        case 7: hipLaunchKernelGGL((sig_wide_kernel<T, 7, 16>), grid, block, lds, st, sh, pl, path, out); break;
        case 8: hipLaunchKernelGGL((sig_wide_kernel<T, 8, 16>), grid, block, lds, st, sh, pl, path, out); break;
        case 9: hipLaunchKernelGGL((sig_wide_kernel<T, 9, 16>), grid, block, lds, st, sh, pl, path, out); break;
        default: return hipErrorNotSupported;
    }
#undef SIG_WIDE_LAUNCH
    return hipGetLastError();
}

}  // namespace

bool wide_supported(const Shape &sh, sig_dtype dtype)
{
    WidePlan pl;
    if (!wide_plan(sh, pl)) return false;
    const size_t elem = dtype == SIG_F32 ? sizeof(float) : sizeof(double);
    return size_t(pl.paths_per_group) * kWideTile * size_t(pl.dpad) * elem <= 64 * 1024;
}

hipError_t launch_wide_f32(const Shape &sh, const float *path, float *out, hipStream_t st) { return launch_wide_t<float>(sh, path, out, st); }
hipError_t launch_wide_f64(const Shape &sh, const double *path, double *out, hipStream_t st) { return launch_wide_t<double>(sh, path, out, st); }

}  // namespace sig
