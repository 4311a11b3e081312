// Small-state kernel family: signatures of at most 512 scalars (e.g. d = 2 up to depth 8, d = 3 up
// to depth 5, any d at depth 1 or 2 while S <= 512), fp32 or fp64, final and stream mode.
//
// One wavefront scans one path; the state lives in LDS and every lane owns up to 8 words of it (1, 2, 4 or 8: a template parameter).
// The fused multiply-exponentiate (paper section 4.1, eq. "fusedterm") is applied element-wise:
// the new coefficient of a word w = w_1..w_k is the end of the scalar Horner chain
//     u_0 = 1,  u_i = u_{i-1} * z[w_i]/(k-i+1) + A_i[w_1..w_i],  A_k[w] <- u_k
// over the prefixes of w.  Which prefixes and letters a lane needs never changes, so they are
// decoded once, before the scan, into registers.  Every chain is run at full length N: a word of
// level k < N starts with N-k idle links u <- u * 1 + 0, which read a constant 1 kept at the end
// of every row of scaled increments and a constant 0 kept behind the state, so the step has no
// divergent control flow.  The scaled increments z/m, m = 1..N, are tabulated for a whole tile of
// increments at a time; a step is then 2N LDS reads and N FMAs per word.  A workgroup is a single
// wavefront, whose LDS accesses complete in program order, so a step reads all of its operands from
// the old state and then overwrites the state in place.
#include "sig_internal.h"

namespace sig {
namespace {

constexpr int kSmallMaxWords = 512;   // S this family accepts
constexpr int kSmallTile = 64;        // increments staged in LDS at a time

// n / d for 0 <= n < 4096 and 1 <= d <= 64 with magic = ceil(2^20 / d): the product stays below 2^32
// and the excess n * (magic*d - 2^20) / (d * 2^20) < n / 2^20 < 1/d never carries into the quotient.
__device__ __forceinline__ int small_div(int n, unsigned magic) { return int((unsigned(n) * magic) >> 20); }

// W = words of the state per lane (the state has at most 64 W scalars).
template <typename T, int N, int W>
__global__ void __launch_bounds__(64)
sig_small_kernel(Shape sh, const T *__restrict__ path, T *__restrict__ out)
{
    __shared__ T st[kSmallMaxWords + 64];             // state; st[S] stays 0
    extern __shared__ __align__(16) unsigned char smem_raw[];
    T *zt = reinterpret_cast<T *>(smem_raw);          // zt[s*row + (m-1)*d + c] = z_s[c]/m, zt[s*row + N*d] = 1

    const int lane = threadIdx.x;
    const int d = sh.d;
    const int S = int(sh.S);
    const int row = N * d + 1;
    const unsigned magic = ((1u << 20) + unsigned(d) - 1u) / unsigned(d);

    // decode this lane's words once: link i of word j reads the state at where[j][i] >> 16 and the
    // scaled increment at (where[j][i] & 0xffff) of the current row
    int where[W][N];
#pragma unroll
    for (int j = 0; j < W; ++j) {
        const int wi = lane + 64 * j;
#pragma unroll
        for (int i = 0; i < N; ++i) where[j][i] = (S << 16) | (N * d);   // idle link
        if (wi < S) {
            int k = 1;
            while (k < N && wi >= int(sh.off[k + 1])) ++k;
            int idx = wi - int(sh.off[k]);  // index inside level k
#pragma unroll
            for (int i = N; i >= 1; --i) {
                if (i <= k) {
                    // prefix of i letters; its last letter is scaled by 1/(k-i+1)
                    const int q = small_div(idx, magic);
                    where[j][N - k + i - 1] = ((int(sh.off[i]) + idx) << 16) | ((k - i) * d + idx - q * d);
                    idx = q;
                }
            }
        }
    }

    for (int64_t b = blockIdx.x; b < sh.B; b += gridDim.x) {
        const ChunkView cv = chunk_view(b, sh.chunks, sh.chunk_len, sh.n_inc);
        const int64_t n_inc = cv.n;
        const T *x = path + cv.path * sh.L * d;
        const T *bpv = static_cast<const T *>(sh.basepoint_value);
        // rows of a stream-mode output when the chunks are laid out there: o is then the row of the first increment
        const int64_t first_row = cv.path * sh.n_inc + cv.inc0;
        T *o = out + (sh.rows_in_stream ? first_row : sh.stream ? b * sh.n_inc : b) * int64_t(S);
        const bool resume = sh.rows_in_stream && sh.stream && cv.inc0 > 0 && n_inc > 0;
        for (int i = lane; i <= S; i += 64) st[i] = resume && i < S ? o[i - S] : T(0);   // o - S: the row before
        const int64_t n_rows = sh.rows_in_stream ? n_inc - 1 : n_inc;   // a chunk's last row holds its value already

        for (int64_t t0 = 0; t0 < n_inc; t0 += kSmallTile) {
            const int nt = int(n_inc - t0 < kSmallTile ? n_inc - t0 : kSmallTile);
            __syncthreads();
            for (int i = lane; i < nt * d; i += 64) {
                const int si = small_div(i, magic);
                const int c = i - si * d;
                const int64_t s = cv.inc0 + t0 + si;
                T hi, lo;
                if (sh.basepoint) {
                    hi = x[s * d + c];
                    lo = s > 0 ? x[(s - 1) * d + c] : bpv != nullptr ? bpv[cv.path * d + c] : T(0);
                } else {
                    hi = x[(s + 1) * d + c];
                    lo = x[s * d + c];
                }
                const T z = hi - lo;
#pragma unroll
                for (int m = 1; m <= N; ++m) zt[si * row + (m - 1) * d + c] = z / T(m);
            }
            if (lane < nt) zt[lane * row + N * d] = T(1);
            __syncthreads();
            for (int s = 0; s < nt; ++s) {
                const T *zr = zt + s * row;
                T fresh[W];
#pragma unroll
                for (int j = 0; j < W; ++j) {
                    T zi[N], a[N];
#pragma unroll
                    for (int i = 0; i < N; ++i) {
                        zi[i] = zr[where[j][i] & 0xffff];
                        a[i] = st[where[j][i] >> 16];
                    }
                    T u = T(1);
#pragma unroll
                    for (int i = 0; i < N; ++i) u = u * zi[i] + a[i];
                    fresh[j] = u;
                }
                __syncthreads();
#pragma unroll
                for (int j = 0; j < W; ++j) {
                    const int wi = lane + 64 * j;
                    if (wi < S) {
                        st[wi] = fresh[j];
                        if (sh.stream && t0 + s < n_rows) o[(t0 + s) * S + wi] = fresh[j];
                    }
                }
                __syncthreads();
            }
        }
        if (!sh.stream && !(sh.rows_in_stream && n_inc == 0))
            for (int i = lane; i < S; i += 64) o[(sh.rows_in_stream ? (n_inc - 1) * int64_t(S) : 0) + i] = st[i];
        __syncthreads();
    }
}

template <typename T, int N>
hipError_t launch_small_n(const Shape &sh, const T *path, T *out, hipStream_t st)
{
    const size_t lds = sizeof(T) * size_t(kSmallTile) * (size_t(N) * size_t(sh.d) + 1);
    const int64_t max_grid = 1 << 20;
    const unsigned grid = unsigned(sh.B < max_grid ? sh.B : max_grid);
    if (sh.S <= 64)
        hipLaunchKernelGGL((sig_small_kernel<T, N, 1>), dim3(grid), dim3(64), lds, st, sh, path, out);
    else if (sh.S <= 128)
        hipLaunchKernelGGL((sig_small_kernel<T, N, 2>), dim3(grid), dim3(64), lds, st, sh, path, out);
    else if (sh.S <= 256)
        hipLaunchKernelGGL((sig_small_kernel<T, N, 4>), dim3(grid), dim3(64), lds, st, sh, path, out);
    else
        hipLaunchKernelGGL((sig_small_kernel<T, N, 8>), dim3(grid), dim3(64), lds, st, sh, path, out);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_small(const Shape &sh, const T *path, T *out, hipStream_t st)
{
    switch (sh.N) {
        case 1: return launch_small_n<T, 1>(sh, path, out, st);
        case 2: return launch_small_n<T, 2>(sh, path, out, st);
        case 3: return launch_small_n<T, 3>(sh, path, out, st);
        case 4: return launch_small_n<T, 4>(sh, path, out, st);
        case 5: return launch_small_n<T, 5>(sh, path, out, st);
        case 6: return launch_small_n<T, 6>(sh, path, out, st);
        case 7: return launch_small_n<T, 7>(sh, path, out, st);
        case 8: return launch_small_n<T, 8>(sh, path, out, st);
    }
    return hipErrorNotSupported;
}

}  // namespace

bool small_supported(const Shape &sh)
{
    // S <= 512 bounds N*d by 64 (d = 64 at depth 1), so one tile of scaled increments is at most
    // 64 * 65 scalars: with the state, well inside the 64 KB of LDS a workgroup gets by default
    return sh.S <= kSmallMaxWords && sh.N <= 8 && sh.d <= 64;
}

hipError_t launch_small_f32(const Shape &sh, const float *path, float *out, hipStream_t st)
{
    return small_supported(sh) ? launch_small<float>(sh, path, out, st) : hipErrorNotSupported;
}

hipError_t launch_small_f64(const Shape &sh, const double *path, double *out, hipStream_t st)
{
    return small_supported(sh) ? launch_small<double>(sh, path, out, st) : hipErrorNotSupported;
}

}  // namespace sig
