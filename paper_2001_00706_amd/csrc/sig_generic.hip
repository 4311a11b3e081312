// Generic kernel family: any channel count d, any depth N, fp32 or fp64.
//
// One workgroup scans one path.  Each increment z is folded in with the fused
// multiply-exponentiate A <- A [x] exp(z) (paper section 4.1, eq. "fusedterm"):
//   new A_k = ((..((z/k + A_1) (x) z/(k-1) + A_2) ..) (x) z/2 + A_{k-1}) (x) z + A_k.
// Written element-wise, a work item owns one (k-1)-letter prefix p = w_1..w_{k-1} of
// level k: it runs the scalar Horner chain
//   u_1 = z[w_1]/k + A_1[w_1],   u_i = u_{i-1} * z[w_i]/(k-i+1) + A_i[w_1..w_i],
// and then updates the d words p.j of level k:  A_k[p.j] = u_{k-1} * z[j] + A_k[p.j].
// Levels are processed highest first, so every read of a lower level sees the old
// value and the update is in place.
//
// Where the state lives:
//   * final mode, small state: in LDS, copied to `out` at the end;
//   * final mode, large state: in the path's own slice of `out` (updated in place,
//     served by L2);
//   * stream mode: entry s of `out` is computed from entry s-1, so the output itself is
//     the state and every prefix signature is written exactly once.
// This family is the fallback that serves every shape; the shapes of the benchmark
// workloads have faster specialised kernels.
#include "sig_internal.h"

namespace sig {
namespace {

constexpr int kMaxThreads = 1024;
constexpr size_t kLdsBudget = 64 * 1024;  // dynamic LDS a workgroup may ask for without opting in

// I: type of the word indices inside one signature (32-bit whenever S < 2^31: integer division,
// which decodes the letters of a word, is several times cheaper than in 64 bits).
template <typename T, typename I>
__global__ void __launch_bounds__(kMaxThreads)
sig_generic_kernel(Shape sh, const T *__restrict__ path, T *out, int state_in_lds, int tile)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    T *zs = reinterpret_cast<T *>(smem_raw);  // zs[(m-1)*d + c] = z[c] / m, m = 1..N
    T *zinc = zs + int64_t(sh.N) * sh.d;      // increments of the current tile, [tile][d]
    T *lds_state = zinc + int64_t(tile) * sh.d;

    const int tid = threadIdx.x;
    const int nt = blockDim.x;
    const int d = sh.d;
    const int N = sh.N;
    const int64_t S = sh.S;

    for (int64_t b = blockIdx.x; b < sh.B; b += gridDim.x) {
        const ChunkView cv = chunk_view(b, sh.chunks, sh.chunk_len, sh.n_inc);
        const int64_t n_inc = cv.n;
        const T *x = path + cv.path * sh.L * d;
        const T *bpv = static_cast<const T *>(sh.basepoint_value);
        T *obase = out + b * (sh.stream ? sh.n_inc * S : S);
        T *cur = nullptr;
        const T *prev = nullptr;
        if (!sh.stream) {
            // the identity of the group is the all-zero element (its k = 0 term is implicit)
            cur = state_in_lds ? lds_state : obase;
            for (int64_t i = tid; i < S; i += nt) cur[i] = T(0);
            prev = cur;
        }
        __syncthreads();

        for (int64_t s = 0; s < n_inc; ++s) {
            const int in_tile = int(s % tile);
            if (in_tile == 0) {
                // stage the increments of the next `tile` steps: one trip to memory per tile, not per step
                const int64_t left = n_inc - s;
                const int n_stage = int(left < tile ? left : tile) * d;
                for (int i = tid; i < n_stage; i += nt) {
                    const int64_t si = cv.inc0 + s + i / d;
                    const int c = i % d;
                    T hi, lo;
                    if (sh.basepoint) {
                        hi = x[si * d + c];
                        lo = si > 0 ? x[(si - 1) * d + c] : bpv != nullptr ? bpv[cv.path * d + c] : T(0);
                    } else {
                        hi = x[(si + 1) * d + c];
                        lo = x[si * d + c];
                    }
                    zinc[i] = hi - lo;
                }
                __syncthreads();
            }
            // the scalings z/1 .. z/N of increment s (true divisions)
            for (int i = tid; i < N * d; i += nt) {
                const int m = i / d + 1;
                const int c = i - (m - 1) * d;
                zs[i] = zinc[in_tile * d + c] / T(m);
            }
            if (sh.stream) {
                cur = obase + s * S;
                prev = s == 0 ? nullptr : cur - S;
            }
            __syncthreads();

            for (int k = N; k >= 1; --k) {
                const I n_pref = I(sh.pw[k - 1]);
                for (I p = tid; p < n_pref; p += nt) {
                    T u = T(0);
                    if (k >= 2) {
                        I q = p / I(sh.pw[k - 2]);  // first letter
                        u = zs[(k - 1) * d + q] + (prev ? prev[I(sh.off[1]) + q] : T(0));
                        for (int i = 2; i <= k - 1; ++i) {
                            q = p / I(sh.pw[k - 1 - i]);   // index of the i-letter prefix
                            const int w = int(q % I(d));   // its last letter
                            u = u * zs[(k - i) * d + w] + (prev ? prev[I(sh.off[i]) + q] : T(0));
                        }
                    }
                    T *dst = cur + I(sh.off[k]) + p * I(d);
                    const T *src = prev ? prev + I(sh.off[k]) + p * I(d) : nullptr;
                    if (k >= 2) {
                        for (int j = 0; j < d; ++j) dst[j] = u * zs[j] + (src ? src[j] : T(0));
                    } else {
                        for (int j = 0; j < d; ++j) dst[j] = zs[j] + (src ? src[j] : T(0));
                    }
                }
                // in place: level k-1 may only be overwritten once every reader of its old
                // value (the chains of level k) is done
                if (!sh.stream) {
                    __threadfence_block();
                    __syncthreads();
                }
            }
            if (sh.stream) {
                __threadfence_block();
                __syncthreads();
            }
        }

        if (!sh.stream && state_in_lds) {
            for (int64_t i = tid; i < S; i += nt) obase[i] = lds_state[i];
        }
        __syncthreads();
    }
}

template <typename T>
hipError_t launch_generic(const Shape &sh, const T *path, T *out, hipStream_t st)
{
    size_t zs_bytes = sizeof(T) * size_t(sh.N) * size_t(sh.d);
    if (zs_bytes > kLdsBudget) return hipErrorInvalidValue;
    // increments staged per tile: up to 8 KB of them, at least one
    int64_t tile = int64_t(8192 / (sizeof(T) * size_t(sh.d)));
    if (tile < 1) tile = 1;
    if (tile > sh.n_inc) tile = sh.n_inc;
    while (tile > 1 && zs_bytes + sizeof(T) * size_t(tile) * size_t(sh.d) > kLdsBudget) tile /= 2;
    zs_bytes += sizeof(T) * size_t(tile) * size_t(sh.d);
    if (zs_bytes > kLdsBudget) return hipErrorInvalidValue;
    const size_t state_bytes = sizeof(T) * size_t(sh.S);
    const int state_in_lds = (!sh.stream && zs_bytes + state_bytes <= kLdsBudget) ? 1 : 0;
    const size_t lds = zs_bytes + (state_in_lds ? state_bytes : 0);
    // enough threads for the widest level's prefixes, in whole wavefronts
    const int64_t widest = sh.pw[sh.N - 1];
    int threads = 64;
    while (threads < kMaxThreads && threads < widest) threads *= 2;
    const int64_t max_grid = 1 << 20;
    const unsigned grid = unsigned(sh.B < max_grid ? sh.B : max_grid);
    if (sh.S < (int64_t(1) << 31)) {
        hipLaunchKernelGGL((sig_generic_kernel<T, uint32_t>), dim3(grid), dim3(threads), lds, st, sh, path, out, state_in_lds, int(tile));
    } else {
        hipLaunchKernelGGL((sig_generic_kernel<T, int64_t>), dim3(grid), dim3(threads), lds, st, sh, path, out, state_in_lds, int(tile));
    }
    return hipGetLastError();
}

}  // namespace

bool generic_supported(const Shape &sh, sig_dtype dtype)
{
    const size_t elem = dtype == SIG_F64 ? sizeof(double) : sizeof(float);
    return elem * (size_t(sh.N) + 1) * size_t(sh.d) <= kLdsBudget;  // the scalings and one staged increment
}

hipError_t launch_generic_f32(const Shape &sh, const float *path, float *out, hipStream_t st)
{
    return launch_generic<float>(sh, path, out, st);
}

hipError_t launch_generic_f64(const Shape &sh, const double *path, double *out, hipStream_t st)
{
    return launch_generic<double>(sh, path, out, st);
}

}  // namespace sig
