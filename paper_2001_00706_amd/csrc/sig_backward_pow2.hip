// Gradient of the signature with respect to the path for d = 2 (N = 2..9) and d = 8 (N = 2..5), fp32
// (paper section 5.3, appendix C): the register-resident scheme of sig_backward_d4.hip written once for any
// power-of-two channel count.
//
// With LG = log2(d), a thread stands for a word of P = min(N, 6/LG + 1) letters (its base-d digits), so that
// the threads below one first letter fill exactly one wavefront (or the whole path fits one).  A thread
// holds the signature A and its cotangent G at its own word and at that word's ancestors (redundantly: all
// threads below an ancestor carry the same value), and the up to two levels below its word as small arrays.
// "Up" (undo the increment, Horner terms T^(k)_i) is a scalar chain along the thread's word.  "Down" sums
// the chains D^(k)_i over the d siblings of each level with lane exchanges inside the wavefront; the only
// workgroup-wide step is the sum of the increments' gradients over the wavefronts, once per tile of 64
// increments.  See sig_backward.hip for the recurrences.
#include "sig_internal.h"
#include "sig_mfma_common.h"
#include "sig_lane_ops.h"

namespace sig {
namespace {

constexpr int kTileP = 64;   // increments staged in LDS at a time

__host__ __device__ constexpr int ilog2(int d) { return d == 2 ? 1 : d == 4 ? 2 : 3; }
__host__ __device__ constexpr int word_letters(int d, int N) { return N < 6 / ilog2(d) + 1 ? N : 6 / ilog2(d) + 1; }
__host__ __device__ constexpr int ipow(int d, int k) { return k <= 0 ? 1 : d * ipow(d, k - 1); }
__host__ __device__ constexpr int level_off(int d, int k)   // offset of level k (1-based) in a flat element
{
    int off = 0;
    for (int j = 1; j < k; ++j) off += ipow(d, j);
    return off;
}

// D consecutive floats from a pointer aligned to min(D, 4) floats.
template <int D>
__device__ __forceinline__ void load_letters(const float *p, float (&v)[D])
{
    if constexpr (D == 2) {
        const float2 a = *reinterpret_cast<const float2 *>(p);
        v[0] = a.x;
        v[1] = a.y;
    } else {
#pragma unroll
        for (int i = 0; i < D / 4; ++i) {
            const f4 a = reinterpret_cast<const f4 *>(p)[i];
            v[4 * i] = a[0];
            v[4 * i + 1] = a[1];
            v[4 * i + 2] = a[2];
            v[4 * i + 3] = a[3];
        }
    }
}

// The "down" pass at levels J, J-1, .. 1, where a thread holds one scalar per chain: chains k = J..N with
// value G_J (k = J) or Dc[k] = D^(k)_J (k > J) at the thread's ancestor of level J.  Adds the level's share of
// the increment's gradient to dz (weighed by the number of threads that hold the same ancestor), replaces
// Dc by the chains of level J-1 (sums over the D siblings, i.e. over lane-number bits LG*(P-J) and up), and
// adds the chains k > J into the cotangent G_J.
template <int D, int N, int J>
struct ScalarLevels {
    static constexpr int LG = ilog2(D), P = word_letters(D, N);
    static __device__ __forceinline__ void run(float (&Glo)[P + 1], const float (&T)[P + 1][N + 2], float (&Dc)[N + 2],
                                               float (&dz)[D], const float (&zc)[P + 1], const int (&cl)[P + 1],
                                               const float (&rk)[N + 2])
    {
        float contrib = J >= 2 ? T[J >= 2 ? J - 1 : 1][J] * Glo[J] : Glo[J];   // T^(k)_0 = 1
        float g_add = 0.0f;
#pragma unroll
        for (int k = J + 1; k <= N; ++k) {
            const float tp = J >= 2 ? T[J >= 2 ? J - 1 : 1][k] * rk[k - J + 1] : rk[k - J + 1];
            contrib = __builtin_fmaf(tp, Dc[k], contrib);
            g_add += Dc[k];
        }
        if constexpr (J >= 2) {
            float E[N + 2];
            E[J] = Glo[J] * zc[J];
#pragma unroll
            for (int k = J + 1; k <= N; ++k) E[k] = Dc[k] * (zc[J] * rk[k - J + 1]);
#pragma unroll
            for (int k = J; k <= N; ++k) Dc[k] = group_sum<LG * (P - J), LG>(E[k]);
        }
        Glo[J] += g_add;
        contrib *= 1.0f / float(ipow(D, P - J));   // a power of two: exact
#pragma unroll
        for (int c = 0; c < D; ++c) dz[c] += cl[J] == c ? contrib : 0.0f;
        if constexpr (J > 1) ScalarLevels<D, N, J - 1>::run(Glo, T, Dc, dz, zc, cl, rk);
    }
};

template <int D, int N>
struct Pow2Shape {
    static constexpr int LG = ilog2(D);
    static constexpr int P = word_letters(D, N);   // letters of a thread's word
    static constexpr int U = N - P;                // levels below it, kept as arrays
    static constexpr int NT = ipow(D, P);          // threads that carry a word
    static constexpr int NTL = NT < 64 ? 64 : NT;  // threads launched
    static constexpr int NW = NTL / 64;
    static_assert(U >= 0 && U <= 2, "at most two levels below the thread's word");
};

template <int D, int N, bool STREAM>
__global__ void __launch_bounds__((Pow2Shape<D, N>::NTL))
sig_backward_pow2_kernel(const float *__restrict__ path, const float *__restrict__ sig, const float *__restrict__ gout,
                         float *__restrict__ gpath, float *__restrict__ gbase, int64_t L, int64_t n_inc, int basepoint,
                         const float *__restrict__ bpv)
{
    using PS = Pow2Shape<D, N>;
    constexpr int LG = PS::LG, P = PS::P, U = PS::U, NT = PS::NT, NW = PS::NW;
    constexpr int kS = level_off(D, N + 1);
    constexpr int H1 = U >= 1 ? D : 1, H2 = U >= 2 ? D * D : 1;
    // stream mode fetches the entries of the next step one step ahead, unless a thread's share is so large
    // that holding two of them would spill registers
    constexpr bool kPrefetch = H1 + H2 <= 24;

    __shared__ __align__(16) float zt[kTileP * D];   // the increments of the current tile
    __shared__ float part[kTileP][NW][D];            // [increment of the tile][wavefront][letter]: partial gradients
    __shared__ float dzs[kTileP][D];                 // gradients of the tile's increments
    __shared__ float dz_after[D];                    // gradient of the increment that follows the tile's last one

    const int tl = threadIdx.x;
    const bool active = tl < NT;
    const int t = tl & (NT - 1);   // idle lanes shadow a word; they are kept out of every sum and store
    const int wave = tl >> 6;
    int cl[P + 1], ul[P + 1];      // this thread's letter and ancestor index at levels 1..P
#pragma unroll
    for (int i = 1; i <= P; ++i) {
        ul[i] = t >> (LG * (P - i));
        cl[i] = ul[i] & (D - 1);
    }
    float rk[N + 2];
#pragma unroll
    for (int m = 1; m <= N + 1; ++m) rk[m] = 1.0f / float(m);

    const int64_t b = blockIdx.x;
    const float *x = path + b * L * D;
    const int64_t per_path = STREAM ? n_inc * int64_t(kS) : int64_t(kS);
    const float *sg = sig + b * per_path;
    const float *go = gout + b * per_path;
    float *gp = gpath + b * L * D;

    struct Share {
        float lo[P + 1];
        float h1[H1];
        float h2[H2];
    };
    // with_h1 / with_h2: whether the levels P+1 / P+2 are wanted
    auto load_share = [&](const float *e, bool with_h1, bool with_h2) {
        Share s = {};
#pragma unroll
        for (int i = 1; i <= P; ++i) s.lo[i] = e[level_off(D, i) + ul[i]];
        if constexpr (U >= 1) {
            if (with_h1) load_letters<D>(e + level_off(D, P + 1) + t * D, s.h1);
        }
        if constexpr (U >= 2) {
            if (with_h2) {
#pragma unroll
                for (int c = 0; c < D; ++c) {
                    float row[D];
                    load_letters<D>(e + level_off(D, P + 2) + (t * D + c) * D, row);
#pragma unroll
                    for (int j = 0; j < D; ++j) s.h2[c * D + j] = row[j];
                }
            }
        }
        return s;
    };

    // G: cotangent of the signature after the increment being processed.  A: that signature below its top level.
    Share G = load_share(STREAM ? go + (n_inc - 1) * int64_t(kS) : go, true, true);
    Share A = {}, nextA = {}, nextG = {};
    if constexpr (!STREAM) A = load_share(sg, U >= 2, false);

    if (tl < D) dz_after[tl] = 0.0f;   // no increment follows the last one

    for (int64_t t0 = ((n_inc - 1) / kTileP) * kTileP; t0 >= 0; t0 -= kTileP) {
        const int nt = int(n_inc - t0 < kTileP ? n_inc - t0 : kTileP);
        __syncthreads();
        for (int i = tl; i < nt * D; i += PS::NTL) {
            const int64_t s = t0 + i / D;
            const int c = i % D;
            const int64_t i_hi = basepoint ? s : s + 1;
            const float lo = i_hi > 0 ? x[(i_hi - 1) * D + c] : bpv != nullptr ? bpv[b * D + c] : 0.0f;
            zt[i] = x[i_hi * D + c] - lo;
        }
        if constexpr (STREAM && kPrefetch) {
            const int64_t s = t0 + nt - 1;
            if (s > 0) {
                nextA = load_share(sg + (s - 1) * int64_t(kS), U >= 2, false);
                nextG = load_share(go + (s - 1) * int64_t(kS), true, true);
            } else {
                nextA = Share{};
            }
        }
        __syncthreads();

        for (int i = nt - 1; i >= 0; --i) {
            const int64_t s = t0 + i;
            float zc[P + 1];   // the increment at this thread's letters
#pragma unroll
            for (int j = 1; j <= P; ++j) zc[j] = zt[i * D + cl[j]];
            float zu[D];       // the whole increment
            if constexpr (U >= 1) load_letters<D>(zt + i * D, zu);

            Share addG = {};
            if constexpr (STREAM && !kPrefetch) {
                A = s > 0 ? load_share(sg + (s - 1) * int64_t(kS), U >= 2, false) : Share{};
            }
            if constexpr (STREAM && kPrefetch) {
                A = nextA;      // signature after s increments = output entry s-1 (zero for s = 0)
                addG = nextG;   // output gradient of entry s-1, added once this step is done
                if (i > 0) {
                    if (s - 1 > 0) {
                        nextA = load_share(sg + (s - 2) * int64_t(kS), U >= 2, false);
                        nextG = load_share(go + (s - 2) * int64_t(kS), true, true);
                    } else {
                        nextA = Share{};
                    }
                }
            }

            // ---- up: T[j][k] = T^(k)_j at this thread's word; the signature before the increment
            float T[P + 1][N + 2];
            float a_lo[P + 1];
            a_lo[1] = STREAM ? A.lo[1] : A.lo[1] - zc[1];
#pragma unroll
            for (int k = 2; k <= N; ++k) T[1][k] = __builtin_fmaf(zc[1], rk[k], a_lo[1]);
#pragma unroll
            for (int j = 2; j <= P; ++j) {
                if (j < N) {
                    a_lo[j] = STREAM ? A.lo[j] : __builtin_fmaf(-T[j - 1][j], zc[j], A.lo[j]);
#pragma unroll
                    for (int k = j + 1; k <= N; ++k) T[j][k] = __builtin_fmaf(T[j - 1][k], zc[j] * rk[k - j + 1], a_lo[j]);
                } else {
                    a_lo[j] = 0.0f;
                }
            }
            float a_h1[H1], Th1[H1];   // level P+1 of the earlier signature; T^(N)_{P+1}[word c]
            if constexpr (U >= 2) {
#pragma unroll
                for (int c = 0; c < D; ++c) {
                    a_h1[c] = STREAM ? A.h1[c] : __builtin_fmaf(-T[P][P + 1], zu[c], A.h1[c]);
                    Th1[c] = __builtin_fmaf(T[P][N], zu[c] * rk[2], a_h1[c]);
                }
            }
            if constexpr (!STREAM) {
#pragma unroll
                for (int j = 1; j <= P; ++j) A.lo[j] = a_lo[j];
                if constexpr (U >= 2) {
#pragma unroll
                    for (int c = 0; c < D; ++c) A.h1[c] = a_h1[c];
                }
            }

            // ---- down
            float dz[D];
#pragma unroll
            for (int c = 0; c < D; ++c) dz[c] = 0.0f;
            float Dc[N + 2];   // Dc[k] = D^(k)_j at this thread's ancestor of the level j being processed, k > j
#pragma unroll
            for (int k = 0; k <= N + 1; ++k) Dc[k] = 0.0f;
            float Dh[H1];      // D^(N)_{P+1}[word c]
            if constexpr (U >= 2) {
#pragma unroll
                for (int c = 0; c < D; ++c) {
                    float acc = 0.0f;
#pragma unroll
                    for (int j = 0; j < D; ++j) {
                        acc = __builtin_fmaf(G.h2[c * D + j], zu[j], acc);
                        dz[j] = __builtin_fmaf(Th1[c], G.h2[c * D + j], dz[j]);
                    }
                    Dh[c] = acc;
                }
            }
            if constexpr (U >= 1) {
                // level P+1: chains k = P+1 (G.h1, divisor 1) and k = P+2 (Dh, divisor 2)
                float acc1 = 0.0f, acc2 = 0.0f;
#pragma unroll
                for (int c = 0; c < D; ++c) {
                    dz[c] = __builtin_fmaf(T[P][P + 1], G.h1[c], dz[c]);
                    acc1 = __builtin_fmaf(G.h1[c], zu[c], acc1);
                    if constexpr (U >= 2) {
                        dz[c] = __builtin_fmaf(T[P][P + 2] * rk[2], Dh[c], dz[c]);
                        acc2 = __builtin_fmaf(Dh[c], zu[c], acc2);
                        G.h1[c] += Dh[c];
                    }
                }
                Dc[P + 1] = acc1;
                if constexpr (U >= 2) Dc[P + 2] = acc2 * rk[2];
            }
            // levels P .. 1, one scalar per thread and chain; level j is shared by the D^(P-j) threads below it
            ScalarLevels<D, N, PS::P>::run(G.lo, T, Dc, dz, zc, cl, rk);

            // ---- the increment's gradient: sum over the wavefront; the wavefronts leave their partial sums in
            // LDS and do not wait for one another inside a tile
#pragma unroll
            for (int c = 0; c < D; ++c) {
                const float total = group_sum<0, 6>(active ? dz[c] : 0.0f);
                if ((tl & 63) == 0) part[i][wave][c] = total;
            }

            if constexpr (STREAM) {
                if (s > 0) {
                    if constexpr (!kPrefetch) addG = load_share(go + (s - 1) * int64_t(kS), true, true);
#pragma unroll
                    for (int j = 1; j <= P; ++j) G.lo[j] += addG.lo[j];
                    if constexpr (U >= 1) {
#pragma unroll
                        for (int c = 0; c < D; ++c) G.h1[c] += addG.h1[c];
                    }
                    if constexpr (U >= 2) {
#pragma unroll
                        for (int c = 0; c < D * D; ++c) G.h2[c] += addG.h2[c];
                    }
                }
            }
        }

        // the tile's gradients: sum over the wavefronts, then every point of the tile gets the gradient of the
        // increment it ends minus that of the increment it starts
        __syncthreads();
        for (int e = tl; e < nt * D; e += PS::NTL) {
            const int i = e / D, c = e % D;
            float sum = 0.0f;
#pragma unroll
            for (int w = 0; w < NW; ++w) sum += part[i][w][c];
            dzs[i][c] = sum;
        }
        __syncthreads();
        for (int e = tl; e < nt * D; e += PS::NTL) {
            const int i = e / D, c = e % D;
            const int64_t point = (basepoint ? t0 : t0 + 1) + i;
            gp[point * D + c] = dzs[i][c] - (i + 1 < nt ? dzs[i + 1][c] : dz_after[c]);
        }
        __syncthreads();
        if (tl < D) dz_after[tl] = dzs[0][tl];   // this tile's first increment follows the last one of the tile before it
    }
    __syncthreads();
    if (tl < D) {
        // dz_after now holds the gradient of increment 0
        if (!basepoint) gp[tl] = -dz_after[tl];                           // the first point only starts increment 0
        else if (gbase != nullptr) gbase[b * D + tl] = -dz_after[tl];     // and so does a basepoint
    }
}

template <int D, int N>
hipError_t launch_pow2(const Shape &sh, const float *path, const float *sig, const float *gout, float *gpath,
                       float *gbase, hipStream_t st)
{
    const dim3 grid(static_cast<unsigned>(sh.B)), block(Pow2Shape<D, N>::NTL);
    const float *bpv = static_cast<const float *>(sh.basepoint_value);
    if (sh.stream)
        hipLaunchKernelGGL((sig_backward_pow2_kernel<D, N, true>), grid, block, 0, st, path, sig, gout, gpath, gbase, sh.L,
                           sh.n_inc, sh.basepoint, bpv);
    else
        hipLaunchKernelGGL((sig_backward_pow2_kernel<D, N, false>), grid, block, 0, st, path, sig, gout, gpath, gbase, sh.L,
                           sh.n_inc, sh.basepoint, bpv);
    return hipGetLastError();
}

}  // namespace

bool backward_pow2_supported(const Shape &sh)
{
    if (sh.B > 0x7fffffff) return false;
    return (sh.d == 2 && sh.N >= 2 && sh.N <= 9) || (sh.d == 8 && sh.N >= 2 && sh.N <= 5);
}

hipError_t launch_backward_pow2_f32(const Shape &sh, const float *path, const float *sig, const float *gout, float *gpath,
                                    float *gbase, hipStream_t st)
{
    if (!backward_pow2_supported(sh)) return hipErrorNotSupported;
    if (sh.d == 2) {
        switch (sh.N) {
            case 2: return launch_pow2<2, 2>(sh, path, sig, gout, gpath, gbase, st);
            case 3: return launch_pow2<2, 3>(sh, path, sig, gout, gpath, gbase, st);
            case 4: return launch_pow2<2, 4>(sh, path, sig, gout, gpath, gbase, st);
            case 5: return launch_pow2<2, 5>(sh, path, sig, gout, gpath, gbase, st);
            case 6: return launch_pow2<2, 6>(sh, path, sig, gout, gpath, gbase, st);
            case 7: return launch_pow2<2, 7>(sh, path, sig, gout, gpath, gbase, st);
            case 8: return launch_pow2<2, 8>(sh, path, sig, gout, gpath, gbase, st);
            default: return launch_pow2<2, 9>(sh, path, sig, gout, gpath, gbase, st);
        }
    }
    switch (sh.N) {
        case 2: return launch_pow2<8, 2>(sh, path, sig, gout, gpath, gbase, st);
        case 3: return launch_pow2<8, 3>(sh, path, sig, gout, gpath, gbase, st);
        case 4: return launch_pow2<8, 4>(sh, path, sig, gout, gpath, gbase, st);
        default: return launch_pow2<8, 5>(sh, path, sig, gout, gpath, gbase, st);
    }
}

}  // namespace sig
