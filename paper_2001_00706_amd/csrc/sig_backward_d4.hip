// Gradient of the signature with respect to the path for d = 4, N = 4..6, fp32 (paper section 5.3,
// appendix C): the recurrences of sig_backward.hip with the whole working set in registers.
//
// One workgroup of 256 threads per path.  Thread t stands for the four-letter word u = w1 w2 w3 w4 whose
// base-4 digits are those of t (w1 = the wavefront, w4 = t % 4).  It keeps
//   * the signature A and its cotangent G at its own word (level 4), at the words u c (level 5) and
//     u c c' (level 6, cotangent only: the top level of A is never needed), and
//   * at its ancestors w1, w1 w2, w1 w2 w3 (levels 1..3), redundantly: the 4, 16 or 64 threads below an
//     ancestor all hold and update the same value with the same arithmetic.
// "Up" (undo the increment, form the Horner terms T^(k)_i) is then a scalar chain along the thread's own
// word with no communication at all.  "Down", the chains D^(k)_i contracted with the increment, needs
// sums over the 4 threads of a quad (level 4 -> 3), the 4 quads of a 16-lane row (3 -> 2) and the 4 rows
// of a wavefront (2 -> 1): lane permutes inside a wavefront, no LDS, no barrier; wavefronts (first
// letters) never exchange anything.  The only workgroup-wide step is the sum of the increments' gradients
// over the four wavefronts, done once per tile of 64 increments from partial sums left in LDS.  Redundant
// holders weigh their contribution to that sum by 1/4, 1/16, 1/64 (exact in binary).
//
// Stream mode reads the earlier signature from the forward output instead of undoing the increment, and
// adds the output gradient of every entry on the way; both are fetched one increment ahead.
#include "sig_internal.h"
#include "sig_mfma_common.h"

namespace sig {
namespace {

constexpr int kOff4[8] = {0, 0, 4, 20, 84, 340, 1364, 5460};  // offset of level k; kOff4[N + 1] = S
constexpr int kTileB = 64;                                    // increments staged in LDS at a time

// Sum over the 4 lanes of a quad, in every lane.
__device__ __forceinline__ float quad_sum(float v)
{
    v += quad_swap<0xB1>(v);   // quad_perm [1,0,3,2]
    v += quad_swap<0x4E>(v);   // quad_perm [2,3,0,1]
    return v;
}

// Sum over the lanes i, i+4, i+8, i+12 of a 16-lane row, in each of them: for a value that is the same in the 4
// lanes of each quad, the sum over the 4 quads of the row.
__device__ __forceinline__ float row_sum_of_quads(float v)
{
    v += quad_swap<0x124>(v);  // row_ror:4
    v += quad_swap<0x128>(v);  // row_ror:8
    return v;
}

// Sum over the lanes i, i+16, i+32, i+48, in each of them: for a value that is the same in the 16 lanes of each
// row, the sum over the 4 rows of the wavefront.
__device__ __forceinline__ float wave_sum_of_rows(float v)
{
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    return v;
}

template <int N, bool STREAM>
__global__ void __launch_bounds__(256)
sig_backward_d4_kernel(const float *__restrict__ path, const float *__restrict__ sig, const float *__restrict__ gout,
                       float *__restrict__ gpath, float *__restrict__ gbase, int64_t L, int64_t n_inc, int basepoint,
                       const float *__restrict__ bpv)
{
    static_assert(N >= 4 && N <= 6, "depths served by this kernel");
    constexpr int kS = kOff4[N + 1];
    constexpr float r2 = 1.0f / 2, r3 = 1.0f / 3, r4 = 1.0f / 4, r5 = 1.0f / 5, r6 = 1.0f / 6;
    constexpr float rk[7] = {0.0f, 1.0f, r2, r3, r4, r5, r6};

    __shared__ __align__(16) float zt[kTileB * 4];   // the increments of the current tile
    __shared__ float part[kTileB][4][4];             // [increment of the tile][wavefront][letter]: partial gradients
    __shared__ float dzs[kTileB][4];                 // gradients of the tile's increments
    __shared__ float dz_after[4];                    // gradient of the increment that follows the tile's last one

    const int t = threadIdx.x;
    const int wave = t >> 6;
    const int c1 = t >> 6, c2 = (t >> 4) & 3, c3 = (t >> 2) & 3, c4 = t & 3;
    const int u2 = t >> 4, u3 = t >> 2;   // ancestors at levels 2 and 3
    const int64_t b = blockIdx.x;
    const f4 zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
    const f4 *x4 = reinterpret_cast<const f4 *>(path) + b * L;
    const f4 x_base = bpv != nullptr ? reinterpret_cast<const f4 *>(bpv)[b] : zero4;
    const int64_t per_path = STREAM ? n_inc * int64_t(kS) : int64_t(kS);
    const float *sg = sig + b * per_path;
    const float *go = gout + b * per_path;
    float *gp = gpath + b * L * 4;

    // this thread's share of one flat element: levels 1..4 scalars, level 5 and 6 vectors
    struct Share {
        float l1, l2, l3, l4;
        f4 l5;
        f4 l6[4];
    };
    auto load_share = [&](const float *e, bool with_top) {
        Share s;
        s.l1 = e[kOff4[1] + c1];
        s.l2 = e[kOff4[2] + u2];
        s.l3 = e[kOff4[3] + u3];
        s.l4 = e[kOff4[4] + t];
        s.l5 = zero4;
#pragma unroll
        for (int c = 0; c < 4; ++c) s.l6[c] = zero4;
        if constexpr (N >= 5) s.l5 = *reinterpret_cast<const f4 *>(e + kOff4[5] + 4 * t);
        if constexpr (N >= 6) {
            if (with_top) {
#pragma unroll
                for (int c = 0; c < 4; ++c) s.l6[c] = *reinterpret_cast<const f4 *>(e + kOff4[6] + 16 * t + 4 * c);
            }
        }
        return s;
    };

    // G: cotangent of the signature after the increment being processed.  A: that signature (final mode).
    Share G = load_share(STREAM ? go + (n_inc - 1) * int64_t(kS) : go, true);
    Share A = {};
    Share nextA = {}, nextG = {};   // stream mode: signature before, and output gradient of, the step to come
    if constexpr (!STREAM) A = load_share(sg, false);

    if (t < 4) dz_after[t] = 0.0f;   // no increment follows the last one

    for (int64_t t0 = ((n_inc - 1) / kTileB) * kTileB; t0 >= 0; t0 -= kTileB) {
        const int nt = int(n_inc - t0 < kTileB ? n_inc - t0 : kTileB);
        __syncthreads();
        if (t < nt) {
            const int64_t s = t0 + t;
            const int64_t i_hi = basepoint ? s : s + 1;
            const f4 lo = i_hi > 0 ? x4[i_hi - 1] : x_base;
            *reinterpret_cast<f4 *>(zt + 4 * t) = x4[i_hi] - lo;
        }
        if constexpr (STREAM) {
            // entries for the first step of this tile (later ones are fetched one step ahead, below)
            const int64_t s = t0 + nt - 1;
            if (s > 0) {
                nextA = load_share(sg + (s - 1) * int64_t(kS), false);
                nextG = load_share(go + (s - 1) * int64_t(kS), true);
            } else {
                nextA = Share{};
            }
        }
        __syncthreads();

        for (int i = nt - 1; i >= 0; --i) {
            const int64_t s = t0 + i;
            const f4 z = *reinterpret_cast<const f4 *>(zt + 4 * i);
            const float z1 = zt[4 * i + c1], z2 = zt[4 * i + c2], z3 = zt[4 * i + c3], z4 = zt[4 * i + c4];

            Share addG = {};
            if constexpr (STREAM) {
                A = nextA;      // signature after s increments = entry s-1 (zero for s = 0)
                addG = nextG;   // output gradient of entry s-1, added to G once this step is done
                if (i > 0) {    // fetch for step s-1 (i-1 >= 0 in this tile); across tiles the code above does it
                    if (s - 1 > 0) {
                        nextA = load_share(sg + (s - 2) * int64_t(kS), false);
                        nextG = load_share(go + (s - 2) * int64_t(kS), true);
                    } else {
                        nextA = Share{};
                    }
                }
            }

            // ---- up: T[i][k] = T^(k)_i at this thread's word; a_i = the signature before the increment
            float T1[7], T2[7], T3[7], T4[7];
            f4 T5 = zero4;   // T^(6)_5[u c]
            const float a1 = STREAM ? A.l1 : A.l1 - z1;
#pragma unroll
            for (int k = 2; k <= N; ++k) T1[k] = __builtin_fmaf(z1, rk[k], a1);
            const float a2 = STREAM ? A.l2 : __builtin_fmaf(-T1[2], z2, A.l2);
#pragma unroll
            for (int k = 3; k <= N; ++k) T2[k] = __builtin_fmaf(T1[k], z2 * rk[k - 1], a2);
            const float a3 = STREAM ? A.l3 : __builtin_fmaf(-T2[3], z3, A.l3);
#pragma unroll
            for (int k = 4; k <= N; ++k) T3[k] = __builtin_fmaf(T2[k], z3 * rk[k - 2], a3);
            float a4 = 0.0f;
            f4 a5 = zero4;
            if constexpr (N >= 5) {
                a4 = STREAM ? A.l4 : __builtin_fmaf(-T3[4], z4, A.l4);
#pragma unroll
                for (int k = 5; k <= N; ++k) T4[k] = __builtin_fmaf(T3[k], z4 * rk[k - 3], a4);
            }
            if constexpr (N >= 6) {
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    a5[c] = STREAM ? A.l5[c] : __builtin_fmaf(-T4[5], z[c], A.l5[c]);
                    T5[c] = __builtin_fmaf(T4[6], z[c] * r2, a5[c]);
                }
            }
            if constexpr (!STREAM) {
                A.l1 = a1;
                A.l2 = a2;
                A.l3 = a3;
                A.l4 = a4;
                A.l5 = a5;
            }

            // ---- down
            f4 dz = zero4;               // contributions by letter
            float D5_4 = 0.0f, D6_4 = 0.0f;   // D^(5)_4[u], D^(6)_4[u]
            if constexpr (N >= 6) {
                f4 D6_5;                 // D^(6)_5[u c]
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    D6_5[c] = G.l6[c][0] * z[0] + G.l6[c][1] * z[1] + G.l6[c][2] * z[2] + G.l6[c][3] * z[3];
                    dz += T5[c] * G.l6[c];
                }
                // level 5: chains k = 5 (G.l5, divisor 1) and k = 6 (D6_5, divisor 2)
                dz += T4[5] * G.l5 + (T4[6] * r2) * D6_5;
                D5_4 = G.l5[0] * z[0] + G.l5[1] * z[1] + G.l5[2] * z[2] + G.l5[3] * z[3];
                D6_4 = (D6_5[0] * z[0] + D6_5[1] * z[1] + D6_5[2] * z[2] + D6_5[3] * z[3]) * r2;
                G.l5 += D6_5;
            } else if constexpr (N >= 5) {
                dz += T4[5] * G.l5;
                D5_4 = G.l5[0] * z[0] + G.l5[1] * z[1] + G.l5[2] * z[2] + G.l5[3] * z[3];
            }

            // level 4: chains k = 4 (G.l4), 5 (D5_4, divisor 2), 6 (D6_4, divisor 3)
            float contrib4 = T3[4] * G.l4;
            float E4 = G.l4 * z4, E5 = 0.0f, E6 = 0.0f;
            if constexpr (N >= 5) {
                contrib4 = __builtin_fmaf(T3[5] * r2, D5_4, contrib4);
                E5 = D5_4 * (z4 * r2);
                G.l4 += D5_4;
            }
            if constexpr (N >= 6) {
                contrib4 = __builtin_fmaf(T3[6] * r3, D6_4, contrib4);
                E6 = D6_4 * (z4 * r3);
                G.l4 += D6_4;
            }
            // level 3 (held by the 4 lanes of a quad): chains k = 3 (G.l3), 4, 5, 6 (divisors 2, 3, 4)
            const float D4_3 = quad_sum(E4);
            float D5_3 = 0.0f, D6_3 = 0.0f;
            float contrib3 = __builtin_fmaf(T2[4] * r2, D4_3, T2[3] * G.l3);
            float F3 = G.l3 * z3, F4 = D4_3 * (z3 * r2), F5 = 0.0f, F6 = 0.0f;
            float g3_add = D4_3;
            if constexpr (N >= 5) {
                D5_3 = quad_sum(E5);
                contrib3 = __builtin_fmaf(T2[5] * r3, D5_3, contrib3);
                F5 = D5_3 * (z3 * r3);
                g3_add += D5_3;
            }
            if constexpr (N >= 6) {
                D6_3 = quad_sum(E6);
                contrib3 = __builtin_fmaf(T2[6] * r4, D6_3, contrib3);
                F6 = D6_3 * (z3 * r4);
                g3_add += D6_3;
            }
            G.l3 += g3_add;
            // level 2 (held by the 16 lanes of a row): chains k = 2 (G.l2), 3..6 (divisors 2..5)
            const float D3_2 = row_sum_of_quads(F3), D4_2 = row_sum_of_quads(F4);
            float D5_2 = 0.0f, D6_2 = 0.0f;
            float contrib2 = __builtin_fmaf(T1[3] * r2, D3_2, T1[2] * G.l2);
            contrib2 = __builtin_fmaf(T1[4] * r3, D4_2, contrib2);
            float H2 = G.l2 * z2, H3 = D3_2 * (z2 * r2), H4 = D4_2 * (z2 * r3), H5 = 0.0f, H6 = 0.0f;
            float g2_add = D3_2 + D4_2;
            if constexpr (N >= 5) {
                D5_2 = row_sum_of_quads(F5);
                contrib2 = __builtin_fmaf(T1[5] * r4, D5_2, contrib2);
                H5 = D5_2 * (z2 * r4);
                g2_add += D5_2;
            }
            if constexpr (N >= 6) {
                D6_2 = row_sum_of_quads(F6);
                contrib2 = __builtin_fmaf(T1[6] * r5, D6_2, contrib2);
                H6 = D6_2 * (z2 * r5);
                g2_add += D6_2;
            }
            G.l2 += g2_add;
            // level 1 (held by the whole wavefront): chains k = 1 (G.l1), 2..6 (divisors 2..6); T^(k)_0 = 1
            const float D2_1 = wave_sum_of_rows(H2), D3_1 = wave_sum_of_rows(H3), D4_1 = wave_sum_of_rows(H4);
            float contrib1 = G.l1 + r2 * D2_1 + r3 * D3_1 + r4 * D4_1;
            float g1_add = D2_1 + D3_1 + D4_1;
            if constexpr (N >= 5) {
                const float D5_1 = wave_sum_of_rows(H5);
                contrib1 = __builtin_fmaf(r5, D5_1, contrib1);
                g1_add += D5_1;
            }
            if constexpr (N >= 6) {
                const float D6_1 = wave_sum_of_rows(H6);
                contrib1 = __builtin_fmaf(r6, D6_1, contrib1);
                g1_add += D6_1;
            }
            G.l1 += g1_add;

            // ---- the increment's gradient: every thread adds its contributions under their letters, redundant
            // holders weighed down; then the sum over the workgroup
            contrib3 *= 0.25f;
            contrib2 *= 0.0625f;
            contrib1 *= 0.015625f;
#pragma unroll
            for (int c = 0; c < 4; ++c)
                dz[c] += (c4 == c ? contrib4 : 0.0f) + (c3 == c ? contrib3 : 0.0f) + (c2 == c ? contrib2 : 0.0f) +
                         (c1 == c ? contrib1 : 0.0f);
            // lane q of every quad takes letter q: transpose the quad's 4x4 values, add the four rows
            const f4 tr = quad_transpose(dz, t & 63);
            float mine = (tr[0] + tr[1]) + (tr[2] + tr[3]);
            mine = wave_sum_of_rows(row_sum_of_quads(mine));   // over the 16 quads: lanes 0..3 hold letters 0..3
            // the four wavefronts never wait for one another inside a tile: each leaves its partial sums in LDS
            if ((t & 63) < 4) part[i][wave][t & 3] = mine;

            if constexpr (STREAM) {
                if (s > 0) {
                    G.l1 += addG.l1;
                    G.l2 += addG.l2;
                    G.l3 += addG.l3;
                    G.l4 += addG.l4;
                    G.l5 += addG.l5;
#pragma unroll
                    for (int c = 0; c < 4; ++c) G.l6[c] += addG.l6[c];
                }
            }
        }

        // the tile's gradients: sum over the wavefronts, then every point of the tile gets the gradient of the
        // increment it ends minus that of the increment it starts
        __syncthreads();
        if (t < nt * 4) {
            const int i = t >> 2, c = t & 3;
            dzs[i][c] = (part[i][0][c] + part[i][1][c]) + (part[i][2][c] + part[i][3][c]);
        }
        __syncthreads();
        float first = 0.0f;
        if (t < nt * 4) {
            const int i = t >> 2, c = t & 3;
            const int64_t point = (basepoint ? t0 : t0 + 1) + i;
            gp[point * 4 + c] = dzs[i][c] - (i + 1 < nt ? dzs[i + 1][c] : dz_after[c]);
            if (i == 0) first = dzs[0][c];
        }
        __syncthreads();
        if (t < 4) dz_after[t] = first;   // this tile's first increment follows the last one of the tile before it
    }
    __syncthreads();
    if (t < 4) {
        // dz_after now holds the gradient of increment 0
        if (!basepoint) gp[t] = -dz_after[t];                             // the first point only starts increment 0
        else if (gbase != nullptr) gbase[b * 4 + t] = -dz_after[t];       // and so does a basepoint
    }
}

template <int N>
hipError_t launch_d4(const Shape &sh, const float *path, const float *sig, const float *gout, float *gpath, float *gbase,
                     hipStream_t st)
{
    const dim3 grid(static_cast<unsigned>(sh.B)), block(256);
    const float *bpv = static_cast<const float *>(sh.basepoint_value);
    if (sh.stream)
        hipLaunchKernelGGL((sig_backward_d4_kernel<N, true>), grid, block, 0, st, path, sig, gout, gpath, gbase, sh.L,
                           sh.n_inc, sh.basepoint, bpv);
    else
        hipLaunchKernelGGL((sig_backward_d4_kernel<N, false>), grid, block, 0, st, path, sig, gout, gpath, gbase, sh.L,
                           sh.n_inc, sh.basepoint, bpv);
    return hipGetLastError();
}

}  // namespace

bool backward_d4_supported(const Shape &sh) { return sh.d == 4 && sh.N >= 4 && sh.N <= 6 && sh.B <= 0x7fffffff; }

hipError_t launch_backward_d4_f32(const Shape &sh, const float *path, const float *sig, const float *gout, float *gpath,
                                  float *gbase, hipStream_t st)
{
    if (!backward_d4_supported(sh)) return hipErrorNotSupported;
    switch (sh.N) {
        case 4: return launch_d4<4>(sh, path, sig, gout, gpath, gbase, st);
        case 5: return launch_d4<5>(sh, path, sig, gout, gpath, gbase, st);
        default: return launch_d4<6>(sh, path, sig, gout, gpath, gbase, st);
    }
}

}  // namespace sig
