// Gradient of the signature with respect to the path for d = 4 channels at depth N = 6, final mode, fp32
// (paper section 5.3, appendix C; the recurrences are those of sig_backward.hip).
//
// The scheme of sig_backward_d16.hip at the benchmark shape of the forward pass: the cotangent of the top level never
// changes in final mode, so it stays in registers for the whole scan, and a thread owns a subtree deep enough that
// most of its work is the two products with that cotangent.  One workgroup of two wavefronts per path; lane
// u = w_1 w_2 w_3 of wavefront h owns the words u c_4 with c_4 = 2h, 2h+1, the 8 words u c_4 c_5 and the 32 words
// u c_4 c_5 c_6 below them: G_6 (32 registers), G_5, G_4, A_5, A_4.  Above its words a thread carries its own copy of the
// signature at the prefixes w_1, w_1 w_2, u and, of the cotangents there, only the part that arrived through its own
// words (the map from cotangents to the gradient is linear, so only the increments' gradients are ever summed).
//
// An increment's gradient has four channels.  A thread's subtree contributes to all of them (the letters c_5, c_6), to
// channel c_4 (two of them, known per wavefront) and, through its prefixes, to the channels w_3, w_2, w_1 of its own
// word.  They meet as follows: a transposing butterfly over the lane quad leaves lane w_3 with the quad's sum of
// channel w_3; its own w_3 term joins as it stands; the quad's sums of the w_2 and w_1 terms join in the lane whose
// w_3 equals that letter; two row rotations sum the four quads of a row; rows and wavefronts meet in LDS once per tile.
#include "sig_tree_backward_impl.h"

namespace sig {
namespace {

constexpr int kOffD4[8] = {0, 0, 4, 20, 84, 340, 1364, 5460};   // offset of level k (1-based); [7] = S(4, 6)
constexpr int kS46 = 5460;
constexpr int kG4Tile = 32;      // increments per tile
constexpr int kG4Threads = 128;

typedef float f4 __attribute__((ext_vector_type(4)));

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}

__global__ void __launch_bounds__(kG4Threads)
sig_backward_d4_n6_kernel(const float *__restrict__ path, const float *__restrict__ sig, const float *__restrict__ gout,
                          float *__restrict__ gz, int64_t L, int64_t n_inc, int basepoint, const float *__restrict__ bpv)
{
    __shared__ __align__(16) float zt[kG4Tile * 4];                 // increments of the tile
    __shared__ float part[kG4Tile * 2 * 4 * 4];                     // [increment][wavefront][row][channel]

    const int tid = threadIdx.x, lane = tid & 63;
    const int h = __builtin_amdgcn_readfirstlane(tid >> 6);         // wavefront: fourth letters 2h, 2h + 1
    const int w1 = lane >> 4, w2 = (lane >> 2) & 3, w3 = lane & 3;
    const int64_t b = blockIdx.x;
    const f4 *x4 = reinterpret_cast<const f4 *>(path) + b * L;
    const float *sg = sig + b * kS46;
    const float *go = gout + b * kS46;
    const int p1 = w1, p2 = w1 * 4 + w2, p3 = lane;                 // the prefixes inside levels 1, 2, 3
    const int u4 = p3 * 4 + 2 * h;                                  // the first of the thread's words inside level 4

    // cotangents: whole for the thread's own words; at a prefix, the output gradient goes to the first thread below it
    float G6[2][4][4], G5[2][4], G4[2], a5[2][4], a4[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        G4[i] = go[kOffD4[4] + u4 + i];
        a4[i] = sg[kOffD4[4] + u4 + i];
        const f4 g5 = *reinterpret_cast<const f4 *>(go + kOffD4[5] + (u4 + i) * 4);
        const f4 s5 = *reinterpret_cast<const f4 *>(sg + kOffD4[5] + (u4 + i) * 4);
#pragma unroll
        for (int c5 = 0; c5 < 4; ++c5) {
            G5[i][c5] = g5[c5];
            a5[i][c5] = s5[c5];
            const f4 g6 = *reinterpret_cast<const f4 *>(go + kOffD4[6] + ((u4 + i) * 4 + c5) * 4);
#pragma unroll
            for (int c6 = 0; c6 < 4; ++c6) G6[i][c5][c6] = g6[c6];
        }
    }
    float g3 = h == 0 ? go[kOffD4[3] + p3] : 0.0f;
    float g2 = (h == 0 && w3 == 0) ? go[kOffD4[2] + p2] : 0.0f;
    float g1 = (h == 0 && w3 == 0 && w2 == 0) ? go[p1] : 0.0f;
    float a3 = sg[kOffD4[3] + p3], a2 = sg[kOffD4[2] + p2], a1 = sg[p1];

    for (int64_t t0 = ((n_inc - 1) / kG4Tile) * kG4Tile; t0 >= 0; t0 -= kG4Tile) {
        const int nt = int(n_inc - t0 < kG4Tile ? n_inc - t0 : kG4Tile);
        __syncthreads();   // the sums of the previous tile have been read, its increments are no longer needed
        if (tid < kG4Tile) {
            f4 z = {0.0f, 0.0f, 0.0f, 0.0f};
            if (tid < nt) {
                const int64_t i_hi = t0 + tid + (basepoint ? 0 : 1);
                const f4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
                const f4 lo = i_hi > 0 ? x4[i_hi - 1] : bpv != nullptr ? reinterpret_cast<const f4 *>(bpv)[b] : zero;
                z = x4[i_hi] - lo;
            }
            *reinterpret_cast<f4 *>(zt + tid * 4) = z;
        }
        __syncthreads();

        for (int i = nt - 1; i >= 0; --i) {
            const f4 zv = *reinterpret_cast<const f4 *>(zt + i * 4);
            const float z[4] = {zv[0], zv[1], zv[2], zv[3]};
            const float z1 = zt[i * 4 + w1], z2 = zt[i * 4 + w2], z3 = zt[i * 4 + w3];
            const float zc[2] = {h ? z[2] : z[0], h ? z[3] : z[1]};

            // ---- up: the signature before the increment and the Horner terms T^(k)_j along the thread's words
            a1 -= z1;
            float t1[7], t2[7], t3[7];   // t1[k] = T^(k)_1 at w_1, t2[k] = T^(k)_2 at w_1 w_2, t3[k] = T^(k)_3 at u
#pragma unroll
            for (int k = 2; k <= 6; ++k) t1[k] = __builtin_fmaf(z1, 1.0f / k, a1);
            a2 = __builtin_fmaf(-t1[2], z2, a2);
#pragma unroll
            for (int k = 3; k <= 6; ++k) t2[k] = __builtin_fmaf(t1[k], z2 * (1.0f / (k - 1)), a2);
            a3 = __builtin_fmaf(-t2[3], z3, a3);
#pragma unroll
            for (int k = 4; k <= 6; ++k) t3[k] = __builtin_fmaf(t2[k], z3 * (1.0f / (k - 2)), a3);
            float t5_4[2], t6_4[2], t6_5[2][4];
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                a4[c] = __builtin_fmaf(-t3[4], zc[c], a4[c]);
                t5_4[c] = __builtin_fmaf(t3[5], zc[c] * (1.0f / 2), a4[c]);
                t6_4[c] = __builtin_fmaf(t3[6], zc[c] * (1.0f / 3), a4[c]);
#pragma unroll
                for (int c5 = 0; c5 < 4; ++c5) {
                    a5[c][c5] = __builtin_fmaf(-t5_4[c], z[c5], a5[c][c5]);
                    t6_5[c][c5] = __builtin_fmaf(t6_4[c], z[c5] * (1.0f / 2), a5[c][c5]);
                }
            }

            // ---- down through the thread's own words: levels 6, 5, 4
            float dz[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            float e4[2];                    // to the channels 2h, 2h + 1
            float d4_3 = 0.0f, d5_3 = 0.0f, d6_3 = 0.0f;   // this thread's parts of D^(k)_3 at u
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                float d5_4 = 0.0f, d6_4 = 0.0f;
#pragma unroll
                for (int c5 = 0; c5 < 4; ++c5) {
                    float d6_5 = 0.0f;
#pragma unroll
                    for (int c6 = 0; c6 < 4; ++c6) {
                        d6_5 = __builtin_fmaf(G6[c][c5][c6], z[c6], d6_5);
                        dz[c6] = __builtin_fmaf(t6_5[c][c5], G6[c][c5][c6], dz[c6]);
                    }
                    d5_4 = __builtin_fmaf(G5[c][c5], z[c5], d5_4);
                    d6_4 = __builtin_fmaf(d6_5, z[c5], d6_4);
                    dz[c5] = __builtin_fmaf(t5_4[c], G5[c][c5], __builtin_fmaf(d6_5, t6_4[c] * (1.0f / 2), dz[c5]));
                    G5[c][c5] += d6_5;
                }
                d6_4 *= 1.0f / 2;
                e4[c] = __builtin_fmaf(G4[c], t3[4], __builtin_fmaf(d5_4, t3[5] * (1.0f / 2), d6_4 * (t3[6] * (1.0f / 3))));
                d4_3 = __builtin_fmaf(G4[c], zc[c], d4_3);
                d5_3 = __builtin_fmaf(d5_4, zc[c], d5_3);
                d6_3 = __builtin_fmaf(d6_4, zc[c], d6_3);
                G4[c] += d5_4 + d6_4;
            }
            d5_3 *= 1.0f / 2;
            d6_3 *= 1.0f / 3;
            if (h) {
                dz[2] += e4[0];
                dz[3] += e4[1];
            } else {
                dz[0] += e4[0];
                dz[1] += e4[1];
            }
            // ---- down along the prefixes: this thread's parts only
            // level 3 (letter w_3)
            const float e3 = __builtin_fmaf(g3, t2[3], __builtin_fmaf(d4_3, t2[4] * (1.0f / 2),
                                            __builtin_fmaf(d5_3, t2[5] * (1.0f / 3), d6_3 * (t2[6] * (1.0f / 4)))));
            const float d3_2 = g3 * z3, d4_2 = d4_3 * (z3 * (1.0f / 2)), d5_2 = d5_3 * (z3 * (1.0f / 3)),
                        d6_2 = d6_3 * (z3 * (1.0f / 4));
            g3 += d4_3 + d5_3 + d6_3;
            // level 2 (letter w_2)
            const float e2 = __builtin_fmaf(g2, t1[2], __builtin_fmaf(d3_2, t1[3] * (1.0f / 2),
                                            __builtin_fmaf(d4_2, t1[4] * (1.0f / 3),
                                            __builtin_fmaf(d5_2, t1[5] * (1.0f / 4), d6_2 * (t1[6] * (1.0f / 5))))));
            const float d2_1 = g2 * z2, d3_1 = d3_2 * (z2 * (1.0f / 2)), d4_1 = d4_2 * (z2 * (1.0f / 3)),
                        d5_1 = d5_2 * (z2 * (1.0f / 4)), d6_1 = d6_2 * (z2 * (1.0f / 5));
            g2 += d3_2 + d4_2 + d5_2 + d6_2;
            // level 1 (letter w_1)
            const float e1 = g1 + d2_1 * (1.0f / 2) + d3_1 * (1.0f / 3) + d4_1 * (1.0f / 4) + d5_1 * (1.0f / 5) + d6_1 * (1.0f / 6);
            g1 += d2_1 + d3_1 + d4_1 + d5_1 + d6_1;

            // ---- the quad: lane w_3 ends up with the quad's sum of channel w_3
            const bool up2 = (lane & 2) != 0, up1 = (lane & 1) != 0;
            float k0 = up2 ? dz[2] : dz[0], k1 = up2 ? dz[3] : dz[1];
            const float s0 = up2 ? dz[0] : dz[2], s1 = up2 ? dz[1] : dz[3];
            k0 += dpp_move<0x4E>(s0);   // quad_perm [2,3,0,1]
            k1 += dpp_move<0x4E>(s1);
            float r = (up1 ? k1 : k0) + dpp_move<0xB1>(up1 ? k0 : k1);   // quad_perm [1,0,3,2]
            float q2 = e2 + dpp_move<0xB1>(e2), q1 = e1 + dpp_move<0xB1>(e1);
            q2 += dpp_move<0x4E>(q2);
            q1 += dpp_move<0x4E>(q1);
            r += e3 + (w3 == w2 ? q2 : 0.0f) + (w3 == w1 ? q1 : 0.0f);
            // ---- the four quads of a row
            r += dpp_move<0x124>(r);    // row_ror:4
            r += dpp_move<0x128>(r);    // row_ror:8
            if ((lane & 12) == 0) part[((i * 2 + h) * 4 + w1) * 4 + w3] = r;
        }
        __syncthreads();
        if (tid < kG4Tile * 4) {
            const int i = tid >> 2, c = tid & 3;
            if (i < nt) {
                float total = 0.0f;
#pragma unroll
                for (int r = 0; r < 8; ++r) total += part[(i * 8 + r) * 4 + c];
                gz[(b * n_inc + t0 + i) * 4 + c] = total;
            }
        }
    }
}

}  // namespace

bool backward_d4n6_supported(const Shape &sh)
{
    return sh.d == 4 && sh.N == 6 && !sh.stream && sh.chunks <= 1 && sh.B <= 0x7fffffff;
}

int64_t backward_d4n6_workspace_bytes(const Shape &sh) { return sh.B * sh.n_inc * 4 * int64_t(sizeof(float)); }

hipError_t launch_backward_d4n6_f32(const Shape &sh, const float *path, const float *sig, const float *gout, float *gpath,
                                    float *gbase, void *workspace, int64_t workspace_bytes, hipStream_t st)
{
    if (!backward_d4n6_supported(sh)) return hipErrorNotSupported;
    if (workspace == nullptr || workspace_bytes < backward_d4n6_workspace_bytes(sh)) return hipErrorInvalidValue;
    float *gz = static_cast<float *>(workspace);
    hipLaunchKernelGGL(sig_backward_d4_n6_kernel, dim3(unsigned(sh.B)), dim3(kG4Threads), 0, st, path, sig, gout, gz, sh.L,
                       sh.n_inc, sh.basepoint, static_cast<const float *>(sh.basepoint_value));
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    const int64_t total = sh.B * (sh.n_inc + 1) * 4;
    const unsigned grid = unsigned((total + 255) / 256 < 65536 ? (total + 255) / 256 : 65536);
    hipLaunchKernelGGL((sig_tree_backward_reduce_kernel<float, 4>), dim3(grid), dim3(256), 0, st, sh, int64_t(1), gz, gpath,
                       gbase);
    return hipGetLastError();
}

}  // namespace sig
