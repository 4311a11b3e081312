// Gradient of the signature with respect to the path for d = 16 channels at depth N = 4, final mode, fp32
// (paper section 5.3, appendix C; the recurrences are those of sig_backward.hip).
//
// Almost all of the work of a backward step at this shape sits at the top level: with G_4 the cotangent of the top
// level (it never changes in final mode) and T = T^(4)_3 the last Horner term of eq. "fusedterm",
//     D^(4)_3[w] = sum_j G_4[w j] z[j]            (cotangent handed down to the three-letter word w)
//     gz[j]     += sum_w T[w] G_4[w j]            (the increment's gradient)
// are two matrix-vector products with the same 4096 x 16 matrix, 2 x 65 536 multiply-adds per increment against
// about 30 000 for everything below.  So G_4 stays in registers for the whole scan: one workgroup of 512 threads per
// path, thread (w_1, w_2, h) owns the eight words w_1 w_2 w_3 with w_3 = 8h .. 8h+7: their rows of G_4 (128
// registers), A_3 and G_3.  The first product is then local to a thread.  The second one leaves every thread with 16
// partial sums per increment; they are summed over the 16 lanes of a row by a transposing butterfly (15 lane
// exchanges instead of 64: at every stage a lane keeps half of its channels and receives its partner's sums of
// those), then over rows and wavefronts through LDS, once per tile of increments.
//
// Above its own words a thread follows the scheme of the prefix-tree gradient kernels: it carries its own copy of the
// signature at the prefixes w_1 and w_1 w_2 (the "up" pass undoes the increment exactly as every other thread below
// that prefix does), and of the cotangent of a prefix only the part that arrived through its own words; the map from
// cotangents to the gradient is linear, so only the increments' gradients are ever summed.
//
// The per-increment gradients go to a workspace [B][n_inc][16]; the closing kernel of the prefix-tree family turns
// them into point gradients (a point ends one increment and starts the next).
#include "sig_tree_backward_impl.h"

namespace sig {
namespace {

constexpr int kD16 = 16;
constexpr int kOff2 = 16, kOff3 = 16 + 256, kOff4 = 16 + 256 + 4096, kS16 = 16 + 256 + 4096 + 65536;
constexpr int kBwTile = 16;       // increments per tile
constexpr int kBwThreads = 512;

typedef float f4 __attribute__((ext_vector_type(4)));

template <int CTRL>
__device__ __forceinline__ float lane_move(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}

// One stage of the transposing butterfly: v holds 2*HALF sums; a lane whose `upper` flag is set keeps the upper HALF
// of them, the others the lower HALF, and each receives from its partner (CTRL pairs lanes with opposite flags) the
// partner's sums of the channels it keeps.
template <int HALF, int CTRL>
__device__ __forceinline__ void butterfly_stage(float *v, bool upper)
{
#pragma unroll
    for (int c = 0; c < HALF; ++c) {
        const float keep = upper ? v[c + HALF] : v[c];
        const float send = upper ? v[c] : v[c + HALF];
        v[c] = keep + lane_move<CTRL>(send);
    }
}

__global__ void __launch_bounds__(kBwThreads)
sig_backward_d16_n4_kernel(const float *__restrict__ path, const float *__restrict__ sig, const float *__restrict__ gout,
                           float *__restrict__ gz, int64_t L, int64_t n_inc, int basepoint, const float *__restrict__ bpv)
{
    __shared__ __align__(16) float zt[kBwTile * kD16];           // increments of the tile
    __shared__ float part[kBwTile * kBwThreads];                 // [increment][wavefront][row][channel]

    const int tid = threadIdx.x, lane = tid & 63;
    const int h = __builtin_amdgcn_readfirstlane(tid >> 8);      // which half of the third letters (wave-uniform)
    const int w1 = (tid >> 4) & 15, w2 = tid & 15;
    const int l16 = lane & 15;
    const int64_t b = blockIdx.x;
    const float *x = path + b * L * kD16;
    const float *sg = sig + b * kS16;
    const float *go = gout + b * kS16;
    const int p2 = w1 * 16 + w2;            // the prefix w_1 w_2 inside level 2
    const int u0 = p2 * 16 + 8 * h;         // the first of this thread's words inside level 3

    // cotangents: the rows of G_4 of the thread's eight words, G_3 at those words, and the thread's part of the
    // cotangents of its prefixes (what the output gradient holds there goes to the first thread below the prefix)
    float M[8][kD16];
#pragma unroll
    for (int cc = 0; cc < 8; ++cc) {
        const f4 *row = reinterpret_cast<const f4 *>(go + kOff4 + (u0 + cc) * kD16);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f4 v = row[q];
            M[cc][4 * q] = v[0];
            M[cc][4 * q + 1] = v[1];
            M[cc][4 * q + 2] = v[2];
            M[cc][4 * q + 3] = v[3];
        }
    }
    float g3[8], a3[8];
#pragma unroll
    for (int cc = 0; cc < 8; ++cc) {
        g3[cc] = go[kOff3 + u0 + cc];
        a3[cc] = sg[kOff3 + u0 + cc];
    }
    float g2 = h == 0 ? go[kOff2 + p2] : 0.0f;
    float g1 = (h == 0 && w2 == 0) ? go[w1] : 0.0f;
    float a2 = sg[kOff2 + p2], a1 = sg[w1];

    for (int64_t t0 = ((n_inc - 1) / kBwTile) * kBwTile; t0 >= 0; t0 -= kBwTile) {
        const int nt = int(n_inc - t0 < kBwTile ? n_inc - t0 : kBwTile);
        __syncthreads();   // the sums of the previous tile have been read, its increments are no longer needed
        if (tid < kBwTile * kD16) {
            const int i = tid >> 4, c = tid & 15;
            float z = 0.0f;
            if (i < nt) {
                const int64_t i_hi = t0 + i + (basepoint ? 0 : 1);
                const float lo = i_hi > 0 ? x[(i_hi - 1) * kD16 + c] : bpv != nullptr ? bpv[b * kD16 + c] : 0.0f;
                z = x[i_hi * kD16 + c] - lo;
            }
            zt[tid] = z;
        }
        __syncthreads();

        for (int i = nt - 1; i >= 0; --i) {
            const float *zrow = zt + i * kD16;
            float z[kD16];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f4 v = *reinterpret_cast<const f4 *>(zrow + 4 * q);
                z[4 * q] = v[0];
                z[4 * q + 1] = v[1];
                z[4 * q + 2] = v[2];
                z[4 * q + 3] = v[3];
            }
            const float z1 = zrow[w1], z2 = zrow[w2];
            float z3[8];
#pragma unroll
            for (int cc = 0; cc < 8; ++cc) z3[cc] = h ? z[8 + cc] : z[cc];

            // ---- up: the signature before the increment and the Horner terms T^(k)_i along the thread's words
            a1 -= z1;
            const float t2_1 = __builtin_fmaf(z1, 1.0f / 2, a1);
            const float t3_1 = __builtin_fmaf(z1, 1.0f / 3, a1);
            const float t4_1 = __builtin_fmaf(z1, 1.0f / 4, a1);
            a2 = __builtin_fmaf(-t2_1, z2, a2);
            const float t3_2 = __builtin_fmaf(t3_1, z2 * (1.0f / 2), a2);
            const float t4_2 = __builtin_fmaf(t4_1, z2 * (1.0f / 3), a2);
            float t4_3[8];
#pragma unroll
            for (int cc = 0; cc < 8; ++cc) {
                a3[cc] = __builtin_fmaf(-t3_2, z3[cc], a3[cc]);
                t4_3[cc] = __builtin_fmaf(t4_2, z3[cc] * (1.0f / 2), a3[cc]);
            }

            // ---- down, level 4: the two products with G_4
            float dz[kD16];
#pragma unroll
            for (int j = 0; j < kD16; ++j) dz[j] = 0.0f;
            float d4_3[8];
#pragma unroll
            for (int cc = 0; cc < 8; ++cc) {
                float acc = 0.0f;
#pragma unroll
                for (int j = 0; j < kD16; ++j) {
                    acc = __builtin_fmaf(M[cc][j], z[j], acc);
                    dz[j] = __builtin_fmaf(t4_3[cc], M[cc][j], dz[j]);
                }
                d4_3[cc] = acc;
            }
            // ---- down, the chains below: this thread's parts only
            float e3[8];                 // to the channels 8h .. 8h+7 (the third letters)
            float d4_2 = 0.0f, d3_2 = 0.0f;
#pragma unroll
            for (int cc = 0; cc < 8; ++cc) {
                d4_2 = __builtin_fmaf(d4_3[cc], z3[cc], d4_2);
                d3_2 = __builtin_fmaf(g3[cc], z3[cc], d3_2);
                e3[cc] = __builtin_fmaf(g3[cc], t3_2, d4_3[cc] * (t4_2 * (1.0f / 2)));
                g3[cc] += d4_3[cc];
            }
            d4_2 *= 1.0f / 2;
            const float d4_1 = d4_2 * (z2 * (1.0f / 3)), d3_1 = d3_2 * (z2 * (1.0f / 2)), d2_1 = g2 * z2;
            // to the channel w_2, and to the channel w_1
            const float e2 = __builtin_fmaf(d4_2, t4_1 * (1.0f / 3), __builtin_fmaf(d3_2, t3_1 * (1.0f / 2), g2 * t2_1));
            const float e1 = __builtin_fmaf(d4_1, 1.0f / 4, __builtin_fmaf(d3_1, 1.0f / 3, __builtin_fmaf(d2_1, 1.0f / 2, g1)));
            g2 += d4_2 + d3_2;
            g1 += d4_1 + d3_1 + d2_1;
            if (h) {
#pragma unroll
                for (int cc = 0; cc < 8; ++cc) dz[8 + cc] += e3[cc];
            } else {
#pragma unroll
                for (int cc = 0; cc < 8; ++cc) dz[cc] += e3[cc];
            }

            // ---- sums over the 16 lanes of a row: afterwards lane r of a row holds channel r
            butterfly_stage<8, 0x140>(dz, (l16 & 8) != 0);   // row_mirror
            butterfly_stage<4, 0x141>(dz, (l16 & 4) != 0);   // row_half_mirror
            butterfly_stage<2, 0x4E>(dz, (l16 & 2) != 0);    // quad_perm [2,3,0,1]
            butterfly_stage<1, 0xB1>(dz, (l16 & 1) != 0);    // quad_perm [1,0,3,2]
            // w_2 is the lane's place in its row, so e2 joins the channel the lane now holds; the row's sum of e1
            // belongs to channel w_1, the same for the whole row
            const float row_e1 = group_sum<0, 4, float>(e1);
            part[i * kBwThreads + tid] = dz[0] + e2 + (l16 == w1 ? row_e1 : 0.0f);
        }
        __syncthreads();
        if (tid < kBwTile * kD16) {
            const int i = tid >> 4, c = tid & 15;
            if (i < nt) {
                float total = 0.0f;
#pragma unroll 8
                for (int r = 0; r < kBwThreads / 16; ++r) total += part[i * kBwThreads + r * 16 + c];
                gz[(b * n_inc + t0 + i) * kD16 + c] = total;
            }
        }
    }
}

}  // namespace

bool backward_d16_supported(const Shape &sh)
{
    return sh.d == 16 && sh.N == 4 && !sh.stream && sh.chunks <= 1 && sh.B <= 0x7fffffff;
}

int64_t backward_d16_workspace_bytes(const Shape &sh) { return sh.B * sh.n_inc * kD16 * int64_t(sizeof(float)); }

hipError_t launch_backward_d16_f32(const Shape &sh, const float *path, const float *sig, const float *gout, float *gpath,
                                   float *gbase, void *workspace, int64_t workspace_bytes, hipStream_t st)
{
    if (!backward_d16_supported(sh)) return hipErrorNotSupported;
    if (workspace == nullptr || workspace_bytes < backward_d16_workspace_bytes(sh)) return hipErrorInvalidValue;
    float *gz = static_cast<float *>(workspace);
    hipLaunchKernelGGL(sig_backward_d16_n4_kernel, dim3(unsigned(sh.B)), dim3(kBwThreads), 0, st, path, sig, gout, gz, sh.L,
                       sh.n_inc, sh.basepoint, static_cast<const float *>(sh.basepoint_value));
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    const int64_t total = sh.B * (sh.n_inc + 1) * kD16;
    const unsigned grid = unsigned((total + 255) / 256 < 65536 ? (total + 255) / 256 : 65536);
    hipLaunchKernelGGL((sig_tree_backward_reduce_kernel<float, kD16>), dim3(grid), dim3(256), 0, st, sh, int64_t(1), gz, gpath,
                       gbase);
    return hipGetLastError();
}

}  // namespace sig
