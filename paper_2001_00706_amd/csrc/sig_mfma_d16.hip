// Matrix-core kernel (fp32) for d = 16 channels, depth N = 4, final mode.
//
// One workgroup of 8 wavefronts scans one path; the 70 k-scalar state lives in the registers of
// the compute unit (two wavefronts per SIMD).  Each Horner stage of the fused multiply-exponentiate
// (paper section 4.1, eq. "fusedterm") is a batch of 16x16 outer products plus an addend, i.e.
// v_mfma_f32_16x16x1_4b_f32: 4 independent blocks of D[i][j] = a[i]*b[j] + C[i][j].
// Operand layout of that instruction (lane = 16*hi + lo):
//     a[i] of block b:   lane hi = b, lo = i          b[j] of block b:   lane hi = b, lo = j
//     D[i][j] of block b: register 4*b + i%4, lane hi = i/4, lo = j
// so the result of a level-k stage, taken register by register, is the left operand of level k+1:
// a result register's lanes carry (w_{k-1}/4, w_k), which is exactly (block, i) of the next stage.
//
// Work split (no communication between wavefronts): the words starting with a given first letter,
// plus that letter itself, are closed under the update, so wavefront v owns the two first letters
//     w_1 in { 4*(2h) + y, 4*(2h+1) + y },   y = v % 4, h = v / 4.
// Per increment a wavefront issues 9 matrix instructions:
//   * one for level 3, whose 4 blocks are [k=4 | k=4 | k=3 | k=3] for its two first letters: blocks
//     0,1 give the Horner term T_4^(3) (left operand of the level-4 update), blocks 2,3 the new A_3;
//   * eight for level 4: group (c, e) holds the words with w_1 = e-th owned letter and w_2 % 4 = c;
//     inside a group, register (w_2/4, w_3%4), lane (w_3/4, w_4).
// Levels 1 and 2 are a handful of vector FMAs, one scalar per lane: lane (b, x) carries the first
// letter of block b and the letter x.
#include "sig_internal.h"
#include "sig_mfma_common.h"

namespace sig {
namespace {

typedef float f16v __attribute__((ext_vector_type(16)));

constexpr int kD = 16;
constexpr int kOff2 = 16, kOff3 = 16 + 256, kOff4 = 16 + 256 + 4096, kS16 = 16 + 256 + 4096 + 65536;
constexpr int kRow16 = 3 * kD;   // floats per staged increment: z, z/2, z/3
constexpr int kTile16 = 128;     // increments staged in LDS at a time

__device__ __forceinline__ f16v outer16(float a, float b, f16v c)
{
    return __builtin_amdgcn_mfma_f32_16x16x1f32(a, b, c, 0, 0, 0);
}

// This lane's view of one staged increment.
struct Row16 {
    float zw, zx, zB, zC;   // z[w1], z[x], z[x]/(k-1), z[x]/(k-2) for this lane's block target k
};

__device__ __forceinline__ Row16 load_row16(const float *tab, int w1, int x, int off_zB, int off_zC)
{
    Row16 r;
    r.zw = tab[w1];
    r.zx = tab[x];
    r.zB = tab[off_zB];
    r.zC = tab[off_zC];
    return r;
}

// Folds one increment into levels 1..3 (result in `cur`) and the previous increment's pending
// T_4^(3) (in `prev`, with its z[x] in `pzx`) into level 4.
__device__ __forceinline__ void half_trip(float &A1, float &A2, f16v (&A4)[8], const f16v &prev, f16v &cur, float &pzx,
                                          const Row16 &r, float inv_k)
{
    // level 1 and 2 terms of this block's target level k, then the level-2 update itself
    const float t1 = __builtin_fmaf(r.zw, inv_k, A1);        // z[w1]/k + A_1[w1]
    const float t2 = __builtin_fmaf(t1, r.zB, A2);           // T_k^(2)[w1, x]
    const float u1 = __builtin_fmaf(r.zw, 0.5f, A1);         // target level 2
    A2 = __builtin_fmaf(u1, r.zx, A2);
    A1 += r.zw;

    // level 3: blocks 0,1 -> T_4^(3) = T_4^(2) (x) z/2 + A_3 ; blocks 2,3 -> A_3 <- T_3^(2) (x) z + A_3
    f16v C3;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        C3[i] = prev[8 + i];
        C3[8 + i] = prev[8 + i];
    }
    cur = outer16(t2, r.zC, C3);
    __builtin_amdgcn_sched_barrier(0);

    // level 4 of the previous increment: A_4 += T_4^(3) (x) z
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int ee = 0; ee < 2; ++ee) A4[2 * c + ee] = outer16(prev[4 * ee + c], pzx, A4[2 * c + ee]);
    pzx = r.zx;
    __builtin_amdgcn_sched_barrier(0);
}

__global__ void __launch_bounds__(512)
sig_mfma_d16_n4_kernel(const float *__restrict__ path, float *__restrict__ out, int64_t L, int64_t n_inc_total, int basepoint,
                       const float *__restrict__ bpv, int chunks, int64_t chunk_len)
{
    __shared__ __align__(16) float lds[kTile16 * kRow16];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int y = wave & 3, h = wave >> 2;
    const int b = lane >> 4, x = lane & 15;       // block and low index of this lane
    const int e = b & 1;                          // which of the two owned first letters this block serves
    const int w1 = 4 * (2 * h + e) + y;           // that first letter
    const bool k4 = b < 2;                        // blocks 0,1 serve target level 4, blocks 2,3 level 3
    const int64_t path_no = blockIdx.x;   // output row: a path, or one chunk of a path
    const ChunkView cv = chunk_view(path_no, chunks, chunk_len, n_inc_total);
    const int64_t n_inc = cv.n;
    const f4 *x4 = reinterpret_cast<const f4 *>(path) + cv.path * L * 4;  // 4 pieces of 16 bytes per point

    // state
    float A1 = 0.0f;                  // A_1[w1]
    float A2 = 0.0f;                  // A_2[w1, x]
    // Result of the last level-3 instruction: registers 0..7 (blocks 0,1) = T_4^(3) of that increment,
    // still to be folded into level 4; registers 8..15 (blocks 2,3) = A_3[w1, 4*(lane/16) + c, x], register
    // 4*b + c.  Two buffers, used alternately.
    f16v Da, Db;
    f16v A4[8];                       // group (c, e'): index 2*c + e'
#pragma unroll
    for (int i = 0; i < 16; ++i) Da[i] = Db[i] = 0.0f;
#pragma unroll
    for (int g = 0; g < 8; ++g)
#pragma unroll
        for (int i = 0; i < 16; ++i) A4[g][i] = 0.0f;

    float pzx = 0.0f;                 // z[x] of the increment whose level-4 update is pending

    // per-lane constants of the low-level stages
    const float inv_k = k4 ? 0.25f : 1.0f / 3.0f;            // 1/k of this block's target level
    const int off_zB = (k4 ? 2 : 1) * kD + x;                // z[x]/(k-1): z/3 for k = 4, z/2 for k = 3
    const int off_zC = (k4 ? 1 : 0) * kD + x;                // z[x]/(k-2): z/2 for k = 4, z for k = 3

    for (int64_t t0 = 0; t0 < n_inc; t0 += kTile16) {
        const int nt = int(n_inc - t0 < kTile16 ? n_inc - t0 : kTile16);
        __syncthreads();
        {
            // 512 threads stage 128 increments: thread t takes 16-byte chunk t%4 of increment t/4
            const int i = tid >> 2, c4 = tid & 3;
            if (i < nt) {
                const int64_t s = t0 + i;
                const int64_t i_hi = cv.inc0 + (basepoint ? s : s + 1);
                const f4 hi = x4[i_hi * 4 + c4];
                const f4 lo = i_hi > 0         ? x4[(i_hi - 1) * 4 + c4]
                              : bpv != nullptr ? reinterpret_cast<const f4 *>(bpv)[cv.path * 4 + c4]
                                               : (f4){0.0f, 0.0f, 0.0f, 0.0f};
                const f4 z = hi - lo;
                f4 *row = reinterpret_cast<f4 *>(lds + i * kRow16) + c4;
                row[0] = z;
                row[4] = z * 0.5f;
                row[8] = z * (1.0f / 3.0f);
            }
        }
        __syncthreads();

        // Software pipeline, two increments per trip with two result buffers (no register copies of
        // matrix results on the critical path): in each half-trip the level-3 instruction of the new
        // increment is issued first, then the eight level-4 instructions of the increment before it.
        // Level 4 feeds nothing else and level 3 needs only levels 1..3, so the matrix pipe never
        // waits for a result: the eight long instructions cover the latency of the level-3 result.
        Row16 r = load_row16(lds, w1, x, off_zB, off_zC);
        int s = 0;
        for (; s + 2 <= nt; s += 2) {
            const Row16 r1 = load_row16(lds + (s + 1) * kRow16, w1, x, off_zB, off_zC);
            half_trip(A1, A2, A4, Da, Db, pzx, r, inv_k);
            const Row16 r2 = load_row16(lds + (s + 2 < nt ? s + 2 : s + 1) * kRow16, w1, x, off_zB, off_zC);
            half_trip(A1, A2, A4, Db, Da, pzx, r1, inv_k);
            r = r2;
        }
        if (s < nt) {
            half_trip(A1, A2, A4, Da, Db, pzx, r, inv_k);
            Da = Db;   // keep "Da = result of the last increment" across tiles (odd tile length only)
        }
    }
    // the last increment's level-4 update is still pending
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int ee = 0; ee < 2; ++ee) A4[2 * c + ee] = outer16(Da[4 * ee + c], pzx, A4[2 * c + ee]);
    f16v A3 = Da;   // registers 8..15 hold A_3

    // store (levels concatenated, lexicographic word order)
    float *o = out + path_no * kS16;
    const int hi4 = lane >> 4;   // as a result lane: the high two bits of the second-to-last letter
    if (lane == 0 || lane == 16) o[w1] = A1;
    if (b < 2) o[kOff2 + w1 * kD + x] = A2;
#pragma unroll
    for (int bb = 2; bb < 4; ++bb) {
        const int w1e = 4 * (2 * h + (bb & 1)) + y;
#pragma unroll
        for (int c = 0; c < 4; ++c) o[kOff3 + (w1e * kD + 4 * hi4 + c) * kD + x] = A3[4 * bb + c];
    }
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int ee = 0; ee < 2; ++ee) {
            const int w1e = 4 * (2 * h + ee) + y;
#pragma unroll
            for (int b4 = 0; b4 < 4; ++b4)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int w2 = 4 * b4 + c, w3 = 4 * hi4 + r;
                    o[kOff4 + ((w1e * kD + w2) * kD + w3) * kD + x] = A4[2 * c + ee][4 * b4 + r];
                }
        }
}

}  // namespace

const char *mfma_d16_kernel_name(const Shape &sh)
{
    if (sh.d == 16 && sh.N == 4 && !sh.stream && sh.B <= 0x7fffffff) return "mfma_d16";
    return nullptr;
}

hipError_t launch_mfma_d16_f32(const Shape &sh, const float *path, float *out, hipStream_t st)
{
    if (mfma_d16_kernel_name(sh) == nullptr) return hipErrorNotSupported;
    hipLaunchKernelGGL(sig_mfma_d16_n4_kernel, dim3(static_cast<unsigned>(sh.B)), dim3(512), 0, st, path, out, sh.L,
                       sh.n_inc, sh.basepoint, static_cast<const float *>(sh.basepoint_value), sh.chunks, sh.chunk_len);
    return hipGetLastError();
}

}  // namespace sig
