// Small device helpers shared by the matrix-core kernels.
#ifndef SIG_MFMA_COMMON_H_
#define SIG_MFMA_COMMON_H_

#include <hip/hip_runtime.h>

namespace sig {

typedef float f4 __attribute__((ext_vector_type(4)));

// v_mfma_f32_4x4x1_16b_f32: 16 independent blocks of D[i][j] = a[i] * b[j] + C[i][j].
// Lane 4*blk + i supplies a[i], lane 4*blk + j supplies b[j]; register i of lane 4*blk + j
// receives D[i][j].
__device__ __forceinline__ f4 outer4(float a, float b, f4 c)
{
    return __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, c, 0, 0, 0);
}

// Value of `v` in the lane whose number differs in bit 0 (XOR1) or bit 1 (XOR2) of the quad.
template <int CTRL>
__device__ __forceinline__ float quad_swap(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}

// Transposes the 4x4 tile held by a lane quad (register r of lane q <-> register q of lane r)
// with two butterfly stages of quad-permute DPP moves.
__device__ __forceinline__ f4 quad_transpose(f4 v, int lane)
{
    const bool b0 = (lane & 1) != 0, b1 = (lane & 2) != 0;
#pragma unroll
    for (int p = 0; p < 4; p += 2) {  // rows (p, p+1) with the lane one to the side
        const float a = v[p], b = v[p + 1];
        const float got = quad_swap<0xB1>(b0 ? a : b);  // quad_perm [1,0,3,2]
        v[p] = b0 ? got : a;
        v[p + 1] = b0 ? b : got;
    }
#pragma unroll
    for (int p = 0; p < 2; ++p) {  // rows (p, p+2) with the lane two to the side
        const float a = v[p], b = v[p + 2];
        const float got = quad_swap<0x4E>(b1 ? a : b);  // quad_perm [2,3,0,1]
        v[p] = b1 ? got : a;
        v[p + 2] = b1 ? b : got;
    }
    return v;
}

}  // namespace sig

#endif  // SIG_MFMA_COMMON_H_
