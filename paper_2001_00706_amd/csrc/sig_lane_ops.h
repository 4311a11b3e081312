// Sums over groups of lanes of a wavefront with DPP moves and ds_bpermute (no LDS traffic, no barrier).
#ifndef SIG_LANE_OPS_H_
#define SIG_LANE_OPS_H_

#include "sig_mfma_common.h"

namespace sig {

// Value of v in a lane of the neighbouring group of MASK lanes (MASK a power of two).  For MASK = 1, 2 it is
// the lane whose number differs in that bit; for 4 and 8 the lane mirrored inside 8 or 16 lanes, which lies in
// the neighbouring group and carries that group's value whenever v is the same throughout each group of MASK
// lanes; for 16 and 32 the lane whose number differs in that bit.
template <int MASK>
__device__ __forceinline__ float neighbour(float v)
{
    if constexpr (MASK == 1) return quad_swap<0xB1>(v);         // quad_perm [1,0,3,2]
    else if constexpr (MASK == 2) return quad_swap<0x4E>(v);    // quad_perm [2,3,0,1]
    else if constexpr (MASK == 4) return quad_swap<0x141>(v);   // row_half_mirror
    else if constexpr (MASK == 8) return quad_swap<0x140>(v);   // row_mirror
    else return __shfl_xor(v, MASK);
}

// The same for a double: its two halves travel separately.
template <int MASK>
__device__ __forceinline__ double neighbour(double v)
{
    if constexpr (MASK >= 16) {
        return __shfl_xor(v, MASK);
    } else {
        const unsigned long long bits = __builtin_bit_cast(unsigned long long, v);
        const float lo = neighbour<MASK>(__builtin_bit_cast(float, unsigned(bits)));
        const float hi = neighbour<MASK>(__builtin_bit_cast(float, unsigned(bits >> 32)));
        return __builtin_bit_cast(double, (unsigned long long)(__builtin_bit_cast(unsigned, hi)) << 32 |
                                              __builtin_bit_cast(unsigned, lo));
    }
}

// Sum of v over the 2^CNT groups of 2^LO lanes that differ in lane-number bits LO .. LO+CNT-1, in every lane.
// v must be the same throughout each aligned group of 2^LO lanes.
template <int LO, int CNT, typename T>
__device__ __forceinline__ T group_sum(T v)
{
    if constexpr (CNT > 0) {
        v += neighbour<(1 << LO)>(v);
        return group_sum<LO + 1, CNT - 1, T>(v);
    } else {
        return v;
    }
}

// A workgroup barrier that orders the LDS traffic only: __syncthreads() would also wait for the global loads and stores a
// wavefront has in flight, which is the latency a kernel that fetches its next tile ahead is built to hide.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

}  // namespace sig

#endif  // SIG_LANE_OPS_H_
