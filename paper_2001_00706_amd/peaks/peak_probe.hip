// Microbenchmarks of the gfx950 limits the signature kernels are priced against (see sig_peaks.h).
#include <hip/hip_runtime.h>

#include "sig_peaks.h"

namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;

__global__ __launch_bounds__(kThreads) void mfma_32x32x2_kernel(float *__restrict__ sink, int iters)
{
    f16 acc[8];
#pragma unroll
    for (int r = 0; r < 8; ++r)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[r][i] = 0.0f;
    const float a = 1.0f + threadIdx.x * 1e-3f, b = 1.0f - threadIdx.x * 1e-3f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 8; ++r) acc[r] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[r], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int r = 0; r < 8; ++r)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[r][i];
    sink[blockIdx.x * kThreads + threadIdx.x] = s;
}

__global__ __launch_bounds__(kThreads) void mfma_4x4x1_kernel(float *__restrict__ sink, int iters)
{
    f4 acc[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) acc[r] = f4{0.0f, 0.0f, 0.0f, 0.0f};
    const float a = 1.0f + threadIdx.x * 1e-3f, b = 1.0f - threadIdx.x * 1e-3f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 8; ++r) acc[r] = __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, acc[r], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int r = 0; r < 8; ++r) s += acc[r][0] + acc[r][1] + acc[r][2] + acc[r][3];
    sink[blockIdx.x * kThreads + threadIdx.x] = s;
}

__global__ __launch_bounds__(kThreads) void valu_fma_kernel(float *__restrict__ sink, int iters)
{
    float acc[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = threadIdx.x * 1e-3f + r;
    const float a = 0.999f, b = 1e-3f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = __builtin_fmaf(acc[r], a, b);
    }
    float s = 0.0f;
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[r];
    sink[blockIdx.x * kThreads + threadIdx.x] = s;
}

// Every wavefront writes runs of 64 consecutive 1 KB pieces (64 KB), the runs of the wavefronts interleaved: the
// pattern this device's memory system absorbs fastest (1 KB pieces interleaved across wavefronts reach about a
// quarter less).
constexpr int kRunPieces = 64;

__global__ __launch_bounds__(kThreads) void hbm_write_kernel(f4 *__restrict__ dst, int64_t n16)
{
    const f4 v = f4{1.0f, 2.0f, 3.0f, 4.0f};
    const int64_t wave = ((int64_t)blockIdx.x * kThreads + threadIdx.x) >> 6, waves = (int64_t)gridDim.x * (kThreads / 64);
    const int lane = threadIdx.x & 63;
    for (int64_t base = wave * kRunPieces * 64; base < n16; base += waves * kRunPieces * 64)
        for (int r = 0; r < kRunPieces; ++r) {
            const int64_t i = base + r * 64 + lane;
            if (i < n16) dst[i] = v;
        }
}

__global__ __launch_bounds__(kThreads) void hbm_copy_kernel(f4 *__restrict__ dst, const f4 *__restrict__ src, int64_t n16)
{
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n16; i += (int64_t)gridDim.x * kThreads)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// The cost of adding into LDS: every wavefront of a workgroup repeats one float add into its own row of 64 scalars,
// with `active` lanes taking part and lane l adding at scalar (l * stride) % 64 (stride 1: every lane its own address,
// 0: all lanes one address).  ATOMIC: ds_add_f32; otherwise a read, an add and a write.
template <bool ATOMIC>
__global__ __launch_bounds__(kThreads) void lds_add_kernel(float *__restrict__ sink, int iters, int active, int stride)
{
    __shared__ float row[kThreads / 64][64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    row[w][lane] = 0.f;
    __syncthreads();
    const float v = float(lane) * 1e-3f;
    float *slot = &row[w][(lane * stride) & 63];
    for (int it = 0; it < iters; ++it) {
        if (lane < active) {
            if (ATOMIC)
                atomicAdd(slot, v);
            else
                *slot = *slot + v;
        }
    }
    __syncthreads();
    sink[blockIdx.x * kThreads + threadIdx.x] = row[w][lane];
}

int finish()
{
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? 0 : -(int)e;
}

bool bad_compute_args(const float *sink, int workgroups, int iters)
{
    return sink == nullptr || workgroups < 1 || workgroups > (1 << 20) || iters < 1;
}

bool bad_memory_args(const void *p, int64_t bytes)
{
    return p == nullptr || bytes < 16 || (bytes & 15) != 0 || (reinterpret_cast<uintptr_t>(p) & 15) != 0;
}

int memory_grid(int64_t n16)
{
    const int64_t want = (n16 + kThreads - 1) / kThreads;
    return (int)(want < 256 * 32 ? want : 256 * 32);
}

}  // namespace

extern "C" int sig_peak_mfma_f32(float *sink, int workgroups, int iters, hipStream_t hip_stream)
{
    if (bad_compute_args(sink, workgroups, iters)) return -1;
    hipLaunchKernelGGL(mfma_32x32x2_kernel, dim3(workgroups), dim3(kThreads), 0, hip_stream, sink, iters);
    return finish();
}

extern "C" int sig_peak_mfma_f32_4x4x1(float *sink, int workgroups, int iters, hipStream_t hip_stream)
{
    if (bad_compute_args(sink, workgroups, iters)) return -1;
    hipLaunchKernelGGL(mfma_4x4x1_kernel, dim3(workgroups), dim3(kThreads), 0, hip_stream, sink, iters);
    return finish();
}

extern "C" int sig_peak_valu_f32(float *sink, int workgroups, int iters, hipStream_t hip_stream)
{
    if (bad_compute_args(sink, workgroups, iters)) return -1;
    hipLaunchKernelGGL(valu_fma_kernel, dim3(workgroups), dim3(kThreads), 0, hip_stream, sink, iters);
    return finish();
}

extern "C" int sig_peak_hbm_write(void *dst, int64_t bytes, hipStream_t hip_stream)
{
    if (bad_memory_args(dst, bytes)) return -1;
    const int64_t n16 = bytes / 16;
    hipLaunchKernelGGL(hbm_write_kernel, dim3(memory_grid(n16)), dim3(kThreads), 0, hip_stream,
                       static_cast<f4 *>(dst), n16);
    return finish();
}

extern "C" int sig_peak_hbm_copy(void *dst, const void *src, int64_t bytes, hipStream_t hip_stream)
{
    if (bad_memory_args(dst, bytes) || bad_memory_args(src, bytes)) return -1;
    const int64_t n16 = bytes / 16;
    hipLaunchKernelGGL(hbm_copy_kernel, dim3(memory_grid(n16)), dim3(kThreads), 0, hip_stream,
                       static_cast<f4 *>(dst), static_cast<const f4 *>(src), n16);
    return finish();
}

extern "C" int sig_peak_lds_add(float *sink, int workgroups, int iters, int active_lanes, int stride, int atomic,
                                hipStream_t hip_stream)
{
    if (bad_compute_args(sink, workgroups, iters) || active_lanes < 1 || active_lanes > 64 || stride < 0 || stride > 64) return -1;
    if (atomic)
        hipLaunchKernelGGL(lds_add_kernel<true>, dim3(workgroups), dim3(kThreads), 0, hip_stream, sink, iters, active_lanes, stride);
    else
        hipLaunchKernelGGL(lds_add_kernel<false>, dim3(workgroups), dim3(kThreads), 0, hip_stream, sink, iters, active_lanes, stride);
    return finish();
}
