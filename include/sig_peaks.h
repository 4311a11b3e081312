/*
 * libsig_peaks — microbenchmarks of the MI355X (gfx950) limits that the signature kernels are priced against.
 * Measurement support for bench.py only: nothing in libsig uses it, and it holds no signature arithmetic.
 * The caller times each call with HIP events on `hip_stream` and divides the work stated below by the time.
 * C ABI, device pointers, nothing allocated, nothing synchronised; every call returns 0, or the hipError_t of the
 * launch as a negative number, or -1 for bad arguments.
 */
#ifndef SIG_PEAKS_H_
#define SIG_PEAKS_H_

#include <stdint.h>
#include <hip/hip_runtime_api.h>

#ifdef __cplusplus
extern "C" {
#endif

/* fp32 matrix-core throughput: `workgroups` x 4 wavefronts, each issuing `iters` x 8 independent
 * v_mfma_f32_32x32x2_f32 (4096 flop each).  sink: DEVICE pointer to at least workgroups * 256 floats (written once,
 * so that the arithmetic is kept).  Work: workgroups * 4 * iters * 8 * 4096 flop. */
int sig_peak_mfma_f32(float *sink, int workgroups, int iters, hipStream_t hip_stream);

/* As above with v_mfma_f32_4x4x1_16b_f32 (512 flop each), the instruction the d = 4 and d = 8 kernels use.
 * Work: workgroups * 4 * iters * 8 * 512 flop. */
int sig_peak_mfma_f32_4x4x1(float *sink, int workgroups, int iters, hipStream_t hip_stream);

/* fp32 vector throughput with plain (not packed) v_fma_f32: `workgroups` x 256 lanes, each running `iters` x 16
 * independent multiply-adds.  Work: workgroups * 256 * iters * 16 * 2 flop. */
int sig_peak_valu_f32(float *sink, int workgroups, int iters, hipStream_t hip_stream);

/* HBM write bandwidth: fills `bytes` (a multiple of 16) at the 16-byte aligned DEVICE pointer `dst` with 16-byte
 * stores, every wavefront writing runs of 64 KB.  Work: `bytes` written.  (A buffer that fits the 256 MB last-level
 * cache measures that cache, not HBM.) */
int sig_peak_hbm_write(void *dst, int64_t bytes, hipStream_t hip_stream);

/* HBM copy bandwidth: `bytes` (a multiple of 16) from `src` to `dst` (both 16-byte aligned DEVICE pointers, not
 * overlapping).  Work: `bytes` read + `bytes` written. */
int sig_peak_hbm_copy(void *dst, const void *src, int64_t bytes, hipStream_t hip_stream);

/* Adding into LDS: `workgroups` x 4 wavefronts, each repeating `iters` times one float add into its own row of 64
 * scalars, `active_lanes` (1..64) lanes taking part, lane l at scalar (l * stride) % 64 (stride 1: an address per lane,
 * 0: one address for all).  atomic != 0: an LDS atomic add; 0: a read, an add and a write (only meaningful with distinct
 * addresses).  Work: workgroups * 4 * iters wavefront operations; with 8 workgroups per compute unit the time per
 * operation and compute unit shows what the LDS port sustains. */
int sig_peak_lds_add(float *sink, int workgroups, int iters, int active_lanes, int stride, int atomic, hipStream_t hip_stream);

#ifdef __cplusplus
}
#endif

#endif /* SIG_PEAKS_H_ */
