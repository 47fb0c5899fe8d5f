/*
 * qflash_peaks.h -- three measurement kernels for the benchmark's roofline denominators (MI355X, gfx950).
 *
 * Not part of the attention path: the benchmark prices the fused kernel against the published peaks
 * (8 TB/s HBM, 5.0 POP/s dense int8 matrix rate; vector rate from unit counts and clock) and
 * reports beside them what this chip sustains,
 * measured with these kernels in the same run.  Every function enqueues one kernel on `hip_stream`
 * (NULL = the default stream) and returns at once; the caller times it with events.  Returns 0, or
 * a negative code: -1 a pointer is NULL, -2 a size is out of range, -8 misaligned, -6 launch failed.
 */
#ifndef QFLASH_PEAKS_H
#define QFLASH_PEAKS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * int8 matrix rate.  `workgroups` workgroups of 4 wavefronts each issue `iters` x 4 independent
 * v_mfma_i32_32x32x32_i8 (operands in registers, nothing else in the loop).  dev_out (device, 8-byte
 * aligned, at least 16 * workgroups + 16 bytes) receives per workgroup two uint64: the shader clock
 * cycles of the loop and the same interval in ticks of the constant 100 MHz clock; their ratio is the
 * sustained clock.  qflash_peaks_mfma_i8_ops gives the number of int8 operations such a launch
 * executes (2 per multiply-add).
 */
int qflash_peaks_mfma_i8(int workgroups, int iters, void* dev_out, size_t dev_out_bytes, void* hip_stream);
double qflash_peaks_mfma_i8_ops(int workgroups, int iters);

/*
 * HBM rate: copies `bytes` (a multiple of 16) from dev_src to dev_dst (device, 16-byte aligned, not
 * overlapping).  The achieved rate is 2 * bytes / time (every byte is read once and written once).
 */
int qflash_peaks_copy(const void* dev_src, void* dev_dst, size_t bytes, void* hip_stream);

/*
 * Vector integer issue rate.  `workgroups` workgroups of 16 wavefronts (four per SIMD when one
 * workgroup runs per compute unit, the occupancy of the attention kernels) each issue `iters` (a
 * multiple of 8) x 16
 * independent 32-bit integer instructions from registers only, a quarter each of saturating subtract,
 * high multiply, add and byte permute (the kinds the softmax part of the attention loop consists of).
 * dev_out as for qflash_peaks_mfma_i8.  qflash_peaks_valu_lane_ops gives the lane-operations of such
 * a launch (64 per instruction and wavefront).
 */
int qflash_peaks_valu(int workgroups, int iters, void* dev_out, size_t dev_out_bytes, void* hip_stream);
double qflash_peaks_valu_lane_ops(int workgroups, int iters);

#ifdef __cplusplus
}
#endif
#endif /* QFLASH_PEAKS_H */
