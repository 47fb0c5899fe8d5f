// Measured roofline denominators for the benchmark: what this chip sustains on the two resources the
// fused attention kernel is priced against.  Three kernels, all launched asynchronously through a C
// ABI of their own (include/qflash_peaks.h); the caller times them with events.
//   - int8 matrix rate: every wavefront issues independent v_mfma_i32_32x32x32_i8 back to back from
//     registers only, and reads the shader clock and the constant 100 MHz clock around the loop,
//     so that both operations per clock and compute unit and the sustained clock can be reported;
//   - HBM rate: a plain device-to-device copy, 16 bytes per lane and iteration;
//   - vector integer issue rate: sixteen wavefronts per workgroup (four per SIMD, the occupancy of
//     the attention kernels) issue independent 32-bit integer instructions of the kinds the softmax
//     part of the attention loop is made of, from registers only.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qflash_peaks.h"

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

namespace {

constexpr int kChains = 4;   // independent accumulators per wavefront (the matrix pipe never waits on a result)

__global__ __launch_bounds__(256) void peak_mfma_i8(int iters, unsigned long long* out, int* sink) {
    const int lane = threadIdx.x & 63;
    v4i a = {lane, lane + 1, lane + 2, lane + 3}, b = {3 * lane, 5 * lane, 7 * lane, 9 * lane};
    v16i acc[kChains];
#pragma unroll
    for (int c = 0; c < kChains; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[c][v] = c + v;
    const unsigned long long c0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int c = 0; c < kChains; ++c) acc[c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[c], 0, 0, 0);
    }
    const unsigned long long c1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
    int s = 0;
#pragma unroll
    for (int c = 0; c < kChains; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) s ^= acc[c][v];
    if (s == 0x7fffffff) *sink = s;          // keeps the loop alive; practically never taken
    if (threadIdx.x == 0) {
        out[2 * blockIdx.x] = c1 - c0;       // shader clock cycles of the loop
        out[2 * blockIdx.x + 1] = r1 - r0;   // the same interval in 10 ns ticks
    }
}

constexpr int kValuRegs = 16;   // independent registers per lane: no instruction waits on the one before it

__global__ __launch_bounds__(1024) void peak_valu(int iters, unsigned long long* out, int* sink) {
    unsigned r[kValuRegs];
#pragma unroll
    for (int i = 0; i < kValuRegs; ++i) r[i] = 0x40000000u + threadIdx.x * 7u + i;
    unsigned b = 0x9e3779b1u + threadIdx.x;
    asm volatile("" : "+v"(b));
    const unsigned long long c0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iters; it += 8)      // (eight rounds per loop iteration: the loop's own scalar instructions do not weigh)
#pragma unroll
      for (int round = 0; round < 8; ++round) {
#pragma unroll
        for (int i = 0; i < kValuRegs; ++i) {
            // a quarter each: saturating subtract, high multiply, add, byte permute
            if ((i & 3) == 0) r[i] = __builtin_elementwise_sub_sat(r[i], b);
            else if ((i & 3) == 1) r[i] = __umulhi(r[i], b);
            else if ((i & 3) == 2) r[i] = r[i] + b;
            else r[i] = __builtin_amdgcn_perm(r[i], b, 0x07020500u);
            asm volatile("" : "+v"(r[i]));       // one instruction each: nothing is merged or hoisted
        }
    }
    const unsigned long long c1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
    unsigned s = 0;
#pragma unroll
    for (int i = 0; i < kValuRegs; ++i) s ^= r[i];
    if (s == 0x7fffffffu && iters < 0) *sink = (int)s;     // keeps the loop alive; never taken
    if (threadIdx.x == 0) {
        out[2 * blockIdx.x] = c1 - c0;
        out[2 * blockIdx.x + 1] = r1 - r0;
    }
}

__global__ __launch_bounds__(256) void peak_copy(const v4i* __restrict__ src, v4i* __restrict__ dst, long long n16) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n16; i += (long long)gridDim.x * 256) dst[i] = src[i];
}

}  // namespace

extern "C" int qflash_peaks_mfma_i8(int workgroups, int iters, void* dev_out, size_t dev_out_bytes, void* hip_stream) {
    if (!dev_out) return -1;
    if (workgroups < 1 || workgroups > 65536 || iters < 1) return -2;
    if (dev_out_bytes < 16 * (size_t)workgroups + 16) return -2;
    if ((uintptr_t)dev_out & 7u) return -8;
    unsigned long long* out = (unsigned long long*)dev_out;
    hipLaunchKernelGGL(peak_mfma_i8, dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)hip_stream, iters, out,
                       (int*)(out + 2 * (size_t)workgroups));
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

extern "C" double qflash_peaks_mfma_i8_ops(int workgroups, int iters) {
    // 4 wavefronts per workgroup, kChains instructions per iteration, 2 * 32 * 32 * 32 operations each
    return 4.0 * workgroups * (double)iters * kChains * 65536.0;
}

extern "C" int qflash_peaks_valu(int workgroups, int iters, void* dev_out, size_t dev_out_bytes, void* hip_stream) {
    if (!dev_out) return -1;
    if (workgroups < 1 || workgroups > 65536 || iters < 8 || (iters & 7)) return -2;
    if (dev_out_bytes < 16 * (size_t)workgroups + 16) return -2;
    if ((uintptr_t)dev_out & 7u) return -8;
    unsigned long long* out = (unsigned long long*)dev_out;
    hipLaunchKernelGGL(peak_valu, dim3((unsigned)workgroups), dim3(1024), 0, (hipStream_t)hip_stream, iters, out,
                       (int*)(out + 2 * (size_t)workgroups));
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

extern "C" double qflash_peaks_valu_lane_ops(int workgroups, int iters) {
    // 16 wavefronts per workgroup, kValuRegs instructions per iteration, 64 lanes each
    return 16.0 * workgroups * (double)iters * kValuRegs * 64.0;
}

extern "C" int qflash_peaks_copy(const void* dev_src, void* dev_dst, size_t bytes, void* hip_stream) {
    if (!dev_src || !dev_dst) return -1;
    if (bytes < 16 || (bytes & 15u)) return -2;
    if (((uintptr_t)dev_src | (uintptr_t)dev_dst) & 15u) return -8;
    hipLaunchKernelGGL(peak_copy, dim3(8192), dim3(256), 0, (hipStream_t)hip_stream, (const v4i*)dev_src, (v4i*)dev_dst,
                       (long long)(bytes / 16));
    return hipGetLastError() == hipSuccess ? 0 : -6;
}
