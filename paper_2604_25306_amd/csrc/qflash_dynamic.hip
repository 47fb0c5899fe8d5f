// Dynamic per-tensor quantisation in front of the attention kernel (Eq. 1-2 evaluated on the fly,
// as in the paper's evaluation set-up), entirely on the GPU: no value ever travels to the host.
//
//   1. abs-max    max |x| over each of Q, K, V (float32): one partial maximum per workgroup (a
//                 maximum is exact in any order, so the result does not depend on the grid)
//   2. quantise   every workgroup finishes the reduction of its tensor; one more workgroup derives the
//                 scales s_X = max|X| / 127 (double) and, from s_Q and s_K, every integer constant of
//                 the attention kernel -- the same routine the host entry point uses -- and builds
//                 the weight table of those constants if it is small enough.  The others compute
//                 x_hat = clip(rint(x * r), -127, 127), r = float32(127) / max|x|: one float32
//                 division per tensor, one float32 multiplication and one round-half-to-even per
//                 element (the precision the rounding decision is defined in)
//   2b. bias      (optional) a bias in real units and an exclusion mask are brought to the integer
//                 score unit of the scales just found and written in the packed layout
//   3. attention  the usual kernel, reading its constants from the device structure of step 2
//
// Steps 1 and 2 stream the float32 tensors once each and are bound by HBM: 12 B read in step 1
// and 12 B read + 3 B written in step 2 per (q, k, v) element triple.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qflash.h"
#include "qflash_internal.h"
#include "qflash_derive.h"
#include "qflash_device.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

// grid.y = tensor (0: Q, 1: K, 2: V); n4 = elements / 4.  Each workgroup leaves its maximum in
// partial[tensor * gridDim.x + workgroup]: atomics on three words would serialise at the L2.
__global__ __launch_bounds__(256) void qflash_dyn_absmax(const float* q, const float* k, const float* v,
                                                        long long n4, float* partial) {
    __shared__ float wmax[4];
    const float* x = blockIdx.y == 0 ? q : blockIdx.y == 1 ? k : v;
    float m = 0.0f;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (long long)gridDim.x * blockDim.x) {
        const v4f t = *(const v4f*)(x + 4 * i);
        m = fmaxf(fmaxf(m, fabsf(t[0])), fmaxf(fabsf(t[1]), fmaxf(fabsf(t[2]), fabsf(t[3]))));
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0)
        partial[blockIdx.y * gridDim.x + blockIdx.x] = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
}

// Maximum over n_partial values by one workgroup of 256 threads; every thread gets the result.
__device__ __forceinline__ float wg_max(const float* partial, int n_partial, float* wmax /* 4 floats of LDS */) {
    float m = 0.0f;
    for (int i = threadIdx.x; i < n_partial; i += 256) m = fmaxf(m, partial[i]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    __syncthreads();                       // wmax may still be read from a previous call
    if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = m;
    __syncthreads();
    return fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
}

// Scales and constants from the three maxima (one thread).
__device__ void derive_on_device(const float am[3], double sqrt_d, int out_round, QflashHeadConsts* hc,
                                 qflash_dynamic_info* info) {
    double s[3];
    for (int t = 0; t < 3; ++t) s[t] = am[t] == 0.0f ? 1.0 : (double)am[t] / 127.0;   // all-zero tensor: scale 1
    qflash_params p;
    int status = qflash_derive_params(s[0], s[1], sqrt_d, &p);
    if (status == QFLASH_OK) {
        p.out_round = out_round;
        if (!qflash_fill_head_consts(p, hc)) status = QFLASH_ERR_PARAM;
    }
    if (status != QFLASH_OK) {
        // Scales outside the supported window: the attention kernel runs on safe constants (those
        // of a mid-range scale) with the requantisation multiplier set to 0, so that every weight is
        // 0, every denominator is 0 and the output is all zeros (Algorithm 1 with l = 0); the status
        // says why.
        (void)qflash_derive_params(0.03, 0.03, sqrt_d, &p);
        p.out_round = out_round;
        (void)qflash_fill_head_consts(p, hc);
        hc->p_mul = 0;
    }
    if (info) {
        info->sQ = s[0]; info->sK = s[1]; info->sV = s[2];
        info->params = p;
        info->status = status;
    }
}

// grid.y = tensor, grid.x = n_partial streaming workgroups + 1; 4 elements per thread and
// iteration: 16 B in, 4 B out.  Every streaming workgroup first finishes the abs-max reduction of
// its tensor from the per-workgroup partial maxima (a few KB, L2-resident).
__global__ __launch_bounds__(256) void qflash_dyn_quantize(const float* q, const float* k, const float* v,
                                                          int8_t* qo, int8_t* ko, int8_t* vo, long long n4,
                                                          const float* partial, int n_partial, double sqrt_d,
                                                          int out_round, QflashHeadConsts* hc,
                                                          qflash_dynamic_info* info, uint8_t* table, int table_max) {
    __shared__ float wmax[4];
    __shared__ QflashHeadConsts sh_hc;
    // One workgroup beyond the streaming ones (x == n_partial, tensor 0) does what needs all three
    // maxima: it derives the scales and constants for the attention kernel that follows on the
    // stream and, if there is room for it, builds the weight table of those constants, all while
    // the others stream.
    if (blockIdx.x == (unsigned)n_partial) {
        if (blockIdx.y != 0) return;
        float a3[3];
        for (int t = 0; t < 3; ++t) a3[t] = wg_max(partial + t * n_partial, n_partial, wmax);
        if (threadIdx.x == 0) {
            derive_on_device(a3, sqrt_d, out_round, &sh_hc, info);
            // table of x_p + 1 entries, x_p = ceil(8 s_inv / 2^k) (the host's rule), padded to 16
            const long long x_p = (8ll * sh_hc.s_inv + (1ll << sh_hc.x_shift) - 1) >> sh_hc.x_shift;
            const long long n_padded = (x_p + 1 + 15) & ~15ll;
            const bool fits = table != nullptr && n_padded <= (long long)table_max;
            sh_hc.lut = fits ? table : nullptr;
            sh_hc.lut_bytes = fits ? (int)n_padded : 0;
            sh_hc.lut_xp = fits ? (int)x_p : 0;
            *hc = sh_hc;
        }
        __syncthreads();
        if (sh_hc.lut_bytes > 0) {
            const QflashHeadConsts h = sh_hc;
            const ExpConst c = make_exp_const(h);
            for (int i = threadIdx.x; i < h.lut_bytes; i += 256)
                table[i] = (uint8_t)(i <= h.lut_xp ? table_entry(i, h.lut_xp, h, c) : 0u);
        }
        return;
    }
    const float* x = blockIdx.y == 0 ? q : blockIdx.y == 1 ? k : v;
    int8_t* y = blockIdx.y == 0 ? qo : blockIdx.y == 1 ? ko : vo;
    const float am = wg_max(partial + blockIdx.y * n_partial, n_partial, wmax);
    const float r = am == 0.0f ? 0.0f : __fdiv_rn(127.0f, am);
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (long long)n_partial * blockDim.x) {
        const v4f t = *(const v4f*)(x + 4 * i);
        unsigned w = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float z = fminf(fmaxf(rintf(__fmul_rn(t[e], r)), -127.0f), 127.0f);
            w |= ((unsigned)(int)z & 0xffu) << (8 * e);
        }
        *(unsigned*)(y + 4 * i) = w;
    }
}

// Real bias and exclusion mask -> int32 bias in the lane-major packed layout the attention kernel
// reads (see qflash_pack_bias_kernel for the layout), in the score unit of the scales just found:
//   unit = (s_Q s_K) / sqrt(d),  b_hat = clip(floor(double(b) / unit + 0.5), -(2^20 - 1), 2^20 - 1)
// evaluated in float64 with one rounding per operation (the precision the decision is defined in).
// One thread per 16-byte word; every workgroup first finishes the abs-max reduction of Q and K.
__global__ __launch_bounds__(256) void qflash_dyn_bias(const float* __restrict__ bias, const uint8_t* __restrict__ mask,
                                                      int32_t* __restrict__ packed, int N, long long n_words,
                                                      const float* partial, int n_partial, double sqrt_d) {
    __shared__ float wmax[4];
    const float aq = wg_max(partial, n_partial, wmax);
    const float ak = wg_max(partial + n_partial, n_partial, wmax);
    const double sq = aq == 0.0f ? 1.0 : __ddiv_rn((double)aq, 127.0);
    const double sk = ak == 0.0f ? 1.0 : __ddiv_rn((double)ak, 127.0);
    const double unit = __ddiv_rn(__dmul_rn(sq, sk), sqrt_d);
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= n_words) return;
    const int nb = (N + 31) / 32;
    const int lane = (int)(t & 63), a4 = (int)((t >> 6) & 3);
    const long long blk = t >> 8;
    const int cb = (int)(blk % nb), rb = (int)((blk / nb) % nb);
    const long long slice = blk / ((long long)nb * nb);
    const int li = lane & 31, g = lane >> 5;
    const int row = min(32 * rb + li, N - 1), col0 = 32 * cb + 8 * a4 + 4 * g;
    const long long base = (slice * N + row) * (long long)N;
    int32_t w[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        int32_t v = INT32_MIN;
        if (col0 + b < N && !(mask && mask[base + col0 + b] != 0)) {
            const double x = bias ? (double)bias[base + col0 + b] : 0.0;
            const double r = floor(__dadd_rn(__ddiv_rn(x, unit), 0.5));
            v = (int32_t)fmin(fmax(r, -1048575.0), 1048575.0);
        }
        w[b] = v;
    }
    *(int4*)(packed + 4 * t) = int4{w[0], w[1], w[2], w[3]};
}

}  // namespace

int qflash_launch_dynamic_bias(const float* bias, const uint8_t* mask, int slices, int N, int32_t* packed,
                               const float* scratch, long long n, double sqrt_d, void* stream) {
    const long long n_words = qflash_packed_bias_words(slices, N);
    hipLaunchKernelGGL(qflash_dyn_bias, dim3((unsigned)((n_words + 255) / 256)), dim3(256), 0, (hipStream_t)stream, bias, mask,
                       packed, N, n_words, scratch, qflash_dynamic_partials(n), sqrt_d);
    return (int)hipGetLastError();
}

int qflash_dynamic_partials(long long n) {
    // enough workgroups to keep every HBM channel busy (two per compute unit and tensor); each
    // streams a grid-strided share
    long long wgs = (n / 4 + 255) / 256;
    // (every workgroup of the second kernel re-reads all partial maxima of its tensor: with 2048
    // of them that prologue cost a fifth of the kernel)
    if (wgs > 512) wgs = 512;
    if (wgs < 1) wgs = 1;
    return (int)wgs;
}

int qflash_launch_dynamic_front(const float* Qf, const float* Kf, const float* Vf, int8_t* Qo, int8_t* Ko, int8_t* Vo,
                                long long n, double sqrt_d, int out_round, float* scratch,
                                QflashHeadConsts* hc_dev, qflash_dynamic_info* info, uint8_t* table, int table_max,
                                void* stream) {
    hipStream_t st = (hipStream_t)stream;
    const long long n4 = n / 4;
    const int wgs = qflash_dynamic_partials(n);
    float* partial = scratch;         // 3 * wgs words
    hipLaunchKernelGGL(qflash_dyn_absmax, dim3((unsigned)wgs, 3), dim3(256), 0, st, Qf, Kf, Vf, n4, partial);
    hipLaunchKernelGGL(qflash_dyn_quantize, dim3((unsigned)wgs + 1, 3), dim3(256), 0, st, Qf, Kf, Vf, Qo, Ko, Vo, n4,
                       (const float*)partial, wgs, sqrt_d, out_round, hc_dev, info, table, table_max);
    return (int)hipGetLastError();
}
