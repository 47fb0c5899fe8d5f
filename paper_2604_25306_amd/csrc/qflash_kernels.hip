// gfx950 (CDNA4) kernels of the integer-only fused attention forward pass (Algorithm 1).
//
// Operand layout (the point of the design)
//   Both products are computed transposed on the 32x32x32 int8 MFMA:
//       S^T = K_j Q_i^T        (A = K rows, B = Q rows)          -> C[kv][query]
//       O^T = V_j^T P^T        (A = V^T rows, B = P^T)           -> C[t][query]
//   In the MFMA result layout lane l holds column (l % 32) and 16 rows, so every lane owns ONE
//   query row: 16 of each 32 scores of that row (the other 16 sit in lane l^32), its running
//   maximum, denominator and alpha, and 16 of each 32 output features.  The row maximum and row
//   sum are in-lane operations plus a single exchange with lane l^32, alpha is a per-lane
//   scalar, and the four dwords of int8 weights a lane produces are, unchanged, its B operand of
//   the second product: P never leaves registers.  The price is that the k-slots of that operand
//   enumerate the kv rows in result-layout order (8*(j/4) + 4*(l/32) + j%4), so V^T is written to
//   LDS with its columns in exactly that order.  Integer addition is associative, so the order of
//   the contraction does not change a single bit of the result.
//
// Two kernels share the per-tile code:
//   resident  one workgroup = one (batch, head) pair and up to 8 (N <= 256) or 12 wavefronts of
//             32 query rows, or several short pairs (windowed attention) side by side; K and V^T
//             of each pair live in LDS (N up to about 1100), every KV tile in a region of its
//             own.  They are staged either all at once (one barrier, then no barrier in the KV
//             loop) or tile by tile, one tile ahead of its use, with the next tile's global loads
//             in flight during the arithmetic and one barrier per tile.  Long sequences keep
//             only two tiles in LDS (the one in use, the one being staged) so that several
//             smaller workgroups share a compute unit.
//   stream    one workgroup = 128 query rows; KV tiles are staged per iteration (any N).
//
// An additive int32 bias (windowed attention) comes in one of two layouts, each a template variant:
// plain [N,N], where every lane reads its own row dword by dword, or packed lane-major (see
// bias_lane_base), where a wavefront reads 1 KiB per instruction and keys beyond the sequence are
// already excluded.
//
// The element-wise integer softmax is what takes the time (about six VALU instructions per score
// a lane handles, against 256 MFMA operations and 1.3 HBM bytes per score), so the per-element
// path is kept short: where the constants allow it the int8 weight of a score comes from a table
// in LDS (one saturating subtraction and one byte read); otherwise Algorithm 2 runs on the
// 24-bit multiplier (v_mul_hi_i32_i24), leaves its int8 result in the top byte of a product, and
// four of them are gathered with v_perm_b32.  Accumulators (and, where registers allow, scores)
// carry an offset of 2^30 that turns the rescale into a multiply-high and an add and the table
// index into a single subtraction.  Inline assembly never reads a register written by an MFMA:
// the compiler only places the wait states of the matrix pipeline for reads it can see.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "qflash_resident.h"

namespace {

// Weight table for the look-up mode: T[i] = int8 weight (Algorithm 2 + Eq. 10) of the score
// difference x = i - x_p, for i in [0, x_p]; x_p is chosen on the host so that the weight is 0 at
// and below -x_p.  Entries [n, n_padded) are 0 and never addressed.  Built by the same device
// functions the arithmetic mode uses, so the two modes cannot disagree.
__global__ __launch_bounds__(256) void qflash_build_table(uint8_t* tbl, int n, int n_padded, int x_p,
                                                          const QflashHeadConsts a) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n_padded) return;
    const ExpConst c = make_exp_const(a);
    tbl[i] = (uint8_t)(i < n ? table_entry(i, x_p, a, c) : 0u);
}

}  // namespace

int qflash_launch_build_table(uint8_t* tbl, int n, int n_padded, int x_p, const QflashHeadConsts& a, void* stream) {
    hipLaunchKernelGGL(qflash_build_table, dim3((unsigned)((n_padded + 255) / 256)), dim3(256), 0,
                       (hipStream_t)stream, tbl, n, n_padded, x_p, a);
    return (int)hipGetLastError();
}

// Plain bias [slices,N,N] -> the lane-major layout bias_lane_base() describes.  One thread per
// 16-byte word.  Rows beyond the sequence repeat row N-1 (never stored), columns beyond it are
// excluded.
__global__ __launch_bounds__(256) void qflash_pack_bias_kernel(const int32_t* __restrict__ bias, int32_t* __restrict__ packed,
                                                               int N, long long n_words) {
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= n_words) return;
    const int nb = (N + 31) / 32;
    const int lane = (int)(t & 63), a4 = (int)((t >> 6) & 3);
    const long long blk = t >> 8;
    const int cb = (int)(blk % nb), rb = (int)((blk / nb) % nb);
    const long long slice = blk / ((long long)nb * nb);
    const int li = lane & 31, g = lane >> 5;
    const int row = min(32 * rb + li, N - 1), col0 = 32 * cb + 8 * a4 + 4 * g;
    const int32_t* src = bias + (slice * N + row) * (long long)N;
    v4i w;
#pragma unroll
    for (int b = 0; b < 4; ++b) w[b] = col0 + b < N ? src[col0 + b] : INT32_MIN;
    *(v4i*)(packed + 4 * t) = w;
}

int qflash_launch_pack_bias(const int32_t* bias, int slices, int N, int32_t* packed, void* stream) {
    const long long n_words = qflash_packed_bias_words(slices, N);
    hipLaunchKernelGGL(qflash_pack_bias_kernel, dim3((unsigned)((n_words + 255) / 256)), dim3(256), 0,
                       (hipStream_t)stream, bias, packed, N, n_words);
    return (int)hipGetLastError();
}

int qflash_launch_fwd(const QflashKernelArgs& a, int d, int kv_tile, int lds_limit, void* stream) {
    hipStream_t st = (hipStream_t)stream;
    if (a.ring && (!a.pipelined || d != 64 || a.kv_tile != kv_tile || a.heads_per_wg != 1 || a.waves_per_head < 4))
        return (int)hipErrorInvalidValue;   // the ring is compiled into the tile-by-tile variants only
    const size_t lds = a.resident ? qflash_resident_lds_bytes(a.N, d, a.heads_per_wg, (a.exp_mode == kExpTable || a.exp_mode == kExpAuto) ? a.lut_bytes_max : 0,
                                                       lds_limit, a.ring ? kv_tile : 0) : 0;
    if (a.resident && lds == 0) return (int)hipErrorInvalidValue;
    const int threads = a.resident ? 64 * a.waves_per_head * a.heads_per_wg : kStreamThreads;
    if (a.qmax) return qflash_launch_fwd_qmax(a, d, kv_tile, lds, lds_limit, threads, stream);
    return launch_shape<false>(a, d, kv_tile, lds, lds_limit, threads, st);
}
