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

// LDS bytes of the resident kernel: K and V^T of `heads` heads of N rows (ring: of two KV tiles)
// and the weight table; 0 if they do not fit.
// Table size assumed when deciding whether two workgroups with the whole sequence in LDS fit a compute unit.
constexpr int kRingTableGuess = 32 * 1024;

static size_t resident_lds_bytes(int N, int d, int heads, int table_bytes, int lds_limit, int ring_tile = 0) {
    const size_t npad = (size_t)((N + 31) & ~31);
    const size_t kv = ring_tile ? 2 * ((size_t)ring_tile * (size_t)(d + 16) + (size_t)d * (size_t)(ring_tile + 16))
                                : npad * (size_t)(d + 16) + (size_t)d * (npad + 16);
    const size_t bytes = (size_t)heads * kv + (size_t)table_bytes;
    return bytes <= (size_t)lds_limit ? bytes : 0;
}

int qflash_plan_fwd(int BH, int N, int d, int kv_tile, int lds_limit, QflashKernelArgs* a) {
    a->resident = resident_lds_bytes(N, d, 1, 0, lds_limit) != 0;
    a->heads_per_wg = 1;
    a->pipelined = 0;
    a->ring = 0;
    a->kv_tile = kv_tile;
    // Long sequences: K and V^T of the whole sequence (plus a weight table) would leave room for
    // one workgroup per compute unit, or for none.  Where the kernel variant can stage tile by
    // tile (d = 64, tile 64), LDS holds two tiles only and workgroups are at most 8 wavefronts,
    // so that two of them share a compute unit.
    const bool two_fit = resident_lds_bytes(N, d, 1, kRingTableGuess, lds_limit / 2) != 0;
    if (d == 64 && N > 256 && (kv_tile == 128 || !two_fit)) {
        const int nblk = (N + 31) / 32;
        const int cus = a->n_cu > 0 ? a->n_cu : 256;
        int waves;
        if (kv_tile == 128) {
            // 160-odd registers leave three wavefront slots per SIMD: three workgroups of four
            // wavefronts (which is also what stages a tile: 256 threads, two items each)
            waves = 4;
        } else {
            // Workgroups of up to 8 wavefronts (two per compute unit: 128 registers leave four
            // wavefront slots per SIMD) or of 4 (four per compute unit, one wavefront on every SIMD,
            // but every wavefront then also stages K/V): whichever gives the busiest compute unit
            // fewer workgroups to run one after the other.
            const int tiles8 = (nblk + 7) / 8, tiles4 = (nblk + 3) / 4;
            const long long turns8 = ((long long)BH * tiles8 + 2ll * cus - 1) / (2ll * cus);
            const long long turns4 = ((long long)BH * tiles4 + 4ll * cus - 1) / (4ll * cus);
            int tiles = turns4 < turns8 ? tiles4 : tiles8;
            if ((nblk + tiles - 1) / tiles < 4) tiles = tiles8;   // staging needs 256 threads
            waves = (nblk + tiles - 1) / tiles;                   // balanced: 4..8
        }
        a->resident = 1;
        a->ring = 1;
        a->pipelined = 1;
        a->rows_per_wg = 32 * waves;
        a->waves_per_head = waves;
    } else if (a->resident) {
        const int nblk = (N + 31) / 32;
        const int max_waves = N <= 256 ? resident_max_waves<true>() : resident_max_waves<false>();
        const int tiles = (nblk + max_waves - 1) / max_waves;
        const int waves = (nblk + tiles - 1) / tiles;       // balanced
        a->rows_per_wg = 32 * waves;
        a->waves_per_head = waves;
        // Short sequences (windowed attention): several (batch, head) pairs per workgroup, so that
        // a workgroup is 8 wavefronts and a weight table is staged once for all of them.
        if (tiles == 1 && waves <= 4) {
            int hp = resident_max_waves<true>() / waves;
            if (hp > BH) hp = BH;
            while (hp > 1 && resident_lds_bytes(N, d, hp, 0, lds_limit / 4) == 0) --hp;
            a->heads_per_wg = hp;
        }
        // Tile-by-tile staging needs a second KV tile to overlap with and 256 staging threads
        // (32-byte pieces of K plus 4x8 blocks of V of one tile, one or two items per thread).
        a->pipelined = a->heads_per_wg == 1 && N > kv_tile && waves >= 4;
    } else {
        a->rows_per_wg = kStreamRows;
        a->waves_per_head = kStreamWaves;
    }
    a->n_qtiles = (N + a->rows_per_wg - 1) / a->rows_per_wg;
    // per-head constants with several pairs per workgroup: group by head (see the kernel)
    a->same_head = a->per_head && a->heads_per_wg > 1 ? 1 : 0;
    const long long units = a->same_head ? (long long)((a->B + a->heads_per_wg - 1) / a->heads_per_wg) * a->H
                            : a->heads_per_wg > 1 ? ((long long)BH + a->heads_per_wg - 1) / a->heads_per_wg
                                                  : (long long)BH * a->n_qtiles;
    if (units >= (1ll << 30)) return -1;
    a->n_units = (int)units;
    a->units_per_xcd = (a->n_units + 7) / 8;
    // Bias slices repeat every bias_B * H pairs: see qflash_unit_of_workgroup.
    a->xcd_period = 0;
    if (a->bias) {
        const long long pairs = (long long)a->bias_B * a->H;
        const long long period = a->same_head ? (a->bias_B % a->heads_per_wg == 0 ? pairs / a->heads_per_wg : 0)
                                 : a->heads_per_wg > 1 ? (pairs % a->heads_per_wg == 0 ? pairs / a->heads_per_wg : 0)
                                                       : pairs * a->n_qtiles;
        if (period >= 8 && period % 8 == 0 && period <= units) {
            a->xcd_period = (int)period;
            a->units_per_xcd = (int)(((units + period - 1) / period) * (period / 8));
        }
    }
    return 0;
}

int qflash_table_fits(const QflashKernelArgs& a, int d, int table_bytes, int lds_limit) {
    // Every workgroup copies the table from L2 into its LDS: worth it only while that stays below
    // the bytes of Q, K, V, O the workgroup moves anyway.
    const long long io = 4ll * a.heads_per_wg * a.N * d;
    if (io < (long long)table_bytes) return 0;
    // keep two workgroups per CU when the sequence is short enough for that to matter
    const int budget = (a.ring || a.N <= 256) ? lds_limit / 2 : lds_limit;
    return resident_lds_bytes(a.N, d, a.heads_per_wg, table_bytes, budget, a.ring ? a.kv_tile : 0) != 0;
}

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

long long qflash_packed_bias_words(int slices, int N) {
    const long long nb = (N + 31) / 32;
    return (long long)slices * nb * nb * 256;
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
    const size_t lds = a.resident ? resident_lds_bytes(a.N, d, a.heads_per_wg, (a.exp_mode == kExpTable || a.exp_mode == kExpAuto) ? a.lut_bytes_max : 0,
                                                       lds_limit, a.ring ? kv_tile : 0) : 0;
    if (a.resident && lds == 0) return (int)hipErrorInvalidValue;
    const int threads = a.resident ? 64 * a.waves_per_head * a.heads_per_wg : kStreamThreads;
    if (a.qmax) return qflash_launch_fwd_qmax(a, d, kv_tile, lds, lds_limit, threads, stream);
    return launch_shape<false>(a, d, kv_tile, lds, lds_limit, threads, st);
}
