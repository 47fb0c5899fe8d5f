// Internal interface between the host side of the C ABI and the gfx950 kernels.
#pragma once
#include <stdint.h>

#include "qflash.h"

// Integer constants of Algorithm 1 / 2 for one head, or for the whole tensor (see qflash_params).
struct QflashHeadConsts {
    int x_shift, s_inv, exp_mul, p_mul, p_shift, a_mul;
    // x_floor <= 0: score differences below it are clamped to it.  Chosen on the host so that
    // ShiftExp2 is exactly 0 at and below it, and every 32-bit intermediate is exact above it.
    int x_floor;
    // look-up mode (resident kernel only): table of int8 weights of these constants
    int lut_xp;              // table index = score - running max + lut_xp, clamped at 0
    int lut_bytes;           // bytes staged into LDS (multiple of 16)
    const uint8_t* lut;      // nullptr = none
};

// Per-head constants travel in the kernel arguments (at most 4 KB in all).
constexpr int kQflashMaxParamHeads = 64;

struct QflashKernelArgs {
    const int8_t* Q;
    const int8_t* K;
    const int8_t* V;
    int8_t* O;
    const int32_t* bias;   // nullptr: no bias
    int bias_B, bias_H;
    int bias_packed;       // bias is in the lane-major layout written by qflash_launch_pack_bias
    int B, H, N;
    int out_round;
    // work decomposition: one unit = (batch*head, query tile); XCD x owns units
    // [x*units_per_xcd, (x+1)*units_per_xcd)
    int rows_per_wg, n_qtiles, n_units, units_per_xcd;
    int xcd_period;          // 0, or the number of units after which the bias slices repeat (a multiple of 8)
    int waves_per_head;      // wavefronts that serve one (batch, head) pair inside a workgroup
    int heads_per_wg;        // > 1 only when a pair fits one workgroup (n_qtiles == 1)
    int same_head;           // heads_per_wg > 1: the pairs of a workgroup are one head of consecutive batch elements
    int resident;            // 1: whole K/V of a head staged in LDS, 0: streamed per KV tile
    int pipelined;           // resident only: K/V tiles are staged one ahead of their use
    int ring;                // pipelined only: LDS holds two KV tiles (in use / being staged), not the whole sequence
    int kv_tile;             // KV tile size the plan was made for
    int n_cu;                // compute units of the device if wave priority alternates by dispatch round, else 0
    // weight mode of the launch (uniform over heads): 2 = every head reads its table,
    // 1 = arithmetic with x_shift == 0 for every head, 0 = arithmetic, 3 = per workgroup: table if the
    // constants of its head have one (lut_bytes > 0), else arithmetic
    int exp_mode;
    int lut_bytes_max;       // LDS bytes reserved for the table: the largest of all heads
    // whole-compute-unit kernel (qflash_plan_cu): 1 if the launch takes it
    int cu_mode;
    int cu_heads;            // (batch, head) pairs per workgroup
    int cu_groups;           // workgroups
    int cu_waves;            // wavefronts per workgroup (at most 16)
    int cu_table_lds;        // LDS bytes reserved for the weight table (a multiple of 1 KiB)
    // two-tile ring fed by direct global-to-LDS loads (d = 64, no bias; set by qflash_plan_fwd): 1 if the launch takes it
    int ring_dma;
    int ring_table_lds;      // LDS bytes reserved for the weight table (a multiple of 1 KiB)
    // windowed-attention kernel (qflash_plan_win): 1 if the launch takes it
    int win_mode;
    int win_streams;         // pairs of wavefronts (one per half of the query rows) per workgroup, at most 8
    int win_chunk;           // consecutive pairs (in slice-major order) each pair of wavefronts works through
    int win_groups;          // workgroups
    int win_table_lds;       // LDS bytes reserved for the weight table (a multiple of 1 KiB)
#ifdef QF_TRACE
    unsigned long long* trace;   // instrumented builds only: [workgroup][wavefront][16] timestamps
#endif
    int qmax;                // 1: the quantised-maximum variant (not Algorithm 1 as printed; every x_shift must be 0)
    int per_head;            // 0: hc[0] serves every head; 1: head h uses hc[h] (H <= kQflashMaxParamHeads)
    // Constants computed on the GPU (dynamic quantisation): if set, the kernel reads this device
    // structure instead of hc[]; exp_mode is then 0 (the host does not know the constants).
    const QflashHeadConsts* hc_dev;
    QflashHeadConsts hc[kQflashMaxParamHeads];
};

// Which unit of work a workgroup takes (host and device: the kernels use it, qflash_plan_unit
// reports it).  Consecutive workgroup indices go to consecutive XCDs (each with its own L2), so XCD
// x = wg % 8 takes the units [x*units_per_xcd, (x+1)*units_per_xcd): neighbouring heads share an
// L2.  With a bias whose slices repeat every xcd_period units (windowed attention: the same windows
// in every image) XCD x instead takes the x-th eighth of every period, so that each L2 only ever
// sees an eighth of the bias.  The result may be >= n_units: such a workgroup has nothing to do.
#if defined(__HIPCC__)
#define QF_UNIT_HD __host__ __device__
#else
#define QF_UNIT_HD
#endif
QF_UNIT_HD inline int qflash_unit_of_workgroup(int wg, int units_per_xcd, int xcd_period) {
    const int x = wg & 7, k = wg >> 3;
    if (xcd_period == 0) return x * units_per_xcd + k;
    const int q = xcd_period >> 3;
    return (k / q) * xcd_period + x * q + k % q;
}

// Wavefronts per workgroup of the resident kernel (short sequences, N <= 256: 8, held to 128
// registers so that two workgroups share a compute unit; longer ones: 12), and of the streamed one.
constexpr int kResidentMaxWavesNarrow = 8;
constexpr int kResidentMaxWavesWide = 12;
constexpr int kStreamWaves = 4;
constexpr int kStreamRows = kStreamWaves * 32;

// Argument checks of the attention entry points (host only).  Returns QFLASH_OK or the error code.
int qflash_check_call(const void* Q, const void* K, const void* V, const void* O, const int32_t* bias, int bias_B,
                      int bias_H, bool bias_packed, int B, int H, int N, int d, int kv_tile, const qflash_params* p,
                      bool per_head, bool consts_on_device, bool qmax);

// LDS bytes of the resident kernel for `heads` pairs of N rows (ring_tile != 0: two KV tiles of that
// size instead of the whole sequence) plus a weight table; 0 if that exceeds lds_limit.  LDS bytes
// of the whole-compute-unit kernel.
size_t qflash_resident_lds_bytes(int N, int d, int heads, int table_bytes, int lds_limit, int ring_tile = 0);
size_t qflash_cu_lds_bytes(int N, int heads, int table_bytes);

// Enqueue the forward kernel for head size d (32|64), KV tile (64|128).  Returns a hipError_t value.
int qflash_launch_fwd(const QflashKernelArgs& args, int d, int kv_tile, int lds_limit, void* stream);
// The same kernels instantiated for the quantised-maximum variant (called by qflash_launch_fwd when args.qmax).
int qflash_launch_fwd_qmax(const QflashKernelArgs& args, int d, int kv_tile, size_t lds_bytes, int lds_limit, int threads, void* stream);

// Choose the kernel variant for BH heads of N rows and fill the work decomposition fields
// (resident, pipelined, ring, ring_dma, rows_per_wg, waves_per_head, heads_per_wg, n_qtiles, n_units, units_per_xcd, xcd_period, same_head; reads bias, bias_B, B, H, per_head).
// Returns non-zero if the launch would be too large.
// lds_limit = LDS bytes one workgroup may use on this device.
int qflash_plan_fwd(int BH, int N, int d, int kv_tile, int lds_limit, QflashKernelArgs* args);   // n_cu is the caller's

// The kernel that gives a whole compute unit to one workgroup (short sequences, 64 features, tile 64,
// no bias, one set of constants): decides whether the launch takes it, assuming a weight table of
// table_bytes (0: none), and fills the cu_* fields.  Reads bias, per_head, n_cu (0: 256).  Returns cu_mode.
int qflash_plan_cu(int BH, int N, int d, int kv_tile, int lds_limit, int table_bytes, QflashKernelArgs* args);
int qflash_launch_fwd_cu(const QflashKernelArgs& args, int lds_limit, void* stream);

// The persistent kernel for windowed attention (33 to 64 tokens, 32 features, one KV tile, no bias or a
// packed bias whose extents divide B and H, one set of constants, Algorithm 1 only): decides whether
// the launch takes it and fills the win_* fields.  Reads bias, bias_packed, bias_B, bias_H, B, H, N,
// per_head, qmax, n_cu (0: 256).  Returns win_mode.
int qflash_plan_win(int d, int kv_tile, int lds_limit, int table_bytes, QflashKernelArgs* args);
int qflash_launch_fwd_win(const QflashKernelArgs& args, int lds_limit, void* stream);
size_t qflash_win_lds_bytes(int streams, int table_bytes);

// The two-tile ring with direct global-to-LDS loads (long sequences, d = 64, no bias, both
// Algorithm 1 and the quantised-maximum variant; work decomposition as for the ring of the resident kernel, four wavefronts per workgroup).
int qflash_launch_fwd_ring(const QflashKernelArgs& args, int lds_limit, void* stream);
size_t qflash_ring_lds_bytes(int waves, int kv_tile, int table_bytes);

// GPUs per process for which per-device launch set-up is remembered.
constexpr int kQflashMaxDevices = 64;

// 1 if the resident kernel can also hold a weight table of table_bytes in LDS and copying it pays.
int qflash_table_fits(const QflashKernelArgs& args, int d, int table_bytes, int lds_limit);

// Enqueue the kernel that fills a weight table of n entries (n_padded bytes) for the constants hc.
int qflash_launch_build_table(uint8_t* tbl, int n, int n_padded, int x_p, const QflashHeadConsts& hc, void* stream);

// Bias in the lane-major layout the kernels read with 16-byte loads: number of 16-byte words for
// `slices` = bias_B * bias_H matrices of N x N, and the kernel that writes them from the plain layout.
long long qflash_packed_bias_words(int slices, int N);
int qflash_launch_pack_bias(const int32_t* bias, int slices, int N, int32_t* packed, void* stream);

// Enqueue the front end of the dynamic pipeline: abs-max of the three float32 tensors of n elements
// each (n a multiple of 4), derivation of the scales and constants into *hc_dev (and *info if not
// null), quantisation into Qo, Ko, Vo.  scratch: 3 * qflash_dynamic_partials(n) device floats.
int qflash_dynamic_partials(long long n);
// table (may be null): room for a weight table of up to table_max bytes; if the table of the
// derived constants fits, the quantising kernel also builds it (one workgroup more, beside the
// streaming ones) and records it in *hc_dev (lut, lut_bytes, lut_xp); lut_bytes == 0 says "none".
int qflash_launch_dynamic_front(const float* Qf, const float* Kf, const float* Vf, int8_t* Qo, int8_t* Ko, int8_t* Vo,
                                long long n, double sqrt_d, int out_round, float* scratch,
                                QflashHeadConsts* hc_dev, qflash_dynamic_info* info, uint8_t* table, int table_max,
                                void* stream);
// Enqueue (after qflash_launch_dynamic_front on the same stream, same scratch and n) the kernel that
// converts a real bias (float32 [slices,N,N] or null) and exclusion mask (uint8, same shape, or
// null) into the packed int32 bias of the scales found by the abs-max step.
int qflash_launch_dynamic_bias(const float* bias, const uint8_t* mask, int slices, int N, int32_t* packed,
                               const float* scratch, long long n, double sqrt_d, void* stream);
