// Internal interface between the host side of the C ABI and the gfx950 kernels.
#pragma once
#include <stdint.h>

struct QflashKernelArgs {
    const int8_t* Q;
    const int8_t* K;
    const int8_t* V;
    int8_t* O;
    const int32_t* bias;   // nullptr: no bias
    int bias_B, bias_H;
    int B, H, N;
    // integer constants of Algorithm 1 / 2 (see qflash_params)
    int x_shift, s_inv, exp_mul, p_mul, p_shift, a_mul, out_round;
    // x_floor <= 0: score differences below it are clamped to it.  Chosen on the host so that
    // ShiftExp2 is exactly 0 at and below it, and every 32-bit intermediate is exact above it.
    int x_floor;
    // work decomposition: one unit = (batch*head, query tile); XCD x owns units
    // [x*units_per_xcd, (x+1)*units_per_xcd)
    int rows_per_wg, n_qtiles, n_units, units_per_xcd;
};

// Enqueue the forward kernel for head size d (32|64), KV tile (64|128).  Returns a hipError_t value.
int qflash_launch_fwd(const QflashKernelArgs& args, int d, int kv_tile, int lds_limit, void* stream);

// Choose the kernel variant for a head of N rows and fill rows_per_wg and n_qtiles.
// lds_limit = LDS bytes one workgroup may use on this device.
int qflash_plan_fwd(int N, int d, int kv_tile, int lds_limit, QflashKernelArgs* args);
