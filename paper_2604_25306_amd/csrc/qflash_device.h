// Device-side scalar building blocks of Algorithm 2 / Eq. 10, shared by every gfx950 source file
// that needs the int8 weight of a score difference (the attention kernels, the table builders).
// One definition, so that the arithmetic mode, the tables built from host constants and the
// table built on the GPU cannot disagree.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qflash_internal.h"

namespace {

// (a * b) >> 32 for operands that fit 24 signed bits: one full-rate v_mul_hi_i32_i24.
__device__ __forceinline__ int mulhi24(int a, int b) {
    const int a24 = (a << 8) >> 8, b24 = (b << 8) >> 8;
    return (int)(((long long)a24 * (long long)b24) >> 32);
}

// Loop-invariant constants of Algorithm 2 / Eq. 10 kept in registers.
struct ExpConst {
    int k, s_inv, x_floor;   // uniform (scalar registers)
    int M_v;                 // exp_mul, in a vector register
    int two_s_inv_v;         // 2 * s_inv, in a vector register
    int p_mul_hi_v;          // p_mul << (24 - p_shift): the requantised weight lands in byte 3
};

// Inline assembly and the matrix pipeline.  A matrix instruction writes its 16 result registers
// dozens of cycles after it issues, and the compiler inserts the idle cycles that a later vector
// instruction touching one of them needs -- for the instructions it emits itself, not for the text
// of an assembly statement.  Two rules keep every statement in these files clear of that window:
//   - no operand of a statement is a matrix result (results are read by ordinary code first);
//   - a statement never has a vector register as a pure output.  A pure output may be given any
//     free register, and a result register whose value happens to be unused (the key groups of a
//     ragged tile beyond the sequence) counts as free while the matrix instruction that will still
//     write it is in flight: the late write then destroys the statement's result.  An output tied
//     to an input ("+v") sits in a register that holds a live value, which cannot be one of those.

// Copy a uniform value into a vector register and keep it there: on this chip a two-operand
// multiply / max / shift with a scalar source issues slower than with two vector sources.  (The
// copy itself is the compiler's; the empty statement only hides where the value came from.)
__device__ __forceinline__ int to_vgpr(int v) {
    int r = v;
    asm volatile("" : "+v"(r));
    return r;
}

// Algorithm 2 for a score t already clamped from below to (m + x_floor).
//   x' = (t - m) << k,  q = (x' * M) >> 32,  r = x' + q * s_inv,  y = ((r >> 1) + s_inv) >> q.
// (r >> 1) + s_inv = floor((r + 2 s_inv) / 2) and nested floors of divisions by powers of two
// compose, so y = (r + 2 s_inv) >> (q + 1).  In the clamped range x' fits 24 bits, 0 <= q <= 28
// and r + 2 s_inv is positive, so the logical shift is exact.
// KZ (k == 0): x' = t - m and x' + 2 s_inv = t - (m - 2 s_inv) are two cheap subtractions.
template <bool KZ>
__device__ __forceinline__ int shift_exp2(int t, int m, int m2 /* m - 2 s_inv */, const ExpConst& c) {
    int xs, xs2;
    if (KZ) {
        xs = t - m;
        xs2 = t - m2;
    } else {
        const int neg_m = -m;
        xs = t;                                      // (output tied to an input, see above)
        asm("v_add_lshl_u32 %0, %0, %1, %2" : "+v"(xs) : "v"(neg_m), "s"(c.k));
        xs2 = xs + c.two_s_inv_v;
    }
    const int q = mulhi24(xs, c.M_v);
    const int r2 = __mul24(q, c.s_inv) + xs2;
    return (int)((unsigned)r2 >> (q + 1));
}

__device__ __forceinline__ ExpConst make_exp_const(const QflashHeadConsts& h) {
    ExpConst c;
    c.k = h.x_shift; c.s_inv = h.s_inv; c.x_floor = h.x_floor;
    c.M_v = to_vgpr(h.exp_mul);
    c.two_s_inv_v = to_vgpr(2 * h.s_inv);
    c.p_mul_hi_v = to_vgpr(h.p_mul << (24 - h.p_shift));
    return c;
}

// The int8 weight (Algorithm 2 + Eq. 10) of the score difference x = i - x_p: entry i of the
// weight table of the constants h (c = make_exp_const(h)).  Differences below x_floor weigh 0
// like x_floor itself.
__device__ __forceinline__ unsigned table_entry(int i, int x_p, const QflashHeadConsts& h, const ExpConst& c) {
    const int x = max(i - x_p, h.x_floor);
    const int y = shift_exp2<false>(x, 0, -2 * h.s_inv, c);
    return ((unsigned)__mul24(y, c.p_mul_hi_v)) >> 24;
}

}  // namespace
