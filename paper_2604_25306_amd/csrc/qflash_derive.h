// Derivation and checking of the integer constants of one call (qflash_params) from the real
// scales, written once for the host entry point qflash_params_from_scales and for the device
// kernel that does the same after an on-the-fly quantisation.  Double-precision division and
// the exact operations used here (ldexp, floor, multiplication by powers of two) give the same
// bits on both sides.
#pragma once
#include <math.h>
#include <stdint.h>

#include "qflash.h"
#include "qflash_internal.h"

#if defined(__HIPCC__)
#define QF_HD __host__ __device__
#else
#define QF_HD
#endif

constexpr int kQfXShiftMax = 13;
constexpr int kQfSInvMin = 1 << 10;
constexpr int kQfSInvMax = 1 << 18;  // exclusive

QF_HD inline int64_t qf_round_half_up(double x) { return (int64_t)floor(x + 0.5); }

// Range and consistency checks that make the 32-bit kernel arithmetic exact (see the comments on
// x_floor in qflash_internal.h and on shift_exp2 in the kernel source).
QF_HD inline bool qflash_params_ok(const qflash_params& p) {
    if (p.x_shift < 0 || p.x_shift > kQfXShiftMax) return false;
    if (p.s_inv < kQfSInvMin || p.s_inv >= kQfSInvMax) return false;
    if (p.exp_shift != 32) return false;
    if (p.exp_mul >= 0 || p.exp_mul <= -(1 << 23)) return false;
    // M * s_inv must be -2^32 to within 0.1 %: both come from the same real scale.
    const int64_t prod = (int64_t)p.exp_mul * (int64_t)p.s_inv + ((int64_t)1 << 32);
    if (prod > ((int64_t)1 << 32) / 1000 || prod < -(((int64_t)1 << 32) / 1000)) return false;
    // the kernel multiplies by p_mul << (24 - p_shift), a 24-bit operand, so that P lands in byte 3
    if (p.p_shift < 8 || p.p_shift > 24 || p.p_mul < 1 || ((int64_t)p.p_mul << (24 - p.p_shift)) >= (1 << 23)) return false;
    // 1.0 (= s_inv) must requantise to at most 127 so that P fits a signed byte.
    if ((int64_t)p.s_inv * p.p_mul >= ((int64_t)128 << p.p_shift)) return false;
    if (p.a_mul < 1 || (int64_t)p.s_inv * p.a_mul >= ((int64_t)1 << 31)) return false;
    // alpha = 1.0 must map to exactly 2^16 (identity), i.e. s_inv * a_mul >= 2^30.
    if ((int64_t)p.s_inv * p.a_mul < ((int64_t)1 << 30)) return false;
    if (p.out_round != 0 && p.out_round != 1) return false;
    return true;
}

// Every field of *out from the scales of Q and K and sqrt(d) (Algorithm 1 "Require",
// Algorithm 2, Eq. 9-10).  Returns QFLASH_OK or QFLASH_ERR_PARAM.
QF_HD inline int qflash_derive_params(double sQ, double sK, double sqrt_d, qflash_params* out) {
    if (!(sQ > 0.0) || !(sK > 0.0) || !(sQ <= 1.0e300) || !(sK <= 1.0e300)) return QFLASH_ERR_PARAM;
    // s = sQ * sK * d^(-1/2) * log2(e), evaluated left to right in double (Algorithm 1, Require).
    const double log2e = 1.4426950408889634;
    const double s = ((sQ * sK) / sqrt_d) * log2e;
    if (!(s > 0.0) || !(s <= 1.0e300)) return QFLASH_ERR_PARAM;
    int k = 0;
    while (qf_round_half_up(ldexp(1.0, k) / s) < kQfSInvMin) {
        if (++k > kQfXShiftMax) return QFLASH_ERR_PARAM;
    }
    const double sk = s / ldexp(1.0, k);
    const double inv = 1.0 / sk;
    if (!(inv < 1.0e9)) return QFLASH_ERR_PARAM;
    const int64_t s_inv = qf_round_half_up(inv);                   // Algorithm 2: round(1/s)
    if (s_inv < kQfSInvMin || s_inv >= kQfSInvMax) return QFLASH_ERR_PARAM;
    const int64_t m = qf_round_half_up(-sk * 4294967296.0);        // Algorithm 2: round(-s * 2^N)
    // Eq. 9: n = floor(log2(127/s_inv)) < 0, found with integers: 2^n <= 127/s_inv < 2^(n+1).
    int e = 0;
    while ((int64_t)127 << e < s_inv) ++e;
    const int r = 8 + e;                                           // r = b - n, b = 8
    const int64_t m_r = (2 * ((int64_t)127 << r) + s_inv) / (2 * s_inv);   // Eq. 10: round(127/s_inv*2^r)
    const int64_t a_mul = (((int64_t)1 << 30) + s_inv - 1) / s_inv;
    qflash_params p;
    p.x_shift = k;
    p.s_inv = (int32_t)s_inv;
    p.exp_mul = (int32_t)m;
    p.exp_shift = 32;
    p.p_mul = (int32_t)m_r;
    p.p_shift = r;
    p.a_mul = (int32_t)a_mul;
    p.out_round = 0;
    if (!qflash_params_ok(p)) return QFLASH_ERR_PARAM;
    *out = p;
    return QFLASH_OK;
}

// Kernel-side constants of one set of parameters.  The clamp point of the exponent is the
// smallest multiple of 2^-k at or below -20.5 octaves: above it q <= 28 and every intermediate
// fits 24/32 bits; at and below it the numerator of Algorithm 2 (< 2^20) is shifted right by
// >= 20, so the exact result is 0.  Returns false if the constants put it beyond 28.5 octaves.
QF_HD inline bool qflash_fill_head_consts(const qflash_params& p, QflashHeadConsts* h) {
    h->x_shift = p.x_shift; h->s_inv = p.s_inv; h->exp_mul = p.exp_mul;
    h->p_mul = p.p_mul; h->p_shift = p.p_shift; h->a_mul = p.a_mul;
    const int64_t x0 = (41 * (int64_t)p.s_inv + ((int64_t)2 << p.x_shift) - 1) >> (p.x_shift + 1);
    if ((x0 << p.x_shift) * 2 > 57 * (int64_t)p.s_inv) return false;
    h->x_floor = (int)-x0;
    h->lut = nullptr; h->lut_bytes = 0; h->lut_xp = 0;
    return true;
}
