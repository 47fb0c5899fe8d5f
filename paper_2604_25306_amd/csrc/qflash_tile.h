// Per-tile device code of the integer-only attention forward pass (Algorithm 1, steps 1-11), shared by
// every gfx950 kernel that walks over KV tiles: the operand layout in registers, the element-wise
// integer softmax of one tile, ScaleRelease, the final normalisation.  Included by the kernel
// source files only.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "qflash_internal.h"
#include "qflash_device.h"

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

namespace {

constexpr int kNegBig = -(1 << 30);   // stands for "excluded": far below any clamp point (so is
                                      // anything a saturating add of INT32_MIN produces)
constexpr int kMInit = -(1 << 21);    // initial running maximum (Algorithm 1)

// ------------------------------------------------------------------ scalar building blocks

// The two lanes l and l ^ 32 hold the halves of one query row.  One cross-lane swap in the vector
// ALU (no round trip through the LDS crossbar) hands each of them both values: the swap exchanges
// the upper half of its first operand with the lower half of the second, so with both operands
// equal to v every lane ends up with {own, partner's} in some order -- enough for max and sum.
struct HalfPair { int x, y; };
__device__ __forceinline__ HalfPair both_halves(int v) {
    const auto sw = __builtin_amdgcn_permlane32_swap((unsigned)v, (unsigned)v, false, false);
    return HalfPair{(int)sw[0], (int)sw[1]};
}

// Gather byte 3 of four dwords into one dword (v_perm_b32: selector bytes 0-3 pick from the
// second operand, 4-7 from the first).
__device__ __forceinline__ unsigned pack_byte3(unsigned p0, unsigned p1, unsigned p2, unsigned p3) {
    unsigned w = __builtin_amdgcn_perm(p1, p0, 0x07030703u);   // [p0.3, p1.3, .., ..]
    w = __builtin_amdgcn_perm(p2, w, 0x07070100u);             // [p0.3, p1.3, p2.3, ..]
    return __builtin_amdgcn_perm(p3, w, 0x07020100u);          // [p0.3, p1.3, p2.3, p3.3]
}
template <int BYTE>
__device__ __forceinline__ unsigned pack_byte(unsigned p0, unsigned p1, unsigned p2, unsigned p3) {
    constexpr unsigned b = BYTE, h = BYTE + 4;
    unsigned w = __builtin_amdgcn_perm(p1, p0, (h << 24) | (b << 16) | (h << 8) | b);
    w = __builtin_amdgcn_perm(p2, w, (h << 24) | (h << 16) | 0x0100u);
    return __builtin_amdgcn_perm(p3, w, (h << 24) | 0x020100u);
}

// ScaleRelease with alpha in 16 fractional bits, floor(x * alpha16 / 2^16), 0 <= alpha16 <= 2^16.
//
// Numerator accumulators are kept with an offset, y = x + 2^30 > 0 (the MFMA adds products modulo
// 2^32, so the offset rides along).  With A = alpha16 << 16:
//   mul_hi_u32(y, A) = floor((x A + 2^30 A) / 2^32) = floor(x alpha16 / 2^16) + A/4   (A is a multiple of 4)
// so the rescaled accumulator, again offset by 2^30, is mul_hi_u32(y, A) + (2^30 - A/4): one
// multiply-high and one add, no shift.  alpha16 = 2^16 (identity) does not fit A; there
// A = 2^32 - 1 gives mul_hi_u32(y, A) = y - 1 for every 1 <= y < 2^32, and the addend is 1.
// (|x| < 2^26 always.)  The offset is 2^30 because that bit pattern (the float 2.0) is an inline
// constant of the instruction set: a matrix instruction can start from a block of it without a
// single register being set aside for it.
struct ReleaseConst {
    unsigned A, C;       // accumulator: y <- mul_hi_u32(y, A) + C
    int alpha14;         // alpha16 << 14, for the (unbiased, non-negative) denominator
};
__device__ __forceinline__ ReleaseConst make_release(unsigned alpha16) {
    ReleaseConst r;
    const unsigned one = alpha16 >> 16;   // 1 only for the identity
    r.A = (alpha16 << 16) - one;
    r.C = 0x40000000u - (alpha16 << 14) + one;
    r.alpha14 = (int)(alpha16 << 14);
    return r;
}
__device__ __forceinline__ int release_acc(int y, const ReleaseConst& r) { return (int)(__umulhi((unsigned)y, r.A) + r.C); }
// Denominator: 0 <= l < 2^20, floor(l * alpha16 / 2^16) = ((l << 2) * (alpha16 << 14)) >> 32.
__device__ __forceinline__ int release_l(int l, const ReleaseConst& r) { return __mulhi(l << 2, r.alpha14); }

constexpr int kAccBias = 0x40000000;   // offset carried by numerator accumulators and biased scores
// A result block full of the offset (the compiler turns it into the inline constant).
__device__ __forceinline__ v16i offset_block() {
    v16i z;
#pragma unroll
    for (int v = 0; v < 16; ++v) z[v] = kAccBias;
    return z;
}
// Offset of the biased scores of 32-key block kb of a tile, relative to kAccBias.  A matrix
// instruction takes a constant as its addend only if the constant is one of the few the instruction
// set has built in (here the bit patterns of 2.0, 4.0, 1.0 and 0.5: 2^30, 2^30 + 2^23, 2^30 - 2^23,
// 2^30 - 2^24) and, with this compiler, only if no other instruction shares it; a block of sixteen
// registers filled with the constant costs eight vector and sixteen scalar instructions per tile
// otherwise.  So each block of a tile gets a constant of its own, and the two places that compare
// scores across blocks (the row maximum, the table index) take the difference out again.
__device__ __forceinline__ constexpr int score_offset_delta(int kb) {
    return kb == 0 ? 0 : kb == 1 ? (1 << 23) : kb == 2 ? -(1 << 23) : -(1 << 24);
}
constexpr int kMaskedBiased = 1 << 24;   // a key beyond the sequence, as a biased score at the common offset
template <int KBI>
__device__ __forceinline__ v16i score_offset_block() {
    v16i z;
#pragma unroll
    for (int v = 0; v < 16; ++v) z[v] = kAccBias + score_offset_delta(KBI);
    return z;
}

// One byte of the weight table.  The table is the first thing in the workgroup's LDS (the resident
// kernel has no other LDS object, so its dynamic LDS starts at address 0): the index is the address.
typedef const __attribute__((address_space(3))) uint8_t lds_u8;
__device__ __forceinline__ int table_weight(unsigned idx) { return (int)*(lds_u8*)(size_t)idx; }

// R = ceil(2^(2L+8) / d) for d in (2^(L-1), 2^L], L = 16 or 20, in integer arithmetic only:
// Newton's iteration for 1/d on 32-bit fixed point (32-bit multiply-high is full rate here),
// then one exact remainder step.  With d31 = d << (31-L) in (2^30, 2^31] and x ~ 2^62 / d31:
//   x0 = (48/17 - 32/17 * d31/2^31) * 2^31,   x <- (x * (2^31 - (d31 * x >> 32)) >> 32) << 2   (3 times)
// q = x >> (23-L) is floor((2^(2L+8) - 1) / d) to within +-1 for every d of both ranges (checked by
// enumerating all of them; tests/test_host_logic.py repeats that); the low 32 bits of the remainder
// (2^(2L+8) - 1) - q d decide the correction, and R = q + 1.
template <int L>
__device__ __forceinline__ unsigned recip_ceil(unsigned d) {
    const unsigned d31 = d << (31 - L);
    unsigned x = (3031741621u - __umulhi(4042322161u, d31)) << 1;
#pragma unroll
    for (int it = 0; it < 3; ++it) {
        const unsigned f = 0x80000000u - __umulhi(d31, x);
        x = __umulhi(x, f) << 2;
    }
    unsigned q = x >> (23 - L);
    const int rem = (int)(0xffffffffu - q * d);
    if (rem < 0) q -= 1;
    else if ((unsigned)rem >= d) q += 1;
    return q + 1;
}

// Quantised-maximum variant: the reference level the initial maximum -2^21 rounds up to,
// ceil(-2^21 / s_inv) * s_inv = -floor(2^21 / s_inv) * s_inv (a_mul = ceil(2^30 / s_inv)).
__device__ __forceinline__ int qmax_initial_reference(int s_inv, int a_mul) {
    unsigned q = __umulhi(1u << 23, (unsigned)a_mul);
    if (q * (unsigned)s_inv > (1u << 21)) q -= 1;
    return -(int)(q * (unsigned)s_inv);
}

// ---------------------------------------------------------------------- per-wavefront state

template <int D>
struct RowState {
    v16i acc[D / 32];   // O^T: features 32*t + 8*(v/4) + 4*g + v%4 of this lane's query row
    int l;              // running denominator
    int m;              // running maximum
};

// One KV tile for one wavefront.  sK: K rows of the tile (row pitch KROW), sV: V^T with the tile's
// columns starting at column 0 (row pitch VROW).  n_valid = number of real kv rows in the tile.
// QMAX selects the quantised-maximum variant, which is NOT Algorithm 1 as printed: RowState::m is
// then the reference level (the running maximum rounded up to a multiple of s_inv; x_shift must be
// 0), scores are referred to it, and ScaleRelease is an exact shift.
// XM selects how the int8 weight of a score is obtained: kExpShift (Algorithm 2 + Eq. 10 in the
// ALUs, any x_shift), kExpShift0 (the same, x_shift == 0) or kExpTable (one LDS look-up in a table
// of the same function, see qflash_build_table).
//
// Offsets.  Numerator accumulators always carry +2^30 (see ReleaseConst).  In table mode without
// bias the scores can carry it too (SB): the first MFMA of a score block starts from a
// block of the offset instead of zeros, which costs nothing, and then
//   table index = max(0, s - m + x_p) = (s + 2^30) -sat- (m + 2^30 - x_p)
// is a single unsigned saturating subtraction per score (both operands are positive: |s| < 2^21);
// RowState::m holds m + 2^30.  Algorithm 2 for alpha only sees differences, which are unchanged.
enum { kExpShift = 0, kExpShift0 = 1, kExpTable = 2, kExpAuto = 3 };   // kExpAuto: per workgroup, table if its head has one
// Bias of a kernel variant: none, the plain [N,N] layout, or the lane-major packed layout.
enum { kBiasNone = 0, kBiasPlain = 1, kBiasPacked = 2 };

// Biased scores: wherever the weight comes from the table and there is no bias to add.
template <int D, int BC, int BIAS, bool NARROW, int XM>
constexpr bool score_biased() { return XM == kExpTable && !BIAS; }

template <bool SB>
__device__ __forceinline__ int smax(int a, int b) { return SB ? (int)max((unsigned)a, (unsigned)b) : max(a, b); }
template <bool SB>
__device__ __forceinline__ int smax3(int a, int b, int c) {
    return SB ? (int)max(max((unsigned)a, (unsigned)b), (unsigned)c) : max(max(a, b), c);
}

//
// LAY selects where the MFMA A operands come from.  kLayPadded: K rows with pitch KROW at sK and V^T
// (columns in result order) with pitch VROW at sV, both written by the staging code of the kernel.
// kLaySwizzled: K and V tiles row-major in LDS exactly as in memory (64-byte rows, the four 16-byte
// pieces of row r stored at piece index p ^ ((r >> 2) & 3), which is what keeps both kinds of read
// free of bank conflicts), put there by direct global-to-LDS loads; kx / vx are then this lane's LDS
// byte addresses inside the tile (see swizzled_lane_offsets) and sK, KROW, sV, VROW are unused.
// The V^T operand is read with the transposing 8-bit LDS read of gfx950.
enum { kLayPadded = 0, kLaySwizzled = 1 };

typedef int v2i_t __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) v2i_t lds_v2i;
typedef const __attribute__((address_space(3))) v4i lds_v4i;

// ds_read_b64_tr_b8 works on blocks of 16 lanes: lane i of a block receives, as byte j, byte i % 8 of
// the 8 bytes that lane 2 j + i / 8 of the block points to.  With even lanes pointing at features
// f0..f0+7 and odd lanes at f0+8..f0+15 of key row kappa(j), lane i ends up with feature f0 + i of
// the eight keys kappa(0..7): a 16 x 8 piece of V^T.  Two such reads (keys 16 apart) are the 16
// bytes of the A operand of O^T += V^T P^T, with kappa chosen as the row order of the score block
// (k-slot 16 g + 4 a + b  <->  key 8 a + 4 g + b).
struct SwizzledLane {
    int k_off;   // K / Q operand: row li, 16-byte piece g (k-step 0; k-step 1 is this ^ 32)
    int v_off;   // V^T operand: first transposing read of feature block 0 (block 1 is this ^ 32; keys +16: + 1024)
};
__device__ __forceinline__ SwizzledLane swizzled_lane_offsets(int lane) {
    const int li = lane & 31, g = lane >> 5;
    SwizzledLane o;
    o.k_off = li * 64 + ((g ^ ((li >> 2) & 3)) << 4);
    const int li_hi = (lane >> 4) & 1, s = lane & 15, odd = s & 1, j = s >> 1, a = j >> 2, b = j & 3;
    o.v_off = (8 * a + 4 * g + b) * 64 + ((li_hi ^ ((2 * a + g) & 3)) << 4) + 8 * odd;
    return o;
}

// NG: 0, or the number of groups of 8 keys the (ragged) tile has, known at compile time: the tests
// "does this group exist" then cost nothing; n_valid_rt still tells which keys of the last group exist.
template <int D, int BC, int BIAS, int XM, bool SB, bool FULL, bool FIRST, int LAY = kLayPadded, int NG = 0, bool QMAX = false>
__device__ __forceinline__ void process_tile(RowState<D>& st, const v4i* qreg, const int8_t* sK, int KROW,
                                            const int8_t* sV, int VROW, int n_valid_rt, int x_p,
                                            const int32_t* bias_row /* + c0 */,
                                            const v4i* bpre /* packed bias of this tile already in registers, or null */,
                                            const ExpConst& c, int a_mul, int li, int g,
                                            int kx = 0, int vx = 0) {
    const v16i zb = offset_block();
    static_assert(LAY == kLayPadded || D == 64, "the swizzled layout is for 64-byte rows");
    constexpr int KSTEPS = D / 32, TB = D / 32, KB = BC / 32;
    constexpr bool KZ = XM == kExpShift0;
    static_assert(!SB || (XM == kExpTable && !BIAS), "biased scores: table mode without bias only");
    static_assert(KB <= 4, "one built-in constant per 32-key block");
    // FULL: the tile has all BC kv rows, every "is this group inside the sequence" test below is
    // true at compile time and the tile is one straight line of code.
    static_assert(NG >= 0 && NG <= BC / 8 && !(FULL && NG != 0), "groups of a ragged tile");
    const int n_valid = FULL ? BC : n_valid_rt;
    // does the 32-key block kb / the group a4 of it exist; does that group reach beyond the sequence
    auto blk_on = [&](int kb) { return NG ? 4 * kb < NG : 32 * kb < n_valid; };
    auto grp_on = [&](int kb, int a4) { return NG ? 4 * kb + a4 < NG : 32 * kb + 8 * a4 < n_valid; };
    auto grp_cut = [&](int kb, int a4) { return NG ? 4 * kb + a4 == NG - 1 : 32 * kb + 8 * a4 + 8 > n_valid; };
    // ---- step 1: S^T blocks (32 kv rows x 32 queries each)
    v16i s[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
        if (blk_on(kb)) {
            const v4i ka0 = LAY == kLaySwizzled ? *(lds_v4i*)(size_t)(kx + 2048 * kb)
                                                : *(const v4i*)(sK + (32 * kb + li) * KROW + 16 * g);
            const v16i zs = kb == 0 ? score_offset_block<0>() : kb == 1 ? score_offset_block<1>()
                          : kb == 2 ? score_offset_block<2>() : score_offset_block<3>();
            s[kb] = SB ? __builtin_amdgcn_mfma_i32_32x32x32_i8(ka0, qreg[0], zs, 0, 0, 0)
                       : __builtin_amdgcn_mfma_i32_32x32x32_i8(ka0, qreg[0], v16i{0}, 0, 0, 0);
#pragma unroll
            for (int ks = 1; ks < KSTEPS; ++ks) {
                const v4i ka = LAY == kLaySwizzled ? *(lds_v4i*)(size_t)((kx ^ (32 * ks)) + 2048 * kb)
                                                   : *(const v4i*)(sK + (32 * kb + li) * KROW + 32 * ks + 16 * g);
                s[kb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ka, qreg[ks], s[kb], 0, 0, 0);
            }
        }
    }
    // ---- bias, exclusion and the ragged end of the sequence.  Groups of 4 scores (one result
    //      dword of P) that lie wholly beyond the sequence are skipped everywhere below: the test
    //      32*kb + 8*a4 < n_valid is uniform over the wavefront.
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int a4 = 0; a4 < 4; ++a4) {
            const int cb = 32 * kb + 8 * a4;            // first kv row of the group for g = 0
            if (BIAS == kBiasPacked) {
                // Packed bias: the four values of this lane's group are one 16-byte word, the 64
                // lanes of the wavefront read 1 KiB in a row; columns beyond the sequence hold the
                // exclusion mark already.
                if (grp_on(kb, a4)) {
                    const v4i bv = bpre ? bpre[4 * kb + a4] : *(const v4i*)(bias_row + (4 * kb + a4) * 256);
#pragma unroll
                    for (int b = 0; b < 4; ++b)
                        s[kb][4 * a4 + b] = __builtin_elementwise_add_sat(s[kb][4 * a4 + b], bv[b]);
                }
            } else if (grp_on(kb, a4) && (BIAS || grp_cut(kb, a4))) {
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int col = cb + 4 * g + b;
                    const bool beyond = !FULL && col >= n_valid;
                    int val = s[kb][4 * a4 + b];
                    if (BIAS) {
                        // One saturating add does it all: the exclusion mark INT32_MIN drags the
                        // score to the bottom of the range, below every clamp point, so it drops
                        // out of the maximum and gets weight 0 without a compare and select.
                        // (A builtin, not inline assembly: the compiler must see this read of an MFMA
                        // result to insert the wait states the matrix pipeline needs.)
                        const int bv = beyond ? INT32_MIN : bias_row[col];
                        val = __builtin_elementwise_add_sat(val, bv);
                    } else if (beyond) {
                        // below every real score in either representation (biased: 2^24 at the
                        // common offset, so that taking the block's own offset out cannot wrap)
                        val = SB ? kMaskedBiased + score_offset_delta(kb) : kNegBig;
                    }
                    s[kb][4 * a4 + b] = val;
                }
            }
        }
    // ---- steps 2,3: row maximum over the tile, running maximum
    // (three-operand maxima, one chain per score block so that they can overlap)
    int m_new = st.m;
    {
        int mk[KB];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            mk[kb] = kb == 0 ? st.m : (SB ? kMaskedBiased + score_offset_delta(kb) : INT32_MIN);
#pragma unroll
            for (int a4 = 0; a4 < 4; ++a4)
                if (grp_on(kb, a4)) {
                    mk[kb] = smax3<SB>(mk[kb], s[kb][4 * a4], s[kb][4 * a4 + 1]);
                    mk[kb] = smax3<SB>(mk[kb], s[kb][4 * a4 + 2], s[kb][4 * a4 + 3]);
                }
        }
        m_new = mk[0];
#pragma unroll
        for (int kb = 1; kb < KB; ++kb) {
            if (SB) {
                // (a block that does not exist has no maximum to bring to the common offset)
                if (blk_on(kb)) m_new = smax<SB>(m_new, (int)((unsigned)mk[kb] - (unsigned)score_offset_delta(kb)));
            } else {
                m_new = smax<SB>(m_new, mk[kb]);
            }
        }
    }
    {
        const HalfPair hp = both_halves(m_new);
        m_new = smax<SB>(hp.x, hp.y);
    }
    // ---- QMAX (not Algorithm 1): the reference moves up by whole octaves only.  st.m is the old
    //      reference (a multiple of s_inv, x_shift = 0) and m_new so far the larger of it and the
    //      tile's maximum; n = ceil((m_new - st.m) / s_inv) octaves are added.  The quotient by
    //      multiply-high with ceil(2^30 / s_inv) overshoots by at most one (numerator < 2^24),
    //      which one comparison corrects.
    int n_oct = 0;
    if (QMAX) {
        const unsigned x = ((unsigned)m_new - (unsigned)st.m) + (unsigned)(c.s_inv - 1);
        unsigned q = __umulhi(x << 2, (unsigned)a_mul);
        if (q * (unsigned)c.s_inv > x) q -= 1;
        n_oct = (int)q;
        m_new = st.m + n_oct * c.s_inv;
    }
    const int lo = m_new + c.x_floor;
    const int m2 = m_new - 2 * c.s_inv;
    // ---- step 4: max-offset factor alpha, brought to 16 fractional bits
    ReleaseConst rel;
    if (!FIRST && !QMAX) {
        const int a_hat = shift_exp2<KZ>(smax<SB>(st.m, lo), m_new, m2, c);
        rel = make_release(min(((unsigned)a_hat * (unsigned)a_mul) >> 14, 65536u));
    }
    // ---- steps 9,10 (the part that concerns the past): ScaleRelease of denominator and numerator.
    //      QMAX: alpha = 2^-n, an arithmetic shift; on the offset representation
    //      floor(x / 2^n) + 2^30 = ((x + 2^30) >> n) + (2^30 - (2^30 >> n)) for n <= 30, and n = 30
    //      stands for every larger n (|x| < 2^26).
    auto release_past = [&]() {
        if (QMAX) {
            const int n = min(n_oct, 30);
            const unsigned addc = (unsigned)kAccBias - ((unsigned)kAccBias >> n);
            st.l = st.l >> n;
#pragma unroll
            for (int t = 0; t < TB; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) st.acc[t][v] = (int)(((unsigned)st.acc[t][v] >> n) + addc);
        } else {
            st.l = release_l(st.l, rel);
#pragma unroll
            for (int t = 0; t < TB; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) st.acc[t][v] = release_acc(st.acc[t][v], rel);
        }
    };
    v4i pk[KB];
    int rowsum = 0;
    if (XM == kExpTable) {
        // ---- steps 5,6 by table: issue every look-up of the tile, rescale the accumulators while
        //      the LDS answers, then pack.  Index 0 of the table is the weight 0 of everything at
        //      or below -x_p (excluded scores included).
        const unsigned x_p_v = (unsigned)to_vgpr(x_p);
        const unsigned edge = (unsigned)m_new - x_p_v;       // score_biased: m + 2^30 - x_p > 0
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const unsigned edge_kb = edge + (unsigned)score_offset_delta(kb);   // (the block's own offset)
#pragma unroll
            for (int a4 = 0; a4 < 4; ++a4)
                if (grp_on(kb, a4)) {
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        // Saturating subtractions are fast-class instructions; as builtins, because
                        // they read MFMA results.
                        const unsigned sv = (unsigned)s[kb][4 * a4 + b];
                        const unsigned idx = SB ? __builtin_elementwise_sub_sat(sv, edge_kb)
                                                : __builtin_elementwise_sub_sat(x_p_v, (unsigned)m_new - sv);
                        s[kb][4 * a4 + b] = table_weight(idx);
                    }
                }
        }
        __builtin_amdgcn_sched_barrier(0);
        if (!FIRST) release_past();
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            pk[kb] = v4i{0, 0, 0, 0};
#pragma unroll
            for (int a4 = 0; a4 < 4; ++a4)
                if (grp_on(kb, a4)) {
                    const unsigned w = pack_byte<0>((unsigned)s[kb][4 * a4], (unsigned)s[kb][4 * a4 + 1],
                                                    (unsigned)s[kb][4 * a4 + 2], (unsigned)s[kb][4 * a4 + 3]);
                    pk[kb][a4] = (int)w;
                    rowsum = __builtin_amdgcn_sdot4((int)w, 0x01010101, rowsum, false);   // step 7
                }
        }
        {
            const HalfPair hp = both_halves(rowsum);
            rowsum = hp.x + hp.y;
        }
        st.l += rowsum;                                                                    // step 9
    } else {
        // ---- steps 5,6,7: score intensity, requantisation to int8 (Eq. 10), row sum
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            pk[kb] = v4i{0, 0, 0, 0};
#pragma unroll
            for (int a4 = 0; a4 < 4; ++a4)
                if (grp_on(kb, a4)) {
                    unsigned pr[4];
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const int y = shift_exp2<KZ>(max(s[kb][4 * a4 + b], lo), m_new, m2, c);
                        pr[b] = (unsigned)__mul24(y, c.p_mul_hi_v);       // Eq. 10, result in byte 3
                    }
                    const unsigned w = pack_byte3(pr[0], pr[1], pr[2], pr[3]);
                    pk[kb][a4] = (int)w;
                    rowsum = __builtin_amdgcn_sdot4((int)w, 0x01010101, rowsum, false);
                }
        }
        {
            const HalfPair hp = both_halves(rowsum);
            rowsum = hp.x + hp.y;
        }
        // Keep the phases apart: letting the scheduler overlap the rescale below with the
        // element-wise work above only lengthens live ranges (spills) without gaining issue slots.
        __builtin_amdgcn_sched_barrier(0);
        // ---- steps 9,10: ScaleRelease of the running denominator and numerator
        if (FIRST) {
            st.l = rowsum;
        } else {
            release_past();
            st.l += rowsum;
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    // ---- step 8: O^T += V_j^T P^T (the first tile starts the accumulators at their offset 2^30)
#pragma unroll
    for (int t = 0; t < TB; ++t)
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
            if (blk_on(kb)) {
                v4i va;
                if (LAY == kLaySwizzled) {
                    const int va_addr = (vx ^ (32 * t)) + 2048 * kb;
                    const v2i_t lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i*)(size_t)va_addr);
                    const v2i_t hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i*)(size_t)(va_addr + 1024));
                    va = __builtin_shufflevector(lo, hi, 0, 1, 2, 3);
                } else {
                    va = *(const v4i*)(sV + (32 * t + li) * VROW + 32 * kb + 16 * g);
                }
                st.acc[t] = (FIRST && kb == 0) ? __builtin_amdgcn_mfma_i32_32x32x32_i8(va, pk[kb], zb, 0, 0, 0)
                                               : __builtin_amdgcn_mfma_i32_32x32x32_i8(va, pk[kb], st.acc[t], 0, 0, 0);
            }
    st.m = m_new;
}

// Step 11: integer normalisation floor(O / l) (or nearest), saturated to int8, without a division
// per element.  With u = O + 128 l clamped to [0, 256 l), t = floor(u / l) lies in [0, 255] and
// floor(O / l) saturated to [-128, 127] equals t - 128, i.e. byte t ^ 0x80.  l is normalised to
// l' = l << z in (2^(L-1), 2^L] and R = ceil(2^(2L+8) / l'); then floor(u' R / 2^(2L+8)) is exact
// for every u' < 256 l' because u' (R l' - 2^(2L+8)) < 2^(L+8) 2^L.  L = 16 or 20 puts the quotient
// into byte 1 or 2 of the high product word.  Nearest: floor((2 O + l) / (2 l)), same scheme with
// numerator 2 O + l and denominator 2 l.
// min(max(u, 0), hi) for hi >= 0 as one instruction (the median of three).  u is the result of an
// ordinary vector instruction, not of a matrix instruction, and the output is tied to it (the rules
// for inline assembly next to to_vgpr).
__device__ __forceinline__ int clamp_0(int u, int hi) {
    int r = u;
    asm("v_med3_i32 %0, %0, 0, %1" : "+v"(r) : "v"(hi));
    return r;
}

// normalise_words leaves the lane's contiguous half of the output row (D / 2 bytes: lane g = 0 the
// first half, g = 1 the second) in out[0 .. D/32); normalise_store also writes it.
template <int D, int L>
__device__ __forceinline__ void normalise_words(const RowState<D>& st, bool round_nearest, v4i* out) {
    constexpr int TB = D / 32;
    static_assert(L == 16 || L == 20, "quotient must be byte aligned");
    const int rs = round_nearest ? 1 : 0;
    const bool empty = st.l == 0;
    const unsigned dsafe = empty ? 1u : ((unsigned)st.l << rs);
    const int z = L - (32 - __clz((int)(dsafe - 1)));          // dsafe << z in (2^(L-1), 2^L]
    const unsigned dn = dsafe << z;
    const unsigned R = recip_ceil<L>(dn);
    const int u_max = (int)(256u * dn) - 1;
    const int zz = z + rs;
    // The accumulators carry their offset (ReleaseConst); it is taken out, modulo 2^32, together
    // with the addition of 128 l.
    int bias_z = (int)(((128u * dsafe + (round_nearest ? (unsigned)st.l : 0u)) << z) - ((unsigned)kAccBias << zz));
    asm volatile("" : "+v"(bias_z));     // (kept as one addend: otherwise the offset is subtracted from every element first)
    // word[j]: features 8 j + 4 g + (0..3) of this lane's row, j = 4 t + a4
    unsigned word[4 * TB];
#pragma unroll
    for (int t = 0; t < TB; ++t)
#pragma unroll
        for (int a4 = 0; a4 < 4; ++a4) {
            unsigned hi[4];
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                int u = (st.acc[t][4 * a4 + b] << zz) + bias_z;
                u = clamp_0(u, u_max);
                hi[b] = __umulhi((unsigned)u, R);
            }
            const unsigned w = pack_byte<(2 * L + 8 - 32) / 8>(hi[0], hi[1], hi[2], hi[3]) ^ 0x80808080u;
            word[4 * t + a4] = empty ? 0u : w;
        }
    // The two lanes of a row hold alternate dwords of it.  Swapping the second half of the row of
    // lane g = 0 against the first half of lane g = 1 (one cross-lane swap per dword) leaves each
    // lane with one contiguous half of the row, written with 16-byte stores: dword-sized stores
    // scattered over 32 rows per instruction cost more time than the whole computation.
    constexpr int HALF = 2 * TB;   // dwords a lane owns after the swap (as many as before it)
    unsigned ev[HALF], od[HALF];   // even / odd dwords of this lane's half
#pragma unroll
    for (int j = 0; j < HALF; ++j) {
        const auto sw = __builtin_amdgcn_permlane32_swap(word[j], word[HALF + j], false, false);
        ev[j] = sw[0];
        od[j] = sw[1];
    }
#pragma unroll
    for (int q = 0; q < HALF / 2; ++q)
        out[q] = v4i{(int)ev[2 * q], (int)od[2 * q], (int)ev[2 * q + 1], (int)od[2 * q + 1]};
}

template <int D, int L>
__device__ __forceinline__ void normalise_store(const RowState<D>& st, int8_t* Orow, int g, bool round_nearest) {
    v4i w[D / 32];
    normalise_words<D, L>(st, round_nearest, w);
    int8_t* dst = Orow + g * (D / 2);
#pragma unroll
    for (int q = 0; q < D / 32; ++q) *(v4i*)(dst + 16 * q) = w[q];
}


// Constants of the head that (batch, head) pair bh belongs to.  bh is uniform over the wavefront,
// so these are scalar loads from the kernel arguments.
// With dynamic quantisation they were computed on the GPU and live in device memory: read field
// by field into scalar registers (selecting between the two structures by pointer would turn every
// access, the table loads included, into generic-address loads).
__device__ __forceinline__ QflashHeadConsts head_consts_or_dev(const QflashKernelArgs& a, QflashHeadConsts h) {
    if (a.hc_dev) {
        const int* g = (const int*)a.hc_dev;     // x_shift, s_inv, exp_mul, p_mul, p_shift, a_mul, x_floor
        h.x_shift = __builtin_amdgcn_readfirstlane(g[0]);
        h.s_inv = __builtin_amdgcn_readfirstlane(g[1]);
        h.exp_mul = __builtin_amdgcn_readfirstlane(g[2]);
        h.p_mul = __builtin_amdgcn_readfirstlane(g[3]);
        h.p_shift = __builtin_amdgcn_readfirstlane(g[4]);
        h.a_mul = __builtin_amdgcn_readfirstlane(g[5]);
        h.x_floor = __builtin_amdgcn_readfirstlane(g[6]);
        // the table, if the GPU built one for these constants (lut_bytes == 0: none)
        h.lut_xp = __builtin_amdgcn_readfirstlane(g[7]);
        h.lut_bytes = __builtin_amdgcn_readfirstlane(g[8]);
        const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane(g[10]), hi = (unsigned)__builtin_amdgcn_readfirstlane(g[11]);
        h.lut = (const uint8_t*)(((unsigned long long)hi << 32) | lo);
    }
    return h;
}
__device__ __forceinline__ QflashHeadConsts head_consts(const QflashKernelArgs& a, int bh) {
    return head_consts_or_dev(a, a.hc[a.per_head ? bh % a.H : 0]);
}
static_assert(offsetof(QflashHeadConsts, x_floor) == 24 && offsetof(QflashHeadConsts, lut_xp) == 28 &&
              offsetof(QflashHeadConsts, lut_bytes) == 32 && offsetof(QflashHeadConsts, lut) == 40,
              "field order read by head_consts");

}  // namespace
