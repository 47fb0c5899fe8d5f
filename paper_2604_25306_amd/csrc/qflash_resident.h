// The kernels that walk over KV tiles with K and V^T staged through LDS by the wavefronts themselves
// (resident: whole sequence or a two-tile ring in LDS; stream: one tile at a time, any length), and
// their launchers, as templates.  Two translation units instantiate them: one for Algorithm 1 as
// printed, one for the quantised-maximum variant (QMAX, see process_tile).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <mutex>

#include "qflash_internal.h"
#include "qflash_device.h"
#include "qflash_tile.h"

namespace {

// 4x4 byte transpose: rows r[0..3] (byte f = feature f) -> o[f] = (r0.f, r1.f, r2.f, r3.f).
// v_perm_b32 picks result bytes from the 8 bytes {first operand (4..7), second operand (0..3)}.
__device__ __forceinline__ void transpose4x4(const unsigned r[4], unsigned o[4]) {
    const unsigned t0 = __builtin_amdgcn_perm(r[1], r[0], 0x05010400u);
    const unsigned t1 = __builtin_amdgcn_perm(r[1], r[0], 0x07030602u);
    const unsigned t2 = __builtin_amdgcn_perm(r[3], r[2], 0x05010400u);
    const unsigned t3 = __builtin_amdgcn_perm(r[3], r[2], 0x07030602u);
    o[0] = __builtin_amdgcn_perm(t2, t0, 0x05040100u);
    o[1] = __builtin_amdgcn_perm(t2, t0, 0x07060302u);
    o[2] = __builtin_amdgcn_perm(t3, t1, 0x05040100u);
    o[3] = __builtin_amdgcn_perm(t3, t1, 0x07060302u);
}

// V rows [r0, r0+4) x features [8*t8, 8*t8+8) -> V^T in LDS, kv columns in result-layout order.
// lds_col_blk = LDS column where the 32-row kv block of r0 starts; r_in_blk = r0 % 32 (multiple of 4).
// Split into the global loads and the transposing LDS writes so that the loads of the next KV
// tile can be in flight while the current one is being processed.
typedef int v2i __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void load_v_4x8(const int8_t* Vh, int D, int N, int r0, int t8, v2i rw[4]) {
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        rw[b] = v2i{0, 0};
        if (r0 + b < N) rw[b] = *(const v2i*)(Vh + (size_t)(r0 + b) * D + 8 * t8);
    }
}
__device__ __forceinline__ void store_v_4x8(const v2i rw[4], int t8, int8_t* sV, int VROW, int lds_col_blk, int r_in_blk) {
    // kv row 8*a4 + 4*g2 + b of a block  ->  slot 16*g2 + 4*a4 + b
    const int pos = lds_col_blk + 16 * ((r_in_blk >> 2) & 1) + 4 * (r_in_blk >> 3);
#pragma unroll
    for (int w = 0; w < 2; ++w) {
        const unsigned r[4] = {(unsigned)rw[0][w], (unsigned)rw[1][w], (unsigned)rw[2][w], (unsigned)rw[3][w]};
        unsigned o[4];
        transpose4x4(r, o);
#pragma unroll
        for (int f = 0; f < 4; ++f) *(unsigned*)(sV + (8 * t8 + 4 * w + f) * VROW + pos) = o[f];
    }
}
__device__ __forceinline__ void stage_v_4x8(const int8_t* Vh, int D, int N, int r0, int t8, int8_t* sV, int VROW,
                                            int lds_col_blk, int r_in_blk) {
    v2i rw[4];
    load_v_4x8(Vh, D, N, r0, t8, rw);
    store_v_4x8(rw, t8, sV, VROW, lds_col_blk, r_in_blk);
}

// ------------------------------------------------------------------------ resident kernel

extern __shared__ __align__(16) int8_t smem[];

// Wavefronts per workgroup.  Short sequences (N <= 256) need at most 8; the kernel is then held to
// 128 registers so that two workgroups share a CU.  Longer sequences get up to 12 wavefronts of
// up to 168 registers (the 32-bit rescale and wider tiles need more live values).
template <bool NARROW>
constexpr int resident_max_waves() { return NARROW ? kResidentMaxWavesNarrow : kResidentMaxWavesWide; }

// Where this lane's bias values start.  Plain layout [bias_B,bias_H,N,N]: the lane's row (lanes
// beyond the sequence read row 0; their results are never stored).  Packed layout
// [bias_B*bias_H][ceil(N/32) row blocks][ceil(N/32) column blocks][4 groups][64 lanes][4]: the
// 16-byte word of lane (li, g) in group a4 of column block cb holds
// bias[32*rb + li][32*cb + 8*a4 + 4*g + 0..3], which is exactly what the lane adds to its four
// scores of that group, so one instruction of the wavefront reads 1 KiB in a row.
__device__ __forceinline__ const int32_t* bias_lane_base(const QflashKernelArgs& a, int bh, int row0, int i,
                                                        int li, int g) {
    const int b = bh / a.H, h = bh % a.H, N = a.N;
    const size_t slice = (size_t)(b % a.bias_B) * a.bias_H + (size_t)(h % a.bias_H);
    if (a.bias_packed) {
        const int nb = (N + 31) / 32;
        return a.bias + ((slice * nb + (size_t)min(row0 / 32, nb - 1)) * nb) * 1024 + 4 * (32 * g + li);
    }
    return a.bias + slice * N * N + (size_t)(i < N ? i : 0) * N;
}

template <int D, int BC, int BIAS, bool NARROW, int XM, bool QMAX>
__device__ __forceinline__ void resident_body(const QflashKernelArgs& a) {
    constexpr int KSTEPS = D / 32;
    constexpr int KROW = D + 16;
    const int N = a.N;
    const int npad = (N + 31) & ~31;
    // a.ring: LDS holds two KV tiles (the one in use and the one being staged) instead of the whole
    // sequence, so that long sequences leave room for a second workgroup on the compute unit.
    const bool ring = a.ring != 0;
    const int VROW = (ring ? BC : npad) + 16;
    // A workgroup serves heads_per_wg consecutive (batch, head) pairs when one pair needs only a
    // few wavefronts (windowed attention): wavefront w belongs to pair w / waves_per_head.  Each
    // pair's K and V^T are staged by its own wavefronts; the weight table is shared.
    // LDS: [weight table, lut_bytes (table mode only)] then per pair [K: npad x KROW] [V^T: D x VROW].
    // The table sits at offset 0 so that its index is the LDS address.
    const int tbytes = XM == kExpTable ? a.lut_bytes_max : 0;   // LDS reserved for the table

    const int wg = blockIdx.x;
    const int unit = qflash_unit_of_workgroup(wg, a.units_per_xcd, a.xcd_period);
    if (unit >= a.n_units) return;
    // Workgroups are handed out in index order, one per compute unit and round.  In a launch of
    // only a few rounds, alternating the wave priority by round puts a newcomer ahead of the older
    // workgroup it shares the unit with: the newcomer is the one the end of the launch waits for.
    // (Only a hint: correctness does not depend on placement.  With many rounds it starves every
    // other workgroup and costs time, so the host switches it off there.)
    if (a.n_cu > 0) {
        if ((wg / a.n_cu) & 1) __builtin_amdgcn_s_setprio(0);
        else __builtin_amdgcn_s_setprio(3);
    }

    const int wg_tid = threadIdx.x, wg_nthr = blockDim.x;
    const int lane = wg_tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(wg_tid >> 6);   // uniform: index math on the scalar unit
    const int g = lane >> 5, li = lane & 31;
    const int sub = a.heads_per_wg > 1 ? wave / a.waves_per_head : 0;   // which pair of this workgroup
    const int tid = wg_tid - sub * a.waves_per_head * 64;    // thread index within the pair
    const int nthr = a.waves_per_head * 64;
    const int qt = a.heads_per_wg > 1 ? 0 : unit % a.n_qtiles;
    // Several pairs per workgroup: consecutive pairs, or (a.same_head, per-head constants) the same
    // head of heads_per_wg consecutive batch elements, so that one weight table serves them all.
    int bh = unit / a.n_qtiles;
    bool pair_valid = bh < a.B * a.H;
    if (a.heads_per_wg > 1) {
        if (a.same_head) {
            const int b = (unit / a.H) * a.heads_per_wg + sub;
            bh = b * a.H + unit % a.H;
            pair_valid = b < a.B;
        } else {
            bh = unit * a.heads_per_wg + sub;
            pair_valid = bh < a.B * a.H;
        }
    }
    // A wavefront whose pair does not exist (the last workgroup of a launch) still helps staging the
    // weight table, so it must read the constants of the workgroup's head: it stands in for batch
    // element 0 of that head (pair 0 where all pairs share one set of constants anyway).
    const int bh_safe = pair_valid ? bh : a.same_head ? unit % a.H : 0;
    const QflashHeadConsts hc = head_consts(a, bh_safe);
    const int row0 = qt * a.rows_per_wg + (wave - sub * a.waves_per_head) * 32;
    const int i = row0 + li;

    const int k_rows = ring ? 2 * BC : npad;                 // K rows held in LDS
    int8_t* sK = smem + tbytes + (size_t)sub * ((size_t)k_rows * KROW + (size_t)D * VROW);
    int8_t* sV = sK + (size_t)k_rows * KROW;                // ring: two V^T slots of D x VROW each

    const size_t head_off = (size_t)bh_safe * N * D;
    const int8_t* Qh = a.Q + head_off;
    const int8_t* Kh = a.K + head_off;
    const int8_t* Vh = a.V + head_off;

    // ---- K (row-major) and V^T (permuted columns) of this pair go to LDS either all at once, or
    //      (a.pipelined) one KV tile at a time: the global loads of tile j+1 are issued before tile
    //      j is processed and written to LDS after it, so that memory latency and the first pass
    //      over HBM overlap with the arithmetic instead of preceding it.  Every tile has its own
    //      LDS region, so one barrier per tile (publishing it) is all the synchronisation needed.
    // (compiled in only where the kernel variant has the registers for the tile in flight)
    constexpr bool PIPE_OK = D == 64 && (BC == 64 || !NARROW);
    const bool pipelined = PIPE_OK && a.pipelined != 0;
    const int n_tiles = (N + BC - 1) / BC;
    // One staging item per thread and tile: 32 bytes of a K row, or a 4-row x 8-feature block of
    // V; either way four 8-byte loads, issued without any branch around them (rows beyond the
    // sequence read row N-1 and are zeroed when written to LDS): straight-line loads are what
    // lets the compiler count exactly which of them a later wait has to cover.
    // kv_tile 128 has twice the items: there every staging thread takes one K item and one V item
    // (256 threads, i.e. the first four wavefronts, stage a whole tile whatever the workgroup size).
    constexpr int PASSES = BC == 128 ? 2 : 1;
    v2i pf[4 * PASSES], pf0[4 * PASSES];   // tile in flight; tile 0 (prologue only)
    const int n_full = N / BC, rem = N - n_full * BC;
    const int tid_ = tid;
    // A full tile (all BC rows inside the sequence) needs no clamping, its item count is a
    // compile-time constant and the item of a thread sits at the same offset in every tile, so
    // its four addresses are a uniform base (head, tile) plus a per-thread constant plus a
    // multiple of a uniform step: a dozen instructions where the general computation (the last
    // tile of a ragged sequence) takes fifty.
    constexpr int NKF = BC * (D / 32);    // K items of a full tile
    // (Both lambdas derive their addresses from a copy of the thread index that the compiler
    // cannot see through: otherwise it hoists every loop-invariant piece of address arithmetic
    // out of the KV loop and pays for it with registers held across all the tile code.)
    auto load_tile = [&](int j, v2i* pf) {
        const int c0 = j * BC;
        int tid = tid_;
        asm volatile("" : "+v"(tid));
        const bool full = j < n_full;                           // uniform
        const int rows_t = full ? BC : min(BC, npad - c0);
        const int nK = rows_t * (D / 32), nV = (rows_t / 4) * (D / 8);
        typedef const __attribute__((address_space(1))) int8_t* gptr;
        if constexpr (PASSES == 2) {
            // nK == nV (d = 64): thread t < nK takes K item t and V item t
            if (__builtin_amdgcn_readfirstlane(tid) < nK) {
                gptr p[8];
                const unsigned vrow = 4u * ((unsigned)tid / (D / 8)), vcol = 8u * ((unsigned)tid % (D / 8));
                if (full) {
                    gptr bk = (gptr)Kh + (size_t)c0 * D + 32u * (unsigned)tid;
                    gptr bv = (gptr)Vh + (size_t)c0 * D + (vrow * D + vcol);
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        p[b] = bk + 8 * b;
                        p[4 + b] = bv + D * b;
                    }
                } else {
                    const int krow = min(c0 + tid / (D / 32), N - 1);
                    gptr bk = (gptr)Kh + (size_t)krow * D + 32 * (tid % (D / 32));
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        p[b] = bk + 8 * b;
                        p[4 + b] = (gptr)Vh + (size_t)min(c0 + (int)vrow + b, N - 1) * D + vcol;
                    }
                }
#pragma unroll
                for (int b = 0; b < 8; ++b) pf[b] = *(const __attribute__((address_space(1))) v2i*)p[b];
            }
        } else
        if (__builtin_amdgcn_readfirstlane(tid) < nK + nV) {   // whole wavefronts, nK + nV is a multiple of 64
            // Only the addresses differ between the two kinds of tile; the four loads themselves
            // are one sequence on every path (loads in different branches would end in different
            // registers, and the copies that reconcile them would have to wait for the data).
            // (global address space spelled out: through the merge of the two computations the
            // compiler would otherwise lose it and fall back to generic-address loads)
            gptr p[4];
            if (full) {
                const bool is_k = __builtin_amdgcn_readfirstlane(tid) < NKF;        // uniform
                const unsigned iv = (unsigned)(tid - NKF);
                const unsigned off = is_k ? 32u * (unsigned)tid : 4u * (iv / (D / 8)) * D + 8u * (iv % (D / 8));
                gptr base = (gptr)(is_k ? Kh : Vh) + (size_t)c0 * D + off;
                const int step = is_k ? 8 : D;
#pragma unroll
                for (int b = 0; b < 4; ++b) p[b] = base + b * step;
            } else {
                const bool is_k = tid < nK;
                const int iv = tid - nK;
                gptr base = (gptr)(is_k ? Kh : Vh);
                const int row = c0 + (is_k ? tid / (D / 32) : 4 * (iv / (D / 8)));
                const int col = is_k ? 32 * (tid % (D / 32)) : 8 * (iv % (D / 8));
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int rb = min(is_k ? row : row + b, N - 1);
                    p[b] = base + (size_t)rb * D + col + (is_k ? 8 * b : 0);
                }
            }
#pragma unroll
            for (int b = 0; b < 4; ++b) pf[b] = *(const __attribute__((address_space(1))) v2i*)p[b];
        }
    };
    auto write_tile = [&](int j, const v2i* pf) {
        const int c0 = j * BC;
        int tid = tid_;
        asm volatile("" : "+v"(tid));
        const int rows_t = min(BC, npad - c0);
        const int nK = rows_t * (D / 32), nV = (rows_t / 4) * (D / 8);
        if constexpr (PASSES == 2) {
            if (__builtin_amdgcn_readfirstlane(tid) < nK) {
                const int l0 = ring ? (j & 1) * BC : c0;
                {
                    const int rt = tid / (D / 32), h = tid % (D / 32);
                    v4i lo = {pf[0][0], pf[0][1], pf[1][0], pf[1][1]}, hi = {pf[2][0], pf[2][1], pf[3][0], pf[3][1]};
                    if (!(c0 + rt < N)) lo = hi = v4i{0, 0, 0, 0};
                    *(v4i*)(sK + (l0 + rt) * KROW + 32 * h) = lo;
                    *(v4i*)(sK + (l0 + rt) * KROW + 32 * h + 16) = hi;
                }
                {
                    const int rt = 4 * (tid / (D / 8));
                    v2i rw[4];
#pragma unroll
                    for (int b = 0; b < 4; ++b) rw[b] = c0 + rt + b < N ? pf[4 + b] : v2i{0, 0};
                    int8_t* sVt = ring ? sV + (size_t)(j & 1) * D * VROW : sV;
                    store_v_4x8(rw, tid % (D / 8), sVt, VROW, (ring ? rt : c0 + rt) & ~31, rt & 31);
                }
            }
        } else
        if (__builtin_amdgcn_readfirstlane(tid) < nK + nV) {
            // LDS position of sequence row c0: its own place, or the start of ring slot j % 2
            const int l0 = ring ? (j & 1) * BC : c0;
            if (__builtin_amdgcn_readfirstlane(tid) < nK) {
                const int rt = tid / (D / 32), h = tid % (D / 32);
                v4i lo = {pf[0][0], pf[0][1], pf[1][0], pf[1][1]}, hi = {pf[2][0], pf[2][1], pf[3][0], pf[3][1]};
                if (!(c0 + rt < N)) lo = hi = v4i{0, 0, 0, 0};
                *(v4i*)(sK + (l0 + rt) * KROW + 32 * h) = lo;
                *(v4i*)(sK + (l0 + rt) * KROW + 32 * h + 16) = hi;
            } else {
                const int iv = tid - nK;
                const int rt = 4 * (iv / (D / 8));
                v2i rw[4];
#pragma unroll
                for (int b = 0; b < 4; ++b) rw[b] = c0 + rt + b < N ? pf[b] : v2i{0, 0};
                int8_t* sVt = ring ? sV + (size_t)(j & 1) * D * VROW : sV;
                store_v_4x8(rw, iv % (D / 8), sVt, VROW, (ring ? rt : c0 + rt) & ~31, rt & 31);
            }
        }
    };
    // Order of the prologue: the loads with the longest way to go first (K/V tile 0 from HBM), then
    // the query rows, then the table (L2); all of them are in flight together and the first wait
    // covers them all.
    if (pipelined) {                        // N > BC: tile 0 is a full one
        load_tile(0, pf0);
        load_tile(1, pf);
    }
    // ---- this lane's query row.  Lanes beyond the sequence read the last row instead (their
    //      results are never stored and rows do not interact), which keeps the loads free of branches.
    v4i qreg[KSTEPS];
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) qreg[s] = *(const v4i*)(Qh + (size_t)min(i, N - 1) * D + 32 * s + 16 * g);
    // ---- packed bias of the first tile (short head size only, where the registers are there):
    //      fetched here, beside K, V and Q, its way through the cache hierarchy is over when the
    //      barrier opens, instead of starting then.  Column blocks wholly beyond the sequence do not
    //      exist in the packed layout and are skipped (the tile code skips them too).
    const int32_t* bias_row = nullptr;
    constexpr bool bias_packed = BIAS == kBiasPacked;
    if (BIAS) bias_row = bias_lane_base(a, bh_safe, row0, i, li, g);
    constexpr bool BPRE_OK = bias_packed && D == 32 && BC == 64;
    v4i bpre[BPRE_OK ? 4 * (BC / 32) : 1];
    if (BPRE_OK) {
#pragma unroll
        for (int q = 0; q < 4 * (BC / 32); ++q)
            if (32 * (q / 4) < N) bpre[q] = *(const v4i*)(bias_row + q * 256);
    }
    // ---- loop-invariant registers, set up before any K/V tile is in flight
    const ExpConst c = make_exp_const(hc);
    constexpr bool SB = score_biased<D, BC, BIAS, NARROW, XM>();
    RowState<D> st;
    st.l = 0;
    const int m_init = QMAX ? qmax_initial_reference(hc.s_inv, hc.a_mul) : kMInit;
    st.m = SB ? (int)((unsigned)m_init + (unsigned)kAccBias) : m_init;

    // ---- stage the weight table (L2-resident, shared by every workgroup of the launch): six
    //      16-byte pieces per thread in flight at a time, which covers the largest table in one
    //      round trip for a workgroup of seven wavefronts (a second round for a few left-over
    //      pieces would cost every wavefront another L2 latency at the barrier)
    if (XM == kExpTable) {
        constexpr int TB_ = 6;
        const int nch = hc.lut_bytes / 16;
        for (int ch0 = wg_tid; ch0 < nch; ch0 += TB_ * wg_nthr) {
            v4i t[TB_];
#pragma unroll
            for (int u = 0; u < TB_; ++u)
                if (ch0 + u * wg_nthr < nch) t[u] = *(const v4i*)(hc.lut + 16 * (ch0 + u * wg_nthr));
#pragma unroll
            for (int u = 0; u < TB_; ++u)
                if (ch0 + u * wg_nthr < nch) *(v4i*)(smem + 16 * (ch0 + u * wg_nthr)) = t[u];
        }
    }
    if (!pipelined) {
        for (int ch = tid; ch < npad * (D / 16); ch += nthr) {
            const int r = ch / (D / 16), c16 = ch % (D / 16);
            v4i val = {0, 0, 0, 0};
            if (r < N) val = *(const v4i*)(Kh + (size_t)r * D + 16 * c16);
            *(v4i*)(sK + r * KROW + 16 * c16) = val;
        }
        for (int sb = tid; sb < (npad / 4) * (D / 8); sb += nthr) {
            const int t8 = sb % (D / 8), r0 = 4 * (sb / (D / 8));
            stage_v_4x8(Vh, D, N, r0, t8, sV, VROW, r0 & ~31, r0 & 31);
        }
    }
    // Touch the query registers here, on every path, where the loads so far have to be waited for
    // anyway.  Otherwise their first use sits inside the tile code, which wavefronts without rows
    // skip, and the compiler has to assume at every later tile that the query load may still be
    // pending; loads complete in order, so that wait would cover the K/V tile in flight as well.
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) asm volatile("" : "+v"(qreg[s]));
    if (BPRE_OK) {
#pragma unroll
        for (int q = 0; q < 4 * (BC / 32); ++q)
            if (32 * (q / 4) < N) asm volatile("" : "+v"(bpre[q]));
    }
    if (pipelined) write_tile(0, pf0);
    __syncthreads();
    // A wavefront without query rows leaves after the only barrier, unless it still has tiles to
    // stage for the others.
    const bool active = row0 < N && pair_valid;
    if (!active && !pipelined) return;

    // First tile (no rescale), the remaining full tiles as one straight-line loop body, then the
    // ragged tile if the sequence does not end on a tile boundary.
    // With a packed bias the keys beyond the sequence carry the exclusion mark (and K, V are zero
    // there), so a last tile whose every 32-key block exists in the packed layout runs the
    // straight-line code of a full tile instead of testing each group of keys.
    const bool ragged_as_full = bias_packed && rem > BC - 32;
#define QF_TILE(FULL_, FIRST_, J_, NV_)                                                                      \
    if (active)                                                                                              \
    process_tile<D, BC, BIAS, XM, SB, FULL_, FIRST_, kLayPadded, 0, QMAX>(st, qreg,                                               \
                                                     sK + (size_t)(ring ? (J_) & 1 : (J_)) * BC * KROW, KROW, \
                                                     ring ? sV + (size_t)((J_) & 1) * D * VROW : sV + (J_) * BC, \
                                                     VROW, NV_, hc.lut_xp,                                   \
                                                     BIAS ? bias_row + (J_) * (bias_packed ? BC * 32 : BC) : nullptr, \
                                                     (BPRE_OK && (FIRST_)) ? bpre : nullptr,                 \
                                                     c, hc.a_mul, li, g)
    // Pipelined mode, around tile j: tile j+1 (loaded while tile j-1 was processed) goes to LDS and
    // the loads of tile j+2 are issued before the arithmetic of tile j; the barrier after it
    // publishes tile j+1, which every wavefront wrote long before.
#define QF_PRE(J_)                                                                                           \
    if (pipelined && (J_) + 1 < n_tiles) {                                                                   \
        write_tile((J_) + 1, pf);                                                                            \
        if ((J_) + 2 < n_tiles) load_tile((J_) + 2, pf);                                                     \
    }
#define QF_POST(J_)                                                                                          \
    if (pipelined && (J_) + 1 < n_tiles) __syncthreads();
    if (n_full > 0) {
        QF_PRE(0)
        QF_TILE(true, true, 0, BC);
        QF_POST(0)
        for (int j = 1; j < n_full; ++j) {
            QF_PRE(j)
            QF_TILE(true, false, j, BC);
            QF_POST(j)
        }
        if (rem > 0) {
            if (ragged_as_full) { QF_TILE(true, false, n_full, BC); }
            else { QF_TILE(false, false, n_full, rem); }
        }
    } else {
        if (ragged_as_full) { QF_TILE(true, true, 0, BC); }
        else { QF_TILE(false, true, 0, rem); }
    }
#undef QF_TILE
#undef QF_PRE
#undef QF_POST
    if (!active) return;
    if (i >= N) return;
    int8_t* Orow = a.O + head_off + (size_t)i * D;
    if (NARROW) normalise_store<D, 16>(st, Orow, g, a.out_round != 0);
    else normalise_store<D, 20>(st, Orow, g, a.out_round != 0);
}

// Wavefronts per SIMD the register allocation has to allow.  Short sequences (NARROW): 4, and 6
// for d = 32 with kv_tile 64 (windowed attention: 80 registers, three workgroups of eight
// wavefronts per compute unit) -- except that its variants that hold the 32 prefetched words of a
// packed bias and compute weights arithmetically spill at 80 registers and run a fifth faster at
// 96 (5 per SIMD).  Long sequences: 4 with kv_tile 64 (the two-tile ring counts on four slots),
// 3 with kv_tile 128.
template <int D, int BC, int BIAS, bool NARROW, int XM>
constexpr int resident_min_waves() {
    if (!NARROW) return BC == 64 ? 4 : 3;
    if (D == 32 && BC == 64) return (BIAS == kBiasPacked && XM != kExpTable) ? 5 : 6;
    return 4;
}

// The kernel: one weight mode for the whole launch, or (kExpAuto: per-head constants of which only
// some have a table that fits, or constants and table made on the GPU) chosen per workgroup from
// the constants of its head.  The choice is uniform over the workgroup, so each workgroup runs
// exactly one of the two bodies.
template <int D, int BC, int BIAS, bool NARROW, int XM, bool QMAX>
__global__ __launch_bounds__(64 * resident_max_waves<NARROW>(), (resident_min_waves<D, BC, BIAS, NARROW, XM>())) void qflash_fwd_resident(const QflashKernelArgs a) {
    if constexpr (XM == kExpAuto) {
        const int unit = qflash_unit_of_workgroup(blockIdx.x, a.units_per_xcd, a.xcd_period);
        if (unit >= a.n_units) return;
        // any pair of the workgroup: all of them share one head when the constants are per head
        const int bh = a.heads_per_wg > 1 ? (a.same_head ? unit % a.H : 0) : unit / a.n_qtiles;
        if (head_consts(a, bh).lut_bytes > 0) resident_body<D, BC, BIAS, NARROW, kExpTable, QMAX>(a);
        else resident_body<D, BC, BIAS, NARROW, kExpShift, QMAX>(a);
    } else {
        resident_body<D, BC, BIAS, NARROW, XM, QMAX>(a);
    }
}

// -------------------------------------------------------------------------- stream kernel

constexpr int kStreamThreads = kStreamWaves * 64;

template <int D, int BC, int BIAS, bool QMAX>
__global__ __launch_bounds__(kStreamThreads) void qflash_fwd_stream(const QflashKernelArgs a) {
    constexpr bool NARROW = false;   // long sequences only
    constexpr int KSTEPS = D / 32;
    constexpr int KROW = D + 16;
    constexpr int VROW = BC + 16;
    __shared__ __align__(16) int8_t sK[BC * KROW];
    __shared__ __align__(16) int8_t sV[D * VROW];

    const int wg = blockIdx.x;
    const int unit = qflash_unit_of_workgroup(wg, a.units_per_xcd, a.xcd_period);
    if (unit >= a.n_units) return;
    const int qt = unit % a.n_qtiles;
    const int bh = unit / a.n_qtiles;
    const int N = a.N;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 5, li = lane & 31;
    const int row0 = qt * kStreamRows + wave * 32;
    const int i = row0 + li;
    const bool wave_active = row0 < N;

    const size_t head_off = (size_t)bh * N * D;
    const int8_t* Qh = a.Q + head_off;
    const int8_t* Kh = a.K + head_off;
    const int8_t* Vh = a.V + head_off;
    const int32_t* bias_row = nullptr;
    constexpr bool bias_packed = BIAS == kBiasPacked;
    if (BIAS) bias_row = bias_lane_base(a, bh, row0, i, li, g);
    v4i qreg[KSTEPS];
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) {
        qreg[s] = v4i{0, 0, 0, 0};
        if (i < N) qreg[s] = *(const v4i*)(Qh + (size_t)i * D + 32 * s + 16 * g);
    }
    const QflashHeadConsts hc = head_consts(a, bh);
    const ExpConst c = make_exp_const(hc);
    RowState<D> st;
    st.l = 0;
    st.m = QMAX ? qmax_initial_reference(hc.s_inv, hc.a_mul) : kMInit;

    const int Tc = (N + BC - 1) / BC;
    for (int j = 0; j < Tc; ++j) {
        const int c0 = j * BC;
        if (j > 0) __syncthreads();   // everyone is done reading the previous tile
        for (int ch = tid; ch < BC * (D / 16); ch += kStreamThreads) {
            const int r = ch / (D / 16), c16 = ch % (D / 16);
            v4i val = {0, 0, 0, 0};
            if (c0 + r < N) val = *(const v4i*)(Kh + (size_t)(c0 + r) * D + 16 * c16);
            *(v4i*)(sK + r * KROW + 16 * c16) = val;
        }
        for (int sb = tid; sb < (BC / 4) * (D / 8); sb += kStreamThreads) {
            const int t8 = sb % (D / 8), r0 = 4 * (sb / (D / 8));
            stage_v_4x8(Vh, D, N, c0 + r0, t8, sV, VROW, r0 & ~31, r0 & 31);
        }
        __syncthreads();
        if (!wave_active) continue;   // uniform per wavefront; still takes part in the barriers
        const int n_valid = min(BC, N - c0);
        const int32_t* brow = BIAS ? bias_row + (bias_packed ? c0 * 32 : c0) : nullptr;
        if (j == 0)
            process_tile<D, BC, BIAS, kExpShift, false, false, true, kLayPadded, 0, QMAX>(st, qreg, sK, KROW, sV, VROW, n_valid, 0, brow, nullptr, c, hc.a_mul, li, g);
        else if (n_valid == BC)
            process_tile<D, BC, BIAS, kExpShift, false, true, false, kLayPadded, 0, QMAX>(st, qreg, sK, KROW, sV, VROW, BC, 0, brow, nullptr, c, hc.a_mul, li, g);
        else
            process_tile<D, BC, BIAS, kExpShift, false, false, false, kLayPadded, 0, QMAX>(st, qreg, sK, KROW, sV, VROW, n_valid, 0, brow, nullptr, c, hc.a_mul, li, g);
    }
    if (!wave_active || i >= N) return;
    int8_t* Orow = a.O + head_off + (size_t)i * D;
    if (NARROW) normalise_store<D, 16>(st, Orow, g, a.out_round != 0);
    else normalise_store<D, 20>(st, Orow, g, a.out_round != 0);
}

// ------------------------------------------------------------------------------ launchers

template <int D, int BC, int BIAS, bool NARROW, int XM, bool QMAX>
int launch_resident(const QflashKernelArgs& a, size_t lds_bytes, int lds_limit, int threads, hipStream_t stream) {
    const dim3 grid((unsigned)(8 * a.units_per_xcd));
    auto kern = qflash_fwd_resident<D, BC, BIAS, NARROW, XM, QMAX>;
    // once per process and device: raise the dynamic LDS limit of this kernel, and make sure that it
    // has no static LDS in front of the dynamic one (the index into the weight table is used as an
    // LDS address)
    static std::once_flag once[kQflashMaxDevices];
    static int status[kQflashMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kQflashMaxDevices) return (int)hipErrorInvalidDevice;
    std::call_once(once[dev], [&] {
        hipFuncAttributes fa;
        hipError_t e = hipFuncGetAttributes(&fa, (const void*)kern);
        if (e == hipSuccess && fa.sharedSizeBytes != 0) e = hipErrorInvalidValue;
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_limit);
        status[dev] = (int)e;
    });
    if (status[dev] != 0) return status[dev];
    hipLaunchKernelGGL(kern, grid, dim3((unsigned)threads), lds_bytes, stream, a);
    return (int)hipGetLastError();
}

template <int D, int BC, int BIAS, bool NARROW, bool QMAX>
int launch_mode(const QflashKernelArgs& a, size_t lds, int lds_limit, int threads, hipStream_t st) {
    if (a.exp_mode == kExpAuto) return launch_resident<D, BC, BIAS, NARROW, kExpAuto, QMAX>(a, lds, lds_limit, threads, st);
    if (a.exp_mode == kExpTable) return launch_resident<D, BC, BIAS, NARROW, kExpTable, QMAX>(a, lds, lds_limit, threads, st);
    if (a.exp_mode == kExpShift0) return launch_resident<D, BC, BIAS, NARROW, kExpShift0, QMAX>(a, lds, lds_limit, threads, st);
    return launch_resident<D, BC, BIAS, NARROW, kExpShift, QMAX>(a, lds, lds_limit, threads, st);
}

template <int D, int BC, int BIAS, bool QMAX>
int launch_dbc_bias(const QflashKernelArgs& a, bool resident, size_t lds, int lds_limit, int threads, hipStream_t st) {
    if (!resident) {
        const dim3 grid((unsigned)(8 * a.units_per_xcd));
        hipLaunchKernelGGL((qflash_fwd_stream<D, BC, BIAS, QMAX>), grid, dim3(kStreamThreads), 0, st, a);
        return (int)hipGetLastError();
    }
    return a.N <= 256 ? launch_mode<D, BC, BIAS, true, QMAX>(a, lds, lds_limit, threads, st)
                      : launch_mode<D, BC, BIAS, false, QMAX>(a, lds, lds_limit, threads, st);
}

template <int D, int BC, bool QMAX>
int launch_dbc(const QflashKernelArgs& a, bool resident, size_t lds, int lds_limit, int threads, hipStream_t st) {
    if (!a.bias) return launch_dbc_bias<D, BC, kBiasNone, QMAX>(a, resident, lds, lds_limit, threads, st);
    return a.bias_packed ? launch_dbc_bias<D, BC, kBiasPacked, QMAX>(a, resident, lds, lds_limit, threads, st)
                         : launch_dbc_bias<D, BC, kBiasPlain, QMAX>(a, resident, lds, lds_limit, threads, st);
}

// d and kv_tile to template arguments.
template <bool QMAX>
int launch_shape(const QflashKernelArgs& a, int d, int kv_tile, size_t lds, int lds_limit, int threads, hipStream_t st) {
    if (d == 64 && kv_tile == 64) return launch_dbc<64, 64, QMAX>(a, a.resident, lds, lds_limit, threads, st);
    if (d == 64 && kv_tile == 128) return launch_dbc<64, 128, QMAX>(a, a.resident, lds, lds_limit, threads, st);
    if (d == 32 && kv_tile == 64) return launch_dbc<32, 64, QMAX>(a, a.resident, lds, lds_limit, threads, st);
    if (d == 32 && kv_tile == 128) return launch_dbc<32, 128, QMAX>(a, a.resident, lds, lds_limit, threads, st);
    return (int)hipErrorInvalidValue;
}

}  // namespace
