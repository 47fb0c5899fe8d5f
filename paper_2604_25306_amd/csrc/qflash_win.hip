// gfx950 kernel of the integer-only fused attention forward pass (Algorithm 1) for windowed
// attention: sequences of 33 to 64 tokens with 32 features per head (7 x 7 windows), one KV tile, an
// optional additive bias in the packed layout (relative-position bias, shifted-window mask).
//
// Such a layer is thousands of tiny independent problems (6 KB of Q, K, V, O per pair, but 16 KB of
// bias), so what matters is what is NOT done per pair.  The kernel is persistent: one workgroup of up
// to 16 wavefronts per compute unit, the weight table staged into LDS once per workgroup, and every
// wavefront on its own from then on -- no barrier, no flag, no shared K/V:
//   - a wavefront owns one half of the query rows (rows 0-31 or 32-63) of a run of consecutive
//     pairs.  Pairs are numbered so that a run shares one bias slice (same window position and head
//     in consecutive images); the 32 bias words of the lane stay in registers, already offset, and
//     serve as the accumulator input of the first matrix product: adding the bias costs nothing.
//   - K, V and the wavefront's 32 query rows go to private LDS buffers (5 KiB, two sets,
//     alternating) by direct global-to-LDS loads, one pair ahead of their use, row-major as in
//     memory.  K and Q rows are MFMA operands exactly as they lie there (lane (l % 32, l / 32) reads
//     bytes 16 (l / 32) .. +15 of row l % 32); the V^T operand is read with the transposing 8-bit
//     LDS read.  No staging registers, no transposition in the vector ALU, no LDS write
//     instruction, and nothing in flight that the compiler has to count: the only wait of an
//     iteration is the one at its top.
// Keys beyond the sequence and excluded pairs carry a large negative accumulator input
// (-2^29 before the offset), far below every real score, so they fall out of the maximum and get
// weight 0 without a test.  Scores carry the offset 2^30 (see qflash_tile.h), which turns the
// table index into one saturating subtraction.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <mutex>

#include "qflash_tile.h"

// (M0 is written by the direct loads below and declared as clobbered)
#pragma clang diagnostic ignored "-Winline-asm"

namespace {

extern __shared__ __align__(1024) int8_t smem_win[];

typedef __attribute__((address_space(3))) void* lds_void_w;
typedef const __attribute__((address_space(1))) void* glb_void_w;

// 64 lanes fetch 16 bytes each from g + lane_off; the 1 KiB lands at lds_addr + 16 * lane.
__device__ __forceinline__ void win_load_1k(const int8_t* g /* uniform */, int lane_off, int lds_addr /* uniform */) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(lane_off), "s"((glb_void_w)g) : "memory", "m0");
}

constexpr int kWinSetBytes = 5 * 1024;     // V, K and 32 query rows of one pair
constexpr int kWinExcluded = -(1 << 29);   // stands for "takes no part" in the offset representation

struct WinPair {      // where a run stands: pair t of the launch order
    int s_idx;        // bias slice = wb * bias_H + hb
    int wb, hb;       // batch and head index of the slice inside the bias
    int i, j;         // replica of the slice: batch step, head step
};

template <int XM>
__device__ __forceinline__ void win_body(const QflashKernelArgs& a) {
    constexpr int D = 32;
    constexpr bool KZ = XM == kExpShift0;
    const int N = a.N;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_waves = (int)(blockDim.x >> 6);
    const int g = lane >> 5, li = lane & 31;
    const QflashHeadConsts hc = head_consts_or_dev(a, a.hc[0]);
    const ExpConst c = make_exp_const(hc);

    // ---- LDS: [weight table, a.win_table_lds bytes][wavefront w: two sets of V (2 KiB), K (2 KiB),
    //      Q (1 KiB)]; the dynamic LDS is the only LDS of the kernel, so the table index is its address
    const int lds0 = (int)(size_t)(lds_void_w)smem_win;
    const int tbytes = XM == kExpTable ? a.win_table_lds : 0;
    if (XM == kExpTable) {
        for (int it = wave; it < (tbytes >> 10); it += n_waves)
            win_load_1k((const int8_t*)hc.lut + 1024 * it, 16 * lane, lds0 + 1024 * it);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    __syncthreads();          // the only barrier: the table is in place

    // ---- this wavefront's run of pairs
    const int half = wave & 1;
    const int sid = blockIdx.x * a.win_streams + (wave >> 1);
    const int T = a.B * a.H;
    const int t0 = sid * a.win_chunk, t1 = min(t0 + a.win_chunk, T);
    if ((wave >> 1) >= a.win_streams || t0 >= t1) return;

    const bool has_bias = a.bias != nullptr;
    const int bias_B = has_bias ? a.bias_B : 1, bias_H = has_bias ? a.bias_H : 1;
    const int Rb = a.B / bias_B, Rh = a.H / bias_H;      // replicas of a slice (the host checked divisibility)
    WinPair p;
    {
        const int R = Rb * Rh;
        p.s_idx = t0 / R;
        const int r = t0 - p.s_idx * R;
        p.i = r / Rh;
        p.j = r - p.i * Rh;
        p.wb = p.s_idx / bias_H;
        p.hb = p.s_idx - p.wb * bias_H;
    }
    auto pair_index = [&](const WinPair& q) {            // (batch, head) pair number b * H + h
        return (q.wb + q.i * bias_B) * a.H + q.hb + q.j * bias_H;
    };
    auto advance = [&](WinPair& q) {                     // (divisions only once per run, above)
        if (++q.j == Rh) {
            q.j = 0;
            if (++q.i == Rb) {
                q.i = 0;
                ++q.s_idx;
                if (++q.hb == bias_H) { q.hb = 0; ++q.wb; }
            }
        }
    };

    // ---- per-lane offsets (bytes).  In memory: the two 1 KiB pieces of K and V of a pair and the
    //      1 KiB of this half's query rows, each clamped to the pair's last 16 bytes (what lands in
    //      rows beyond the sequence meets weight 0 or is never stored).  In LDS: operand rows, the
    //      V^T operand.
    const int row = 32 * half + li;
    const int voff0 = min(16 * lane, N * D - 16), voff1 = min(1024 + 16 * lane, N * D - 16);
    const int qoff = min(1024 * half + 16 * lane, N * D - 16);
    const int wbuf = lds0 + tbytes + wave * (2 * kWinSetBytes);
    const int op_lane = 32 * li + 16 * g;
    int v_lane;
    {
        const int li_hi = (lane >> 4) & 1, s = lane & 15, odd = s & 1, jj = s >> 1, aa = jj >> 2, bb = jj & 3;
        v_lane = (8 * aa + 4 * g + bb) * D + 16 * li_hi + 8 * odd;
    }
    const size_t pair_bytes = (size_t)N * D;

    auto issue_loads = [&](const WinPair& q, int parity) {
        const size_t off = (size_t)pair_index(q) * pair_bytes;
        const int set = wbuf + kWinSetBytes * parity;
        win_load_1k(a.K + off, voff0, set + 2048);
        win_load_1k(a.Q + off, qoff, set + 4096);
        win_load_1k(a.K + off, voff1, set + 3072);
        win_load_1k(a.V + off, voff0, set);
        win_load_1k(a.V + off, voff1, set + 1024);
    };

    // ---- accumulator input of the score product: bias (or 0) + 2^30, excluded / beyond the sequence: -2^29 + 2^30
    v16i cb[2];
    auto load_slice = [&](int s_idx) {
        if (has_bias) {
            const int nb = (N + 31) / 32;                               // 2
            const int32_t* base = a.bias + (((size_t)s_idx * nb + half) * nb) * 1024 + 4 * lane;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int a4 = 0; a4 < 4; ++a4) {
                    const v4i w = *(const v4i*)(base + kb * 1024 + a4 * 256);
#pragma unroll
                    for (int b = 0; b < 4; ++b) cb[kb][4 * a4 + b] = max(w[b], kWinExcluded) + kAccBias;
                }
        } else {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    cb[kb][v] = (32 * kb + 8 * (v >> 2) + 4 * g + (v & 3) < N ? 0 : kWinExcluded) + kAccBias;
        }
    };

    // ---- the run.  Loads of a pair are issued one pair ahead; the output of a pair is stored one
    //      pair late, right after the only wait of the iteration, so that neither the loads nor the
    //      store are waited for while they are young.  Pairs of one bias slice form the inner loop:
    //      the accumulator input is invariant there.
    issue_loads(p, 0);
    int parity = 0;
    v4i o_prev = v4i{0, 0, 0, 0};
    size_t o_prev_off = 0;
    bool have_prev = false;
    const unsigned o_lane = (unsigned)(row * D + 16 * g);
    int t = t0;
    while (t < t1) {
        load_slice(p.s_idx);
        const int t_end = min(t1, t + (Rb - p.i) * Rh - p.j);       // pairs of this slice from here on
        for (; t < t_end; ++t) {
            // everything in flight belongs to this pair (or is the store of the one before the last)
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            const size_t o_off = (size_t)pair_index(p) * pair_bytes;
            advance(p);
            if (t + 1 < t1) issue_loads(p, parity ^ 1);
            if (have_prev && row < N) *(v4i*)(a.O + o_prev_off + o_lane) = o_prev;

            // ---- step 1: S^T + bias (two blocks of 32 keys x 32 queries)
            const int set = wbuf + kWinSetBytes * parity;
            const v4i q_cur = *(lds_v4i*)(size_t)(set + 4096 + op_lane);
            v16i s[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const v4i k_cur = *(lds_v4i*)(size_t)(set + 2048 + 1024 * kb + op_lane);
                s[kb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(k_cur, q_cur, cb[kb], 0, 0, 0);
            }
            // ---- steps 2, 3: row maximum (unsigned: every value carries 2^30), never below the initial maximum
            int m_new;
            {
                unsigned mk[2];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    mk[kb] = kb == 0 ? (unsigned)kMInit + (unsigned)kAccBias : 0u;
#pragma unroll
                    for (int a4 = 0; a4 < 4; ++a4) {
                        mk[kb] = max(max(mk[kb], (unsigned)s[kb][4 * a4]), (unsigned)s[kb][4 * a4 + 1]);
                        mk[kb] = max(max(mk[kb], (unsigned)s[kb][4 * a4 + 2]), (unsigned)s[kb][4 * a4 + 3]);
                    }
                }
                const HalfPair hp = both_halves((int)max(mk[0], mk[1]));
                m_new = (int)max((unsigned)hp.x, (unsigned)hp.y);
            }
            // ---- steps 5-7: weights, packed four to a dword (the B operand of the second product), row sum
            v4i pk[2];
            int rowsum = 0;
            if (XM == kExpTable) {
                const unsigned edge = (unsigned)m_new - (unsigned)to_vgpr(hc.lut_xp);
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        s[kb][v] = table_weight(__builtin_elementwise_sub_sat((unsigned)s[kb][v], edge));
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int a4 = 0; a4 < 4; ++a4) {
                        const unsigned w = pack_byte<0>((unsigned)s[kb][4 * a4], (unsigned)s[kb][4 * a4 + 1],
                                                        (unsigned)s[kb][4 * a4 + 2], (unsigned)s[kb][4 * a4 + 3]);
                        pk[kb][a4] = (int)w;
                        rowsum = __builtin_amdgcn_sdot4((int)w, 0x01010101, rowsum, false);
                    }
            } else {
                const int lo = m_new + c.x_floor;
                const int m2 = m_new - 2 * c.s_inv;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int a4 = 0; a4 < 4; ++a4) {
                        unsigned pr[4];
#pragma unroll
                        for (int b = 0; b < 4; ++b) {
                            const int y = shift_exp2<KZ>(max(s[kb][4 * a4 + b], lo), m_new, m2, c);
                            pr[b] = (unsigned)__mul24(y, c.p_mul_hi_v);
                        }
                        const unsigned w = pack_byte3(pr[0], pr[1], pr[2], pr[3]);
                        pk[kb][a4] = (int)w;
                        rowsum = __builtin_amdgcn_sdot4((int)w, 0x01010101, rowsum, false);
                    }
            }
            RowState<D> st;
            {
                const HalfPair hp = both_halves(rowsum);
                st.l = hp.x + hp.y;
            }
            st.m = m_new;
            // ---- step 8: O^T = V^T P^T, the V^T operand read transposed from the row-major V in LDS
            {
                const int vb = set + v_lane;
                v16i acc = offset_block();
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    const v2i_t lo2 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i*)(size_t)(vb + 1024 * kb));
                    const v2i_t hi2 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i*)(size_t)(vb + 1024 * kb + 512));
                    const v4i va = __builtin_shufflevector(lo2, hi2, 0, 1, 2, 3);
                    acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(va, pk[kb], acc, 0, 0, 0);
                }
                st.acc[0] = acc;
            }
            // ---- step 11; the store follows in the next iteration
            normalise_words<D, 16>(st, a.out_round != 0, &o_prev);
            o_prev_off = o_off;
            have_prev = true;
            parity ^= 1;
        }
    }
    if (have_prev && row < N) *(v4i*)(a.O + o_prev_off + o_lane) = o_prev;
}

template <int XM>
__global__ __launch_bounds__(1024) void qflash_fwd_win(const QflashKernelArgs a) {
    if constexpr (XM == kExpAuto) {
        if (head_consts_or_dev(a, a.hc[0]).lut_bytes > 0) win_body<kExpTable>(a);
        else win_body<kExpShift>(a);
    } else {
        win_body<XM>(a);
    }
}

template <int XM>
int launch_win(const QflashKernelArgs& a, size_t lds, int lds_limit, hipStream_t st) {
    auto kern = qflash_fwd_win<XM>;
    // once per process and device: raise the dynamic LDS limit, and make sure that the kernel has no
    // static LDS in front of the dynamic one (the table index is used as an LDS address)
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
    hipLaunchKernelGGL(kern, dim3((unsigned)a.win_groups), dim3((unsigned)(128 * a.win_streams)), lds, st, a);
    return (int)hipGetLastError();
}

}  // namespace

int qflash_launch_fwd_win(const QflashKernelArgs& a, int lds_limit, void* stream) {
    hipStream_t st = (hipStream_t)stream;
    // everything the kernel's indexing assumes, checked once more where it is launched
    if (!a.win_mode || a.N <= 32 || a.N > 64 || a.win_streams < 1 || a.win_streams > 8 || a.win_chunk < 1 || a.win_groups < 1)
        return (int)hipErrorInvalidValue;
    if ((long long)a.win_groups * a.win_streams * a.win_chunk < (long long)a.B * a.H) return (int)hipErrorInvalidValue;
    if (a.bias && (!a.bias_packed || a.bias_B < 1 || a.bias_H < 1 || a.B % a.bias_B != 0 || a.H % a.bias_H != 0))
        return (int)hipErrorInvalidValue;
    if (a.per_head || a.qmax) return (int)hipErrorInvalidValue;
    const bool table = a.exp_mode == kExpTable || a.exp_mode == kExpAuto;
    if (table && a.lut_bytes_max > a.win_table_lds) return (int)hipErrorInvalidValue;
    const size_t lds = qflash_win_lds_bytes(a.win_streams, table ? a.win_table_lds : 0);
    if (lds > (size_t)lds_limit) return (int)hipErrorInvalidValue;
    if (a.exp_mode == kExpAuto) return launch_win<kExpAuto>(a, lds, lds_limit, st);
    if (a.exp_mode == kExpTable) return launch_win<kExpTable>(a, lds, lds_limit, st);
    if (a.exp_mode == kExpShift0) return launch_win<kExpShift0>(a, lds, lds_limit, st);
    return launch_win<kExpShift>(a, lds, lds_limit, st);
}
