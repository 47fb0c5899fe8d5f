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
//   - K and Q rows are MFMA operands exactly as they lie in memory (lane (l % 32, l / 32) needs
//     bytes 16 (l / 32) .. +15 of row l % 32): they go from global memory straight to registers,
//     one pair ahead of their use.
//   - V goes to a private 2 KiB LDS buffer (two of them, alternating) by direct global-to-LDS
//     loads, row-major as in memory, and the V^T operand is read with the transposing 8-bit LDS
//     read: no transposition in the vector ALU, no LDS write instruction.
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

    // ---- LDS: [weight table, a.win_table_lds bytes][wavefront w: two V buffers of 2 KiB]; the
    //      dynamic LDS is the only LDS of the kernel, so the table index is its address
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

    // ---- per-lane offsets inside a pair (bytes): K rows of the two key blocks, the query row, the
    //      two 1 KiB pieces of V (clamped to the pair's last 16 bytes: what lands in rows beyond the
    //      sequence meets weight 0), the V^T operand in LDS, the output row
    const unsigned koff0 = (unsigned)(min(li, N - 1) * D + 16 * g);
    const unsigned koff1 = (unsigned)(min(32 + li, N - 1) * D + 16 * g);
    const int row = 32 * half + li;
    const unsigned qoff = (unsigned)(min(row, N - 1) * D + 16 * g);
    const int voff0 = min(16 * lane, N * D - 16), voff1 = min(1024 + 16 * lane, N * D - 16);
    const int vbuf = lds0 + tbytes + wave * 4096;
    int v_lane;
    {
        const int li_hi = (lane >> 4) & 1, s = lane & 15, odd = s & 1, jj = s >> 1, aa = jj >> 2, bb = jj & 3;
        v_lane = (8 * aa + 4 * g + bb) * D + 16 * li_hi + 8 * odd;
    }
    const size_t pair_bytes = (size_t)N * D;

    v4i k_cur[2], q_cur, k_nxt[2] = {v4i{0, 0, 0, 0}, v4i{0, 0, 0, 0}}, q_nxt = v4i{0, 0, 0, 0};
    auto issue_loads = [&](const WinPair& q, int parity, v4i* kk, v4i& qq) {
        const size_t off = (size_t)pair_index(q) * pair_bytes;
        const int8_t* Kp = a.K + off;
        const int8_t* Qp = a.Q + off;
        kk[0] = *(const v4i*)(Kp + koff0);
        kk[1] = *(const v4i*)(Kp + koff1);
        qq = *(const v4i*)(Qp + qoff);
        win_load_1k(a.V + off, voff0, vbuf + 2048 * parity);
        win_load_1k(a.V + off, voff1, vbuf + 2048 * parity + 1024);
    };

    // ---- accumulator input of the score product: bias (or 0) + 2^30, excluded / beyond the sequence: -2^29 + 2^30
    v16i cb[2];
    int cur_slice = -1;
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
        cur_slice = s_idx;
    };

    issue_loads(p, 0, k_cur, q_cur);
    int parity = 0;
    for (int t = t0; t < t1; ++t) {
        if (p.s_idx != cur_slice) load_slice(p.s_idx);
        const size_t o_off = (size_t)pair_index(p) * pair_bytes;
        // everything in flight belongs to this pair (and to the stores of the previous one)
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        WinPair pn = p;
        advance(pn);
        if (t + 1 < t1) issue_loads(pn, parity ^ 1, k_nxt, q_nxt);

        // ---- step 1: S^T + bias (two blocks of 32 keys x 32 queries)
        v16i s[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) s[kb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(k_cur[kb], q_cur, cb[kb], 0, 0, 0);
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
            const int vb = vbuf + 2048 * parity + v_lane;
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
        // ---- step 11 and the store
        if (row < N) normalise_store<D, 16>(st, a.O + o_off + (size_t)row * D, g, a.out_round != 0);

        p = pn;
        parity ^= 1;
        k_cur[0] = k_nxt[0];
        k_cur[1] = k_nxt[1];
        q_cur = q_nxt;
    }
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
