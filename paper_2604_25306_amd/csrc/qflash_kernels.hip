// gfx950 (CDNA4) kernels of the integer-only fused attention forward pass (Algorithm 1).
//
// Work decomposition
//   One workgroup = 4 wavefronts = one (batch, head) and 128 consecutive query rows; each
//   wavefront owns 32 query rows for the whole kernel.  KV tiles of B_c rows are staged through
//   LDS once per workgroup and shared by its four wavefronts.
//
// Operand layout (the point of the design)
//   Both products are computed transposed on the 32x32x32 int8 MFMA:
//       S^T = K_j Q_i^T        (A = K rows, B = Q rows)          -> C[kv][query]
//       O^T = V_j^T P^T        (A = V^T rows, B = P^T)           -> C[t][query]
//   In the MFMA result layout lane l holds column (l % 32) and 16 rows, so every lane owns ONE
//   query row: 16 of each 32 scores of that row (the other 16 sit in lane l^32), its running
//   maximum, denominator and alpha, and 16 of each 32 output features.  The row maximum and row
//   sum are 15 in-lane operations plus a single exchange with lane l^32, alpha is a per-lane
//   scalar, and the four dwords of int8 weights a lane produces are, unchanged, its B operand of
//   the second product: P never leaves registers.  The price is that the k-slots of that operand
//   enumerate the kv rows in result-layout order (8*(j/4) + 4*(l/32) + j%4), so V^T is written to
//   LDS with its columns in exactly that order.  Integer addition is associative, so the order of
//   the contraction does not change a single bit of the result.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qflash_internal.h"

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

namespace {

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kRowsPerWave = 32;
constexpr int kRowsPerWg = kWaves * kRowsPerWave;
constexpr int kNegBig = -(1 << 30);   // stands for "excluded": far below any clamp point
constexpr int kMInit = -(1 << 21);    // initial running maximum (Algorithm 1)

// (a * b) >> 32 for operands that fit 24 signed bits: one full-rate v_mul_hi_i32_i24.
__device__ __forceinline__ int mulhi24(int a, int b) {
    const int a24 = (a << 8) >> 8, b24 = (b << 8) >> 8;
    return (int)(((long long)a24 * (long long)b24) >> 32);
}

// Algorithm 2 for an argument already clamped to [x_floor, 0].  With x' = x << k:
//   q = (x' * M) >> 32,  r = x' + q * s_inv,  y = ((r >> 1) + s_inv) >> q.
// (r >> 1) + s_inv = floor((r + 2 s_inv) / 2) and nested floors of divisions by powers of two
// compose, so y = (r + 2 s_inv) >> (q + 1).  In the clamped range x' fits 24 bits, 0 <= q <= 28
// and r + 2 s_inv is positive, so the logical shift is exact.
__device__ __forceinline__ int shift_exp2(int x, const QflashKernelArgs& a) {
    const int xs = x << a.x_shift;
    const int q = mulhi24(xs, a.exp_mul);
    const int r2 = __mul24(q, a.s_inv) + xs + 2 * a.s_inv;
    return (int)((unsigned)r2 >> (q + 1));
}

// Eq. 10: int32 -> [0,127].  y <= s_inv and s_inv * p_mul < 128 << p_shift (checked on the host).
__device__ __forceinline__ int requant(int y, const QflashKernelArgs& a) {
    return (int)((unsigned)__mul24(y, a.p_mul) >> a.p_shift);
}

// ScaleRelease with alpha in 16 fractional bits: floor(x * alpha16 / 2^16).
__device__ __forceinline__ int scale_release(int x, int alpha16) {
    return (int)(((long long)x * (long long)alpha16) >> 16);
}

__device__ __forceinline__ int floor_div_pos(int a, int b) {   // b > 0
    int q = a / b;
    if (a - q * b < 0) q -= 1;
    return q;
}

__device__ __forceinline__ int xor32(int v) { return __shfl_xor(v, 32, 64); }

template <int D, int BC, bool BIAS>
__global__ __launch_bounds__(kThreads) void qflash_fwd_kernel(const QflashKernelArgs a) {
    constexpr int KSTEPS = D / 32;   // 32-wide steps of the Q.K contraction
    constexpr int TB = D / 32;       // 32-row blocks of O^T
    constexpr int KB = BC / 32;      // 32-row kv blocks of one KV tile
    constexpr int KROW = D + 16;     // LDS row pitch of the K tile in bytes (pad against conflicts)
    constexpr int VROW = BC + 16;    // LDS row pitch of the transposed V tile
    __shared__ __align__(16) int8_t sK[BC * KROW];
    __shared__ __align__(16) int8_t sV[D * VROW];

    // XCD-aware placement: workgroup ids are dealt round-robin to the 8 XCDs, so XCD x gets the
    // ids congruent to x; give it a contiguous range of units so that the query tiles of one head
    // meet in one L2.
    const int wg = blockIdx.x;
    const int unit = (wg & 7) * a.units_per_xcd + (wg >> 3);
    if (unit >= a.n_units) return;
    const int qt = unit % a.n_qtiles;
    const int bh = unit / a.n_qtiles;
    const int N = a.N;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int g = lane >> 5;          // which half of the k-slots / result rows this lane holds
    const int li = lane & 31;
    const int row0 = qt * kRowsPerWg + wave * kRowsPerWave;
    const int i = row0 + li;          // query row of this lane
    const bool wave_active = row0 < N;

    const size_t head_off = (size_t)bh * N * D;
    const int8_t* Qh = a.Q + head_off;
    const int8_t* Kh = a.K + head_off;
    const int8_t* Vh = a.V + head_off;
    const int32_t* bias_row = nullptr;
    if (BIAS) {
        const int b = bh / a.H, h = bh % a.H;
        bias_row = a.bias + ((size_t)(b % a.bias_B) * a.bias_H + (size_t)(h % a.bias_H)) * N * N +
                   (size_t)(i < N ? i : 0) * N;
    }

    // Q rows of this lane as MFMA B operand: 16 contiguous bytes per 32-wide step.
    v4i qreg[KSTEPS];
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) {
        qreg[s] = v4i{0, 0, 0, 0};
        if (i < N) qreg[s] = *(const v4i*)(Qh + (size_t)i * D + 32 * s + 16 * g);
    }

    v16i acc[TB];
#pragma unroll
    for (int t = 0; t < TB; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0;
    int l = 0;
    int m = kMInit;

    const int Tc = (N + BC - 1) / BC;
    for (int j = 0; j < Tc; ++j) {
        const int c0 = j * BC;
        if (j > 0) __syncthreads();   // everyone is done reading the previous tile

        // ---- K tile -> LDS, row-major, 16-byte chunks (coalesced: consecutive threads read
        //      consecutive chunks of consecutive rows)
        constexpr int KCH = BC * D / 16;
#pragma unroll
        for (int ch = tid; ch < KCH; ch += kThreads) {
            const int r = ch / (D / 16), c16 = ch % (D / 16);
            v4i val = {0, 0, 0, 0};
            if (c0 + r < N) val = *(const v4i*)(Kh + (size_t)(c0 + r) * D + 16 * c16);
            *(v4i*)(sK + r * KROW + 16 * c16) = val;
        }
        // ---- V tile -> LDS, transposed to [t][kv], kv columns permuted to the result-layout
        //      order of the first product.  Each thread transposes 4 kv rows x 4 features.
        constexpr int VSB = (BC / 4) * (D / 4);
#pragma unroll
        for (int sb = tid; sb < VSB; sb += kThreads) {
            const int tg = sb % (D / 4), cg = sb / (D / 4);
            unsigned rw[4];
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int c = c0 + 4 * cg + b;
                rw[b] = 0;
                if (c < N) rw[b] = *(const unsigned*)(Vh + (size_t)c * D + 4 * tg);
            }
            // kv row (within the tile) 4*cg = 32*kb + 8*a4 + 4*g2  ->  slot 32*kb + 16*g2 + 4*a4
            const int w = (4 * cg) & 31;
            const int pos = ((4 * cg) & ~31) + 16 * ((w >> 2) & 1) + 4 * (w >> 3);
#pragma unroll
            for (int f = 0; f < 4; ++f) {
                const unsigned o = ((rw[0] >> (8 * f)) & 0xffu) | (((rw[1] >> (8 * f)) & 0xffu) << 8) |
                                   (((rw[2] >> (8 * f)) & 0xffu) << 16) | (((rw[3] >> (8 * f)) & 0xffu) << 24);
                *(unsigned*)(sV + (4 * tg + f) * VROW + pos) = o;
            }
        }
        __syncthreads();
        if (!wave_active) continue;   // uniform per wavefront; still takes part in the barriers

        // ---- step 1: S^T blocks (32 kv rows x 32 queries each)
        v16i s[KB];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
            for (int v = 0; v < 16; ++v) s[kb][v] = 0;
            if (c0 + 32 * kb < N) {
#pragma unroll
                for (int st = 0; st < KSTEPS; ++st) {
                    const v4i ka = *(const v4i*)(sK + (32 * kb + li) * KROW + 32 * st + 16 * g);
                    s[kb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ka, qreg[st], s[kb], 0, 0, 0);
                }
            }
        }
        // ---- bias, exclusion and the ragged end of the sequence
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const bool ragged = c0 + 32 * kb + 32 > N;
            if (BIAS || ragged) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int c = c0 + 32 * kb + 8 * (v >> 2) + 4 * g + (v & 3);
                    int val = s[kb][v];
                    bool excl = c >= N;
                    if (BIAS && !excl) {
                        const int bv = bias_row[c];
                        excl = (bv == INT32_MIN);
                        val += excl ? 0 : bv;
                    }
                    s[kb][v] = excl ? kNegBig : val;
                }
            }
        }
        // ---- steps 2,3: row maximum over the tile, running maximum
        int m_new = m;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
            if (c0 + 32 * kb < N) {
#pragma unroll
                for (int v = 0; v < 16; ++v) m_new = max(m_new, s[kb][v]);
            }
        m_new = max(m_new, xor32(m_new));
        // ---- step 4: max-offset factor alpha, brought to 16 fractional bits
        const int a_hat = shift_exp2(max(m - m_new, a.x_floor), a);
        const int alpha16 = min((int)(((unsigned)a_hat * (unsigned)a.a_mul) >> 14), 65536);
        // ---- steps 5,6,7: score intensity, requantisation to int8, row sum
        v4i pk[KB];
        int rowsum = 0;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            pk[kb] = v4i{0, 0, 0, 0};
            if (c0 + 32 * kb < N) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int x = max(s[kb][v] - m_new, a.x_floor);
                    const int pv = requant(shift_exp2(x, a), a);
                    rowsum += pv;
                    pk[kb][v >> 2] |= pv << (8 * (v & 3));
                }
            }
        }
        rowsum += xor32(rowsum);
        // ---- steps 9,10: ScaleRelease of the running denominator and numerator
        l = scale_release(l, alpha16) + rowsum;
        if (j > 0) {
#pragma unroll
            for (int t = 0; t < TB; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[t][v] = scale_release(acc[t][v], alpha16);
        }
        // ---- step 8: O^T += V_j^T P^T
#pragma unroll
        for (int t = 0; t < TB; ++t)
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
                if (c0 + 32 * kb < N) {
                    const v4i va = *(const v4i*)(sV + (32 * t + li) * VROW + 32 * kb + 16 * g);
                    acc[t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(va, pk[kb], acc[t], 0, 0, 0);
                }
        m = m_new;
    }

    // ---- step 11: integer normalisation, saturate to int8, store.  Lane holds features
    //      32*t + 8*(v/4) + 4*g + v%4 of query i: four consecutive features per dword.
    if (!wave_active || i >= N) return;
    int8_t* Orow = a.O + head_off + (size_t)i * D;
#pragma unroll
    for (int t = 0; t < TB; ++t)
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
            unsigned word = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int o = acc[t][4 * v4 + b];
                int q = 0;
                if (l != 0) q = a.out_round ? floor_div_pos(2 * o + l, 2 * l) : floor_div_pos(o, l);
                q = min(127, max(-128, q));
                word |= ((unsigned)q & 0xffu) << (8 * b);
            }
            *(unsigned*)(Orow + 32 * t + 8 * v4 + 4 * g) = word;
        }
}

template <int D, int BC>
int launch(const QflashKernelArgs& a, hipStream_t stream) {
    const dim3 grid((unsigned)(8 * a.units_per_xcd)), block(kThreads);
    if (a.bias)
        hipLaunchKernelGGL((qflash_fwd_kernel<D, BC, true>), grid, block, 0, stream, a);
    else
        hipLaunchKernelGGL((qflash_fwd_kernel<D, BC, false>), grid, block, 0, stream, a);
    return (int)hipGetLastError();
}

}  // namespace

int qflash_fwd_rows_per_workgroup(int, int) { return kRowsPerWg; }

int qflash_launch_fwd(const QflashKernelArgs& a, int d, int kv_tile, void* stream) {
    hipStream_t st = (hipStream_t)stream;
    if (d == 64 && kv_tile == 64) return launch<64, 64>(a, st);
    if (d == 64 && kv_tile == 128) return launch<64, 128>(a, st);
    if (d == 32 && kv_tile == 64) return launch<32, 64>(a, st);
    if (d == 32 && kv_tile == 128) return launch<32, 128>(a, st);
    return (int)hipErrorInvalidValue;
}
