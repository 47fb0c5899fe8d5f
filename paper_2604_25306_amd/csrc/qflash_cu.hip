// gfx950 kernel of the integer-only fused attention forward pass (Algorithm 1) for short sequences
// with 64 features per head and no bias: one workgroup fills a whole compute unit.
//
// A workgroup of up to 16 wavefronts takes `cu_heads` consecutive (batch, head) pairs.  Q, K and V
// of all of them, plus the weight table, go to LDS once, by direct global-to-LDS loads: no staging
// registers, no vector instructions besides a few address computations, no LDS write instructions.
// The tensors sit in LDS row-major as in memory (64-byte rows, the 16-byte pieces of a row permuted
// by the row number so that operand reads are free of bank conflicts); the transposed operand of the
// second product is read with the transposing 8-bit LDS read (see qflash_tile.h).  The unit of work
// is one block of 32 query rows of one pair.  Each wavefront starts with the unit of its own index
// and then takes further units from a counter in LDS, so wavefronts run at their own pace: there is
// no barrier after the start.
//
// Synchronisation.  The loads of a pair are issued by the wavefronts whose first unit belongs to it
// (pairs without such wavefronts: by the last group that has some), in the order of need.  Loads
// complete in order, so a wavefront knows from its own load counter (vmcnt) when its share of a
// tile has landed; it then adds 1 to the counter of (pair, tile) in LDS, and a wavefront may touch
// the data of a tile once that counter has reached the size of the issuing group.  Every wait in
// the kernel is for loads that were issued unconditionally before it and for counters that other
// wavefronts raise without waiting for anybody but their own loads, so every wavefront reaches its
// exit.
//
// QF_TRACE (never defined in the library build) adds per-wavefront timestamps for timeline studies.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <mutex>

#include "qflash_tile.h"

// (M0 is written by the direct loads below and declared as clobbered; the compiler's remark that it
// reserves the register for itself does not apply to a kernel that uses no other M0 instruction)
#pragma clang diagnostic ignored "-Winline-asm"

namespace {

extern __shared__ __align__(1024) int8_t smem_cu[];

typedef __attribute__((address_space(3))) void* lds_void;
typedef const __attribute__((address_space(1))) void* glb_void;
typedef __attribute__((address_space(3))) int lds_int;

// One direct load: the 64 lanes fetch 16 bytes each from g + lane_off (their own offset from a
// uniform address) and the 1 KiB lands at lds_addr + 16 * lane (lds_addr uniform).
// (Spelled out as instructions: for loads it knows to write LDS, the compiler makes the next LDS
// access of the wavefront wait for all of them, while this kernel counts them itself, tile by tile.
// M0 holds the LDS address of such a load; one idle cycle separates writing it from using it.)
__device__ __forceinline__ void load_1k_to_lds(const int8_t* g /* uniform */, int lane_off, int lds_addr /* uniform */) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(lane_off), "s"((glb_void)g) : "memory", "m0");
}

// Wait until the counter at flag_addr (LDS) has reached target.  The LDS serves the requests of a
// wavefront in order, so the reads that follow in program order see what was written before the
// counter was; the empty statement only keeps the compiler from moving them up.
__device__ __forceinline__ void wait_count(int flag_addr, int target) {
    lds_int* f = (lds_int*)(size_t)flag_addr;
    while (__hip_atomic_load(f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) < target) __builtin_amdgcn_s_sleep(2);
    asm volatile("" ::: "memory");
}
// Add 1 to a counter after the loads it stands for have landed (the caller has waited for them).
// Written as an instruction of its own: the compiler would otherwise make every LDS access that it
// cannot tell apart from the destination of a direct load wait for all direct loads still in flight.
__device__ __forceinline__ void count_up(int flag_addr) {
    const int one = 1;
    asm volatile("ds_add_u32 %0, %1" ::"v"(flag_addr), "v"(one) : "memory");
}
#ifdef QF_TRACE
// timestamps go to LDS (an instruction the compiler does not count, like the counters) and are copied out at the end
#define QF_T(K_) do { if ((K_) < 16) { const unsigned long long t_ = __builtin_amdgcn_s_memrealtime(); \
    const int ta_ = trace_base + 8 * (16 * wave + (K_)); \
    asm volatile("ds_write_b64 %0, %1" :: "v"(ta_), "v"(t_) : "memory"); } } while (0)
#else
#define QF_T(K_) do {} while (0)
#endif

template <int XM>
__device__ __forceinline__ void cu_body(const QflashKernelArgs& a) {
    constexpr int D = 64, BC = 64;
    constexpr bool SB = XM == kExpTable;
    const int N = a.N;
    const int rows16 = (N + 15) & ~15;
    const int slot = rows16 * D;                    // LDS bytes of one tensor of one pair
    const int nblk = (N + 31) >> 5;                 // units per pair
    const int hpw = a.cu_heads;
    const int head0 = blockIdx.x * hpw;
    const int n_heads = min(hpw, a.B * a.H - head0);
    const int units = n_heads * nblk;
    const int n_waves = min((int)(blockDim.x >> 6), units);   // the last workgroup may have fewer pairs: extra wavefronts leave
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 5, li = lane & 31;

    // LDS map (dynamic LDS is the only LDS of this kernel, so it starts at address 0 and the index
    // into the weight table is its address): [table][pair 0: K, V, Q][pair 1: ...] ... [1 KiB that
    // reads of the 32-row blocks past the last 16-row block may touch][counters]
    const int lds0 = (int)(size_t)(lds_void)smem_cu;          // 0: checked by the host before the first launch
    const int tbytes = XM == kExpTable ? a.cu_table_lds : 0;
    const int kv_base = lds0 + tbytes;
    // counters: [pair][tile]: wavefronts of the group whose loads for that tile have landed; [4 * hpw]: next unit
    const int cnt_base = kv_base + hpw * 3 * slot + 1024;
#ifdef QF_TRACE
    const int trace_base = cnt_base + 4 * (5 * hpw + 1) + 8;
    for (int t = threadIdx.x; t < 512; t += blockDim.x) *(lds_int*)(size_t)(trace_base + 4 * t) = 0;
    __syncthreads();
#endif
    QF_T(0);
    for (int t = threadIdx.x; t <= 5 * hpw; t += blockDim.x) *(lds_int*)(size_t)(cnt_base + 4 * t) = t == 4 * hpw ? n_waves : 0;
    __syncthreads();
    if (wave >= n_waves) return;
    QF_T(1);

    const QflashHeadConsts hc = head_consts_or_dev(a, a.hc[0]);   // one set of constants per launch

    // ---- loop-invariant registers
    const ExpConst c = make_exp_const(hc);
    const SwizzledLane sl = swizzled_lane_offsets(lane);
    const int nb16 = rows16 >> 4;                   // 1 KiB loads per tensor of a pair
    const int nt = tbytes >> 10;                    // 1 KiB loads of the table

    // ---- the loads.  The wavefronts whose first unit belongs to pair g (its group) share the loads of
    //      that pair: member m of a group of n takes the pieces of the table (group 0 only), the 16-row
    //      blocks of Q and the blocks of K and V (numbered 2 * block + (V ? 1 : 0), i.e. tile by tile)
    //      whose number is m modulo n, and issues them at once in that order, which is the order of
    //      need.  Groups start one after the other (a short sleep), so that the memory system sees
    //      the requests of pair 0 first.  Pairs beyond the last group are taken by that group as
    //      well, after its own; they are only needed in the second round.
    //      A wavefront waits for its loads of the first tile right after issuing them and adds 1 to
    //      the counter of (pair, tile 0); before the second tile of its first unit it waits for all its
    //      loads (they have had a whole tile's time) and adds 1 to the counters of all other tiles.
    //      Before any tile of any unit a wavefront waits until the counter of (pair, tile) has reached
    //      the size of the group.
    const int last_group = (n_waves - 1) / nblk;
    const int my_group = wave / nblk;
    const int group_size = min(nblk, n_waves - my_group * nblk);
    const int member = wave - my_group * nblk;
    const int n_extra = my_group == last_group ? n_heads - 1 - my_group : 0;     // whole pairs
    // A last group of fewer wavefronts than the others gets help with the first tile of its pair from
    // group 0 (whose wavefronts issue their share after their own loads and report it with their
    // other late loads, before the second tile of their first unit).
    const int last_size = n_waves - last_group * nblk;
    const bool small_last = last_group > 0 && last_size < nblk;
    const bool helper = small_last && my_group == 0, helped = small_last && my_group == last_group;
    {
        // Lane part of the address inside a 16-row block: row lane / 4, 16-byte piece (lane % 4)
        // permuted by the row.  The last block of a tensor may reach beyond the sequence: its rows are
        // clamped to the last row (what lands in the padding rows is never used).
        const int lrow = lane >> 2, piece = ((lane & 3) ^ ((lane >> 4) & 3)) << 4;
        const int off_norm = lrow * D + piece;
        const int off_last = (min(16 * (nb16 - 1) + lrow, N - 1) - 16 * (nb16 - 1)) * D + piece;
        // First tile of the own pair (and the table).  The other groups start when the first tile of
        // group 0 has landed: the memory system shares its bandwidth evenly between whatever is in
        // flight, so this is what lets group 0 start computing while the others are still loading.
        if (my_group > 0) wait_count(cnt_base, nblk);
        if (XM == kExpTable && my_group == 0)
            for (int it = member; it < nt; it += group_size)
                load_1k_to_lds((const int8_t*)hc.lut + 1024 * it, 16 * lane, lds0 + 1024 * it);
        const int x0 = min(8, 2 * nb16);                            // K/V block numbers of the first tile
        auto load_q = [&](int h, int mi, int np) {
            const size_t head_off = (size_t)(head0 + h) * N * D;
            for (int b = mi; b < nb16; b += np)
                load_1k_to_lds(a.Q + head_off + 1024 * b, b == nb16 - 1 ? off_last : off_norm,
                               kv_base + (3 * h + 2) * slot + 1024 * b);
        };
        auto load_kv = [&](int h, int x_lo, int x_hi, int mi, int np) {
            const size_t head_off = (size_t)(head0 + h) * N * D;
            const int first = x_lo + ((mi - x_lo) % np + np) % np;
            for (int x = first; x < x_hi; x += np) {
                const int b = x >> 1;
                load_1k_to_lds(((x & 1) ? a.V : a.K) + head_off + 1024 * b, b == nb16 - 1 ? off_last : off_norm,
                               kv_base + (3 * h + (x & 1)) * slot + 1024 * b);
            }
        };
        // (a last group of few wavefronts shares the first tile of its pair with the group before it)
        const int s0_np = helped ? group_size + nblk : group_size, s0_mi = helped ? nblk + member : member;
        load_q(my_group, s0_mi, s0_np);
        load_kv(my_group, 0, x0, s0_mi, s0_np);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (lane == 0) count_up(cnt_base + 4 * (4 * my_group));
        // the other tiles, then further pairs, then the share of the next group's first tile
        load_kv(my_group, x0, 2 * nb16, member, group_size);
        for (int e = 1; e <= n_extra; ++e) {
            load_q(my_group + e, member, group_size);
            load_kv(my_group + e, 0, 2 * nb16, member, group_size);
        }
        if (helper) {
            load_q(last_group, member, nblk + last_size);
            load_kv(last_group, 0, x0, member, nblk + last_size);
        }
    }
    const int n_tiles = (N + BC - 1) / BC;
    [[maybe_unused]] int tk = 3;
    QF_T(2);

    // Units: wavefront w starts with unit w; all further ones come from the counter.
    bool first_unit = true;
    int u = wave;
    while (u < units) {
        // (the sequence length through an opaque copy: the compiler would otherwise evaluate every
        // "is this group of keys inside the sequence" test of the ragged tile once, ahead of the loop,
        // and keep the answers in more scalar registers than there are)
        int N_ = N;
        asm volatile("" : "+s"(N_));
        // (likewise the lane's half: the key indices of the ragged tile derive from it, two dozen
        // registers' worth if they are prepared ahead of the loop)
        int g_ = g;
        asm volatile("" : "+v"(g_));
        const int n_full = N_ / BC, rem = N_ - n_full * BC;
        const int h = u / nblk, blk = u - h * nblk;
        const int owner = min(h, last_group);
        const int target = min(nblk, n_waves - owner * nblk);
        const int Kb = kv_base + 3 * h * slot, Vb = Kb + slot, Qb = Vb + slot;
        const int row0 = 32 * blk, i = row0 + li;
        RowState<D> st;
        st.l = 0;
        st.m = SB ? (int)((unsigned)kMInit + (unsigned)kAccBias) : kMInit;
        v4i qreg[2];
#define QF_TILE(FULL_, FIRST_, J_, NV_, NG_)                                                               \
        if (first_unit && (J_) == (n_tiles > 1 ? 1 : 0)) {                                                 \
            /* second tile of the first unit (or its only one): all own loads have had a tile's time */   \
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                                               \
            if (lane == 0) {                                                                               \
                if (helper) count_up(cnt_base + 4 * (4 * last_group));                                     \
                for (int s = 1; s < n_tiles; ++s) count_up(cnt_base + 4 * (4 * my_group + s));             \
                for (int e = my_group + 1; e <= my_group + n_extra; ++e)                                   \
                    for (int s = 0; s < n_tiles; ++s) count_up(cnt_base + 4 * (4 * e + s));                \
            }                                                                                              \
        }                                                                                                  \
        if ((FIRST_) && XM == kExpTable && h != 0) wait_count(cnt_base, min(nblk, n_waves));               \
        wait_count(cnt_base + 4 * (4 * h + (J_)), (J_) == 0 && small_last && h == last_group ? target + nblk : target); \
        if (FIRST_) QF_T(tk);                                                                              \
        if (FIRST_) {                                                                                      \
            _Pragma("unroll") for (int s = 0; s < 2; ++s)                                                  \
                qreg[s] = *(lds_v4i*)(size_t)(Qb + row0 * D + (sl.k_off ^ (32 * s)));                      \
        }                                                                                                  \
        process_tile<D, BC, kBiasNone, XM, SB, FULL_, FIRST_, kLaySwizzled, NG_>(                          \
            st, qreg, nullptr, 0, nullptr, 0, NV_, hc.lut_xp, nullptr, nullptr, c, hc.a_mul, li, g_,      \
            Kb + 4096 * (J_) + sl.k_off, Vb + 4096 * (J_) + sl.v_off);                                     \
        if (tk == 6) QF_T(9 + (J_))
        // the ragged tile, with its number of groups of 8 keys as a compile-time constant
#define QF_RAGGED(FIRST_, J_)                                                                              \
        switch ((rem + 7) >> 3) {                                                                          \
            case 1: { QF_TILE(false, FIRST_, J_, rem, 1); } break;                                         \
            case 2: { QF_TILE(false, FIRST_, J_, rem, 2); } break;                                         \
            case 3: { QF_TILE(false, FIRST_, J_, rem, 3); } break;                                         \
            case 4: { QF_TILE(false, FIRST_, J_, rem, 4); } break;                                         \
            case 5: { QF_TILE(false, FIRST_, J_, rem, 5); } break;                                         \
            case 6: { QF_TILE(false, FIRST_, J_, rem, 6); } break;                                         \
            case 7: { QF_TILE(false, FIRST_, J_, rem, 7); } break;                                         \
            default: { QF_TILE(false, FIRST_, J_, rem, 8); } break;                                        \
        }
        if (n_full > 0) {
            QF_TILE(true, true, 0, BC, 0);
            for (int j = 1; j < n_full; ++j) { QF_TILE(true, false, j, BC, 0); }
            if (rem > 0) { QF_RAGGED(false, n_full) }
        } else {
            QF_RAGGED(true, 0)
        }
#undef QF_RAGGED
#undef QF_TILE
        first_unit = false;
        QF_T(tk + 1);
        if (i < N) {
            // (uniform base plus a 32-bit lane offset made here: a per-lane 64-bit pointer prepared ahead of
            // the unit loop would be held in registers across all the tile code, or spilled)
            v4i w[2];
            normalise_words<D, 16>(st, a.out_round != 0, w);
            int8_t* Ob = a.O + (size_t)(head0 + h) * N * D;
            unsigned o_lane = (unsigned)(i * D + g * (D / 2));
            asm volatile("" : "+v"(o_lane));
            *(v4i*)(Ob + o_lane) = w[0];
            *(v4i*)(Ob + o_lane + 16) = w[1];
        }
        // next unit
        int nxt = 0;
        if (lane == 0) nxt = __hip_atomic_fetch_add((lds_int*)(size_t)(cnt_base + 4 * 4 * hpw), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        u = __builtin_amdgcn_readfirstlane(nxt);
        QF_T(tk + 2);
        tk += 3;
    }
    QF_T(15);
#ifdef QF_TRACE
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if (a.trace && lane < 16)
        a.trace[((size_t)blockIdx.x * 16 + wave) * 16 + lane] = *(const __attribute__((address_space(3))) unsigned long long*)(size_t)(trace_base + 8 * (16 * wave + lane));
#endif
}

template <int XM>
__global__ __launch_bounds__(1024) void qflash_fwd_cu(const QflashKernelArgs a) {
    if constexpr (XM == kExpAuto) {
        if (head_consts_or_dev(a, a.hc[0]).lut_bytes > 0) cu_body<kExpTable>(a);
        else cu_body<kExpShift>(a);
    } else {
        cu_body<XM>(a);
    }
}

template <int XM>
int launch_cu(const QflashKernelArgs& a, size_t lds, int lds_limit, hipStream_t st) {
    auto kern = qflash_fwd_cu<XM>;
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
    hipLaunchKernelGGL(kern, dim3((unsigned)a.cu_groups), dim3((unsigned)(64 * a.cu_waves)), lds, st, a);
    return (int)hipGetLastError();
}

}  // namespace

// LDS bytes of the kernel above for `heads` pairs of N rows and a table of table_bytes.
int qflash_launch_fwd_cu(const QflashKernelArgs& a, int lds_limit, void* stream) {
    hipStream_t st = (hipStream_t)stream;
    if (!a.cu_mode || a.cu_heads < 1 || a.cu_waves < 1 || a.cu_waves > 16 || a.N > 256 || a.bias) return (int)hipErrorInvalidValue;
    const bool table = a.exp_mode == kExpTable || a.exp_mode == kExpAuto;
    if (table && a.lut_bytes_max > a.cu_table_lds) return (int)hipErrorInvalidValue;
    const size_t lds = qflash_cu_lds_bytes(a.N, a.cu_heads, table ? a.cu_table_lds : 0);
    if (lds > (size_t)lds_limit) return (int)hipErrorInvalidValue;
    if (a.exp_mode == kExpAuto) return launch_cu<kExpAuto>(a, lds, lds_limit, st);
    if (a.exp_mode == kExpTable) return launch_cu<kExpTable>(a, lds, lds_limit, st);
    if (a.exp_mode == kExpShift0) return launch_cu<kExpShift0>(a, lds, lds_limit, st);
    return launch_cu<kExpShift>(a, lds, lds_limit, st);
}
