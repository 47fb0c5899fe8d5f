// gfx950 kernel of the integer-only fused attention forward pass (Algorithm 1) for long sequences
// with 64 features per head and no bias: the two-tile ring, fed by direct
// global-to-LDS loads.
//
// A workgroup of up to 8 wavefronts (4 where the sequence allows it) serves 32 query rows per wavefront of one (batch, head) pair and
// walks over all KV tiles of the pair.  LDS holds the weight table and two KV tiles: the one in use and the one on its way.  K and V tiles arrive row-major as they lie
// in memory (64-byte rows, 16-byte pieces permuted by the row so that operand reads are free of bank
// conflicts), put there by `global_load_lds_dwordx4`; the K/Q operands are plain 16-byte LDS reads
// and the V^T operand is read with the transposing 8-bit LDS read (see qflash_tile.h).  Compared with
// staging through registers (qflash_resident.h) there are no staging registers, no byte transposes
// in the vector ALU and no LDS write instructions: about a third of that kernel's vector
// instructions on these shapes.
//
// Synchronisation: the wavefronts share the loads of a tile (1 KiB pieces, dealt round robin).
// While tile j is computed, tile j+1 lands in the other slot; after its arithmetic a wavefront waits
// for its own loads (vmcnt) and then for the others at a workgroup barrier, which also says that
// everybody is done with tile j, whose slot the loads of tile j+2 may now overwrite.  Every
// wavefront of a workgroup executes every barrier, with or without query rows of its own.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <mutex>

#include "qflash_tile.h"

// (M0 is written by the direct loads below and declared as clobbered)
#pragma clang diagnostic ignored "-Winline-asm"

namespace {

extern __shared__ __align__(1024) int8_t smem_ring[];

typedef __attribute__((address_space(3))) void* lds_void_r;
typedef const __attribute__((address_space(1))) void* glb_void_r;

// 64 lanes fetch 16 bytes each from g + lane_off; the 1 KiB lands at lds_addr + 16 * lane.
__device__ __forceinline__ void ring_load_1k(const int8_t* g /* uniform */, int lane_off, int lds_addr /* uniform */) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(lane_off), "s"((glb_void_r)g) : "memory", "m0");
}

template <int BC, int XM, bool QMAX>
__device__ __forceinline__ void ring_body(const QflashKernelArgs& a) {
    constexpr int D = 64;
    constexpr int kRingTileBytes = 2 * BC * D;      // one KV tile in LDS: K (BC rows x 64 bytes), then V
    constexpr int kPieces = 2 * BC / 16;            // 1 KiB pieces of a tile: K blocks of 16 rows, then V blocks
    constexpr bool SB = XM == kExpTable;
    const int N = a.N;
    const int unit = qflash_unit_of_workgroup(blockIdx.x, a.units_per_xcd, a.xcd_period);
    if (unit >= a.n_units) return;
    const int qt = unit % a.n_qtiles, bh = unit / a.n_qtiles;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_waves = (int)(blockDim.x >> 6);
    const int g = lane >> 5, li = lane & 31;
    const QflashHeadConsts hc = head_consts(a, bh);
    const ExpConst c = make_exp_const(hc);
    const SwizzledLane sl = swizzled_lane_offsets(lane);

    // ---- LDS: [weight table][slot 0][slot 1]; the dynamic LDS is the only LDS of the kernel, so the
    //      table index is its address
    const int lds0 = (int)(size_t)(lds_void_r)smem_ring;
    const int tbytes = XM == kExpTable ? a.ring_table_lds : 0;
    const int ring_base = lds0 + tbytes;

    const size_t head_off = (size_t)bh * N * D;
    const int8_t* Kh = a.K + head_off;
    const int8_t* Vh = a.V + head_off;
    const int row0 = qt * a.rows_per_wg + wave * 32;
    const bool active = row0 < N;
    const int n_tiles = (N + BC - 1) / BC;

    // Lane part of the address of a 16-row block: row lane / 4, 16-byte piece (lane % 4) permuted by the
    // row.  Rows beyond the sequence are clamped to the last row (what lands there is never used).
    const int lrow = lane >> 2, piece = ((lane & 3) ^ ((lane >> 4) & 3)) << 4;
    auto block_off = [&](int first_row) { return min(first_row + lrow, N - 1) * D + piece; };
    // The 1 KiB pieces of tile j (the K blocks, then the V blocks), dealt round robin to the wavefronts.
    auto issue_tile = [&](int j) {
        const int slot = ring_base + kRingTileBytes * (j & 1);
        for (int x = wave; x < kPieces; x += n_waves) {
            const int b = x % (kPieces / 2);
            ring_load_1k(x < kPieces / 2 ? Kh : Vh, block_off(BC * j + 16 * b), slot + 1024 * x);
        }
    };

    // ---- prologue: table (shared), first tile, this lane's query row (straight to its operand
    //      registers; rows beyond the sequence read the last row and are never stored); one wait,
    //      one barrier.  The query registers are touched right after the wait: these are the only
    //      loads the compiler counts, and it must not find them pending later, when waiting for
    //      them would mean waiting for the tile in flight.
    if (XM == kExpTable)
        for (int it = wave; it < (tbytes >> 10); it += n_waves)
            ring_load_1k((const int8_t*)hc.lut + 1024 * it, 16 * lane, lds0 + 1024 * it);
    issue_tile(0);
    v4i qreg[2];
    {
        const int8_t* Qrow = a.Q + head_off + (size_t)min(row0 + li, N - 1) * D + 16 * g;
#pragma unroll
        for (int s = 0; s < 2; ++s) qreg[s] = *(const v4i*)(Qrow + 32 * s);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
    for (int s = 0; s < 2; ++s) asm volatile("" : "+v"(qreg[s]));
    __syncthreads();

    RowState<D> st;
    st.l = 0;
    const int m_init = QMAX ? qmax_initial_reference(hc.s_inv, hc.a_mul) : kMInit;
    st.m = SB ? (int)((unsigned)m_init + (unsigned)kAccBias) : m_init;

    const int n_full = N / BC, rem = N - n_full * BC;
#define QF_RING_TILE(FULL_, FIRST_, J_, NV_)                                                                   \
    {                                                                                                          \
        if ((J_) + 1 < n_tiles) issue_tile((J_) + 1);                                                          \
        if (active) {                                                                                          \
            const int slot = ring_base + kRingTileBytes * ((J_) & 1);                                          \
            process_tile<D, BC, kBiasNone, XM, SB, FULL_, FIRST_, kLaySwizzled, 0, QMAX>(                            \
                st, qreg, nullptr, 0, nullptr, 0, NV_, hc.lut_xp, nullptr, nullptr, c, hc.a_mul, li, g,       \
                slot + sl.k_off, slot + BC * D + sl.v_off);                                                      \
        }                                                                                                      \
        if ((J_) + 1 < n_tiles) {                                                                              \
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                                                   \
            __syncthreads();                                                                                   \
        }                                                                                                      \
    }
    if (n_full > 0) {
        QF_RING_TILE(true, true, 0, BC)
        for (int j = 1; j < n_full; ++j) QF_RING_TILE(true, false, j, BC)
        if (rem > 0) QF_RING_TILE(false, false, n_full, rem)
    } else {
        QF_RING_TILE(false, true, 0, rem)
    }
#undef QF_RING_TILE
    const int i = row0 + li;
    if (!active || i >= N) return;
    normalise_store<D, 20>(st, a.O + head_off + (size_t)i * D, g, a.out_round != 0);
}

// Wavefronts per SIMD the register allocation has to allow: with KV tiles of 64, 5 for the look-up
// variant (94 registers) and 4 for the others (which would spill at 96); 3 with tiles of 128 (137
// registers; held to 128 it spills a dozen and is a sixth slower).
// QMAX: the quantised-maximum variant (not Algorithm 1 as printed; see process_tile).
template <int BC, int XM, bool QMAX>
__global__ __launch_bounds__(512, (BC == 128 ? 3 : XM == kExpTable ? 5 : 4)) void qflash_fwd_ring(const QflashKernelArgs a) {
    if constexpr (XM == kExpAuto) {
        const int unit = qflash_unit_of_workgroup(blockIdx.x, a.units_per_xcd, a.xcd_period);
        if (unit >= a.n_units) return;
        if (head_consts(a, unit / a.n_qtiles).lut_bytes > 0) ring_body<BC, kExpTable, QMAX>(a);
        else ring_body<BC, kExpShift, QMAX>(a);
    } else {
        ring_body<BC, XM, QMAX>(a);
    }
}

template <int BC, int XM, bool QMAX>
int launch_ring(const QflashKernelArgs& a, size_t lds, int lds_limit, hipStream_t st) {
    auto kern = qflash_fwd_ring<BC, XM, QMAX>;
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
    hipLaunchKernelGGL(kern, dim3((unsigned)(8 * a.units_per_xcd)), dim3((unsigned)(64 * a.waves_per_head)), lds, st, a);
    return (int)hipGetLastError();
}

}  // namespace

namespace {
template <bool QMAX>
int launch_variant(const QflashKernelArgs& a, size_t lds, int lds_limit, hipStream_t st) {
    if (a.kv_tile == 64) {
        if (a.exp_mode == kExpAuto) return launch_ring<64, kExpAuto, QMAX>(a, lds, lds_limit, st);
        if (a.exp_mode == kExpTable) return launch_ring<64, kExpTable, QMAX>(a, lds, lds_limit, st);
        if (a.exp_mode == kExpShift0) return launch_ring<64, kExpShift0, QMAX>(a, lds, lds_limit, st);
        return launch_ring<64, kExpShift, QMAX>(a, lds, lds_limit, st);
    }
    if (a.exp_mode == kExpAuto) return launch_ring<128, kExpAuto, QMAX>(a, lds, lds_limit, st);
    if (a.exp_mode == kExpTable) return launch_ring<128, kExpTable, QMAX>(a, lds, lds_limit, st);
    if (a.exp_mode == kExpShift0) return launch_ring<128, kExpShift0, QMAX>(a, lds, lds_limit, st);
    return launch_ring<128, kExpShift, QMAX>(a, lds, lds_limit, st);
}
}  // namespace

int qflash_launch_fwd_ring(const QflashKernelArgs& a, int lds_limit, void* stream) {
    hipStream_t st = (hipStream_t)stream;
    // everything the kernel's indexing assumes, checked once more where it is launched
    if (!a.ring_dma || !a.ring || a.bias || a.heads_per_wg != 1 || (a.kv_tile != 64 && a.kv_tile != 128))
        return (int)hipErrorInvalidValue;
    if (a.waves_per_head < 1 || a.waves_per_head > 8 || a.rows_per_wg != 32 * a.waves_per_head) return (int)hipErrorInvalidValue;
    if ((long long)a.rows_per_wg * a.n_qtiles < a.N) return (int)hipErrorInvalidValue;
    const bool table = a.exp_mode == kExpTable || a.exp_mode == kExpAuto;
    if (table && a.lut_bytes_max > a.ring_table_lds) return (int)hipErrorInvalidValue;
    const size_t lds = qflash_ring_lds_bytes(a.waves_per_head, a.kv_tile, table ? a.ring_table_lds : 0);
    if (lds > (size_t)lds_limit) return (int)hipErrorInvalidValue;
    return a.qmax ? launch_variant<true>(a, lds, lds_limit, st) : launch_variant<false>(a, lds, lds_limit, st);
}
