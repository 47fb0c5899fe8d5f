// Host-only part of the library: everything that decides about a call without touching the GPU --
// derivation of the integer constants from the real scales, the argument checks of the attention
// entry points, and the choice of kernel and work decomposition.  Plain C++ (no HIP): this file is
// also compiled, together with the CPU oracle, into a sanitizer build (address + undefined
// behaviour) that the tests without a GPU run.
#include <cmath>
#include <cstddef>
#include <cstdint>

#include "qflash.h"
#include "qflash_internal.h"
#include "qflash_derive.h"

extern "C" int qflash_params_from_scales(double sQ, double sK, double sV, int d, qflash_params* out) {
    if (!out) return QFLASH_ERR_NULL;
    if (d != 32 && d != 64) return QFLASH_ERR_SHAPE;
    if (!(sQ > 0.0) || !(sK > 0.0) || !(sV > 0.0) || !std::isfinite(sQ) || !std::isfinite(sK) ||
        !std::isfinite(sV))
        return QFLASH_ERR_PARAM;
    return qflash_derive_params(sQ, sK, std::sqrt((double)d), out);
}

// The argument checks shared by every attention entry point, in the order the header documents.
// consts_on_device: the integer constants are computed on the GPU (dynamic quantisation), p is unused.
int qflash_check_call(const void* Q, const void* K, const void* V, const void* O, const int32_t* bias, int bias_B,
                      int bias_H, bool bias_packed, int B, int H, int N, int d, int kv_tile, const qflash_params* p,
                      bool per_head, bool consts_on_device, bool qmax) {
    if (!Q || !K || !V || !O || (!p && !consts_on_device)) return QFLASH_ERR_NULL;
    if (d != 32 && d != 64) return QFLASH_ERR_SHAPE;
    if (B < 1 || H < 1 || N < 1 || N > QFLASH_MAX_N) return QFLASH_ERR_SHAPE;
    if ((int64_t)B * H * N * d >= ((int64_t)1 << 31)) return QFLASH_ERR_SHAPE;
    if (per_head && H > QFLASH_MAX_PARAM_HEADS) return QFLASH_ERR_SHAPE;
    if (bias) {
        if (bias_B < 1 || bias_H < 1) return QFLASH_ERR_SHAPE;
        if ((int64_t)bias_B * bias_H * N * N >= ((int64_t)1 << 31)) return QFLASH_ERR_SHAPE;
        if (bias_packed && qflash_packed_bias_words(bias_B * bias_H, N) >= ((int64_t)1 << 29)) return QFLASH_ERR_SHAPE;
    } else if (bias_packed) {
        return QFLASH_ERR_NULL;
    }
    if (kv_tile != 64 && kv_tile != 128) return QFLASH_ERR_TILE;
    const int n_p = consts_on_device ? 0 : per_head ? H : 1;
    for (int h = 0; h < n_p; ++h) {
        if (!qflash_params_ok(p[h])) return QFLASH_ERR_PARAM;
        if (p[h].out_round != p[0].out_round) return QFLASH_ERR_PARAM;   // one rounding mode per call
        if (qmax && p[h].x_shift != 0) return QFLASH_ERR_PARAM;
    }
    if (((uintptr_t)Q | (uintptr_t)K | (uintptr_t)V | (uintptr_t)O) & 15u) return QFLASH_ERR_ALIGN;
    if (bias && ((uintptr_t)bias & (bias_packed ? 15u : 3u))) return QFLASH_ERR_ALIGN;
    return QFLASH_OK;
}

long long qflash_packed_bias_words(int slices, int N) {
    const long long nb = (N + 31) / 32;
    return (long long)slices * nb * nb * 256;
}


// LDS bytes of the resident kernel: K and V^T of `heads` heads of N rows (ring: of two KV tiles)
// and the weight table; 0 if they do not fit.
// Table size assumed when deciding whether two workgroups with the whole sequence in LDS fit a compute unit.
constexpr int kRingTableGuess = 32 * 1024;

size_t qflash_resident_lds_bytes(int N, int d, int heads, int table_bytes, int lds_limit, int ring_tile) {
    const size_t npad = (size_t)((N + 31) & ~31);
    const size_t kv = ring_tile ? 2 * ((size_t)ring_tile * (size_t)(d + 16) + (size_t)d * (size_t)(ring_tile + 16))
                                : npad * (size_t)(d + 16) + (size_t)d * (npad + 16);
    const size_t bytes = (size_t)heads * kv + (size_t)table_bytes;
    return bytes <= (size_t)lds_limit ? bytes : 0;
}

int qflash_plan_fwd(int BH, int N, int d, int kv_tile, int lds_limit, QflashKernelArgs* a) {
    a->resident = qflash_resident_lds_bytes(N, d, 1, 0, lds_limit) != 0;
    a->heads_per_wg = 1;
    a->pipelined = 0;
    a->ring = 0;
    a->ring_dma = 0;
    a->kv_tile = kv_tile;
    // Long sequences: K and V^T of the whole sequence (plus a weight table) would leave room for
    // one workgroup per compute unit, or for none.  Where the kernel variant can stage tile by
    // tile (d = 64, tile 64), LDS holds two tiles only and workgroups are at most 8 wavefronts,
    // so that two of them share a compute unit.
    const bool two_fit = qflash_resident_lds_bytes(N, d, 1, kRingTableGuess, lds_limit / 2) != 0;
    // (without a bias the ring fed by direct loads is the faster kernel for every long sequence)
    if (d == 64 && N > 256 && (kv_tile == 128 || !two_fit || !a->bias)) {
        const int nblk = (N + 31) / 32;
        const int cus = a->n_cu > 0 ? a->n_cu : 256;
        int waves;
        // Without a bias the ring is fed by direct global-to-LDS loads (qflash_fwd_ring): no wavefront
        // stages anything, registers allow five (tile 64) or three (tile 128) wavefronts per SIMD, and
        // workgroups of four wavefronts, one per SIMD, measured best (DeiT-B/384: 45.3 us against
        // 50.9 with seven or eight and 54.6 with five or six).
        a->ring_dma = !a->bias ? 1 : 0;
        if (a->ring_dma) {
            const int tiles = (nblk + 3) / 4;
            waves = (nblk + tiles - 1) / tiles;                   // balanced: at most 4
        } else if (kv_tile == 128) {
            // 160-odd registers leave three wavefront slots per SIMD: three workgroups of four
            // wavefronts (which is also what stages a tile: 256 threads, two items each)
            waves = 4;
        } else {
            // Workgroups of up to 8 wavefronts (two per compute unit: 128 registers leave four
            // wavefront slots per SIMD) or of 4 (four per compute unit, one wavefront on every SIMD,
            // but every wavefront then also stages K/V): whichever gives the busiest compute unit
            // fewer workgroups to run one after the other.
            const int tiles8 = (nblk + 7) / 8, tiles4 = (nblk + 3) / 4;
            const long long turns8 = ((long long)BH * tiles8 + 2ll * cus - 1) / (2ll * cus);
            const long long turns4 = ((long long)BH * tiles4 + 4ll * cus - 1) / (4ll * cus);
            int tiles = turns4 < turns8 ? tiles4 : tiles8;
            if ((nblk + tiles - 1) / tiles < 4) tiles = tiles8;   // staging needs 256 threads
            waves = (nblk + tiles - 1) / tiles;                   // balanced: 4..8
        }
        a->resident = 1;
        a->ring = 1;
        a->pipelined = 1;
        a->rows_per_wg = 32 * waves;
        a->waves_per_head = waves;
    } else if (a->resident) {
        const int nblk = (N + 31) / 32;
        const int max_waves = N <= 256 ? kResidentMaxWavesNarrow : kResidentMaxWavesWide;
        const int tiles = (nblk + max_waves - 1) / max_waves;
        const int waves = (nblk + tiles - 1) / tiles;       // balanced
        a->rows_per_wg = 32 * waves;
        a->waves_per_head = waves;
        // Short sequences (windowed attention): several (batch, head) pairs per workgroup, so that
        // a workgroup is 8 wavefronts and a weight table is staged once for all of them.
        if (tiles == 1 && waves <= 4) {
            int hp = kResidentMaxWavesNarrow / waves;
            if (hp > BH) hp = BH;
            while (hp > 1 && qflash_resident_lds_bytes(N, d, hp, 0, lds_limit / 4) == 0) --hp;
            a->heads_per_wg = hp;
        }
        // Tile-by-tile staging needs a second KV tile to overlap with and 256 staging threads
        // (32-byte pieces of K plus 4x8 blocks of V of one tile, one or two items per thread).
        a->pipelined = a->heads_per_wg == 1 && N > kv_tile && waves >= 4;
    } else {
        a->rows_per_wg = kStreamRows;
        a->waves_per_head = kStreamWaves;
    }
    a->n_qtiles = (N + a->rows_per_wg - 1) / a->rows_per_wg;
    // per-head constants with several pairs per workgroup: group by head (see the kernel)
    a->same_head = a->per_head && a->heads_per_wg > 1 ? 1 : 0;
    const long long units = a->same_head ? (long long)((a->B + a->heads_per_wg - 1) / a->heads_per_wg) * a->H
                            : a->heads_per_wg > 1 ? ((long long)BH + a->heads_per_wg - 1) / a->heads_per_wg
                                                  : (long long)BH * a->n_qtiles;
    if (units >= (1ll << 30)) return -1;
    a->n_units = (int)units;
    a->units_per_xcd = (a->n_units + 7) / 8;
    // Bias slices repeat every bias_B * H pairs: see qflash_unit_of_workgroup.
    a->xcd_period = 0;
    if (a->bias) {
        const long long pairs = (long long)a->bias_B * a->H;
        const long long period = a->same_head ? (a->bias_B % a->heads_per_wg == 0 ? pairs / a->heads_per_wg : 0)
                                 : a->heads_per_wg > 1 ? (pairs % a->heads_per_wg == 0 ? pairs / a->heads_per_wg : 0)
                                                       : pairs * a->n_qtiles;
        if (period >= 8 && period % 8 == 0 && period <= units) {
            a->xcd_period = (int)period;
            a->units_per_xcd = (int)(((units + period - 1) / period) * (period / 8));
        }
    }
    return 0;
}

int qflash_table_fits(const QflashKernelArgs& a, int d, int table_bytes, int lds_limit) {
    // Every workgroup copies the table from L2 into its LDS: worth it only while that stays below
    // the bytes of Q, K, V, O the workgroup moves anyway.
    const long long io = 4ll * a.heads_per_wg * a.N * d;
    if (io < (long long)table_bytes) return 0;
    if (a.ring_dma) return qflash_ring_lds_bytes(a.waves_per_head, a.kv_tile, table_bytes) <= (size_t)lds_limit / 2;
    // Short sequences with the wide tile: that variant is out of registers with the table's
    // addressing on top (ViT-B/16 B=64: 34 us with the table, 25.5 us without).
    if (d == 64 && a.kv_tile == 128 && a.N <= 256) return 0;
    // keep two workgroups per CU when the sequence is short enough for that to matter
    const int budget = (a.ring || a.N <= 256) ? lds_limit / 2 : lds_limit;
    return qflash_resident_lds_bytes(a.N, d, a.heads_per_wg, table_bytes, budget, a.ring ? a.kv_tile : 0) != 0;
}

size_t qflash_cu_lds_bytes(int N, int heads, int table_bytes) {
    const size_t rows16 = (size_t)((N + 15) & ~15);
    const size_t table = ((size_t)table_bytes + 1023) & ~(size_t)1023;
    return table + (size_t)heads * 3 * rows16 * 64 + 1024 + 4 * (5 * (size_t)heads + 1)
#ifdef QF_TRACE
           + 8 + 2048
#endif
        ;
}

int qflash_plan_cu(int BH, int N, int d, int kv_tile, int lds_limit, int table_bytes, QflashKernelArgs* a) {
    a->cu_mode = 0;
    if (d != 64 || kv_tile != 64 || a->bias || a->per_head || N > 256) return 0;
    const int cus = a->n_cu > 0 ? a->n_cu : 256;
    const int hpw = (BH + cus - 1) / cus;                 // every pair in a single round of workgroups
    if (qflash_cu_lds_bytes(N, hpw, table_bytes) > (size_t)lds_limit) return 0;
    const int nblk = (N + 31) / 32;
    const int units = hpw * nblk;
    a->cu_mode = 1;
    a->cu_heads = hpw;
    a->cu_groups = (BH + hpw - 1) / hpw;
    a->cu_waves = units < 16 ? units : 16;
    a->cu_table_lds = (table_bytes + 1023) & ~1023;
    return 1;
}

// LDS bytes of the direct-load ring kernel: table (rounded up to 1 KiB) and two KV tiles (K and V,
// 64-byte rows).
size_t qflash_ring_lds_bytes(int waves, int kv_tile, int table_bytes) {
    (void)waves;
    return (((size_t)table_bytes + 1023) & ~(size_t)1023) + 2 * (size_t)kv_tile * 128;
}

// LDS bytes of the windowed-attention kernel: the table (rounded up to 1 KiB) and, per wavefront
// (two to a stream), two sets of V, K and 32 query rows (5 KiB each).
size_t qflash_win_lds_bytes(int streams, int table_bytes) {
    return (((size_t)table_bytes + 1023) & ~(size_t)1023) + (size_t)streams * 2 * 2 * 5120;
}

int qflash_plan_win(int d, int kv_tile, int lds_limit, int table_bytes, QflashKernelArgs* a) {
    (void)kv_tile;                      // a single KV tile either way: 64 and 128 give the same result
    a->win_mode = 0;
    if (d != 32 || a->N <= 32 || a->N > 64 || a->per_head || a->qmax) return 0;
    if (a->bias && (!a->bias_packed || a->bias_B < 1 || a->bias_H < 1 || a->B % a->bias_B != 0 || a->H % a->bias_H != 0)) return 0;
    const long long T = (long long)a->B * a->H;
    const int cus = a->n_cu > 0 ? a->n_cu : 256;
    // as many runs as there are pairs, up to eight per compute unit (fewer where the table leaves
    // less LDS); equal shares
    int max_streams = 8;
    while (max_streams > 0 && qflash_win_lds_bytes(max_streams, table_bytes) > (size_t)lds_limit) --max_streams;
    if (max_streams == 0) return 0;
    long long runs = T < (long long)max_streams * cus ? T : (long long)max_streams * cus;
    const long long chunk = (T + runs - 1) / runs;
    runs = (T + chunk - 1) / chunk;
    int streams = (int)((runs + cus - 1) / cus);
    if (streams > max_streams) streams = max_streams;
    const long long groups = (runs + streams - 1) / streams;
    if (chunk >= (1ll << 30) || groups >= (1ll << 30)) return 0;
    if (qflash_win_lds_bytes(streams, table_bytes) > (size_t)lds_limit) return 0;
    a->win_mode = 1;
    a->win_streams = streams;
    a->win_chunk = (int)chunk;
    a->win_groups = (int)groups;
    a->win_table_lds = (table_bytes + 1023) & ~1023;
    return 1;
}
