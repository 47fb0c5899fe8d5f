// Host side of the C ABI declared in include/qflash.h: argument checking, derivation of the
// integer constants from the real scales, context bookkeeping, kernel selection.  No arithmetic
// of the attention itself happens here; all of it runs in the gfx950 kernels.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstring>
#include <mutex>
#include <new>
#include <set>

#include "qflash.h"
#include "qflash_internal.h"

// One immutable weight table.  A slot is written once (by a kernel enqueued on `stream`) and only
// ever used by launches on that same stream, so stream order alone makes it safe; it is never
// rewritten, so captured graphs and in-flight kernels can keep reading it.
struct TableSlot {
    int32_t key[5];   // x_shift, s_inv, exp_mul, p_mul, p_shift
    void* stream;
    int n, n_padded, x_p;
};

constexpr int kTableSlots = 32;
constexpr int kTableMaxBytes = 40 * 1024;

struct qflash_ctx {
    int device;
    int lds_limit;        // LDS bytes one workgroup may allocate on this device
    int use_table;        // QFLASH_CFG_EXP_TABLE
    uint8_t* tables;      // device, kTableSlots x kTableMaxBytes
    int n_slots;          // slots in use
    TableSlot slots[kTableSlots];
};

namespace {

std::mutex g_mu;
std::set<const qflash_ctx*>& live_contexts() {
    static std::set<const qflash_ctx*> s;
    return s;
}

constexpr int kXShiftMax = 13;
constexpr int kSInvMin = 1 << 10;
constexpr int kSInvMax = 1 << 18;  // exclusive

int64_t round_half_up(double x) { return (int64_t)std::floor(x + 0.5); }

// Range and consistency checks that make the 32-bit kernel arithmetic exact (see the comments on
// x_floor in qflash_internal.h and on shift_exp2 in the kernel source).
bool params_ok(const qflash_params& p) {
    if (p.x_shift < 0 || p.x_shift > kXShiftMax) return false;
    if (p.s_inv < kSInvMin || p.s_inv >= kSInvMax) return false;
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

}  // namespace

extern "C" int qflash_params_from_scales(double sQ, double sK, double sV, int d, qflash_params* out) {
    if (!out) return QFLASH_ERR_NULL;
    if (d != 32 && d != 64) return QFLASH_ERR_SHAPE;
    if (!(sQ > 0.0) || !(sK > 0.0) || !(sV > 0.0) || !std::isfinite(sQ) || !std::isfinite(sK) ||
        !std::isfinite(sV))
        return QFLASH_ERR_PARAM;
    // s = sQ * sK * d^(-1/2) * log2(e), evaluated left to right in double (Algorithm 1, Require).
    const double log2e = 1.4426950408889634;
    const double s = ((sQ * sK) / std::sqrt((double)d)) * log2e;
    if (!(s > 0.0) || !std::isfinite(s)) return QFLASH_ERR_PARAM;
    int k = 0;
    while (round_half_up(std::ldexp(1.0, k) / s) < kSInvMin) {
        if (++k > kXShiftMax) return QFLASH_ERR_PARAM;
    }
    const double sk = s / std::ldexp(1.0, k);
    const int64_t s_inv = round_half_up(1.0 / sk);                 // Algorithm 2: round(1/s)
    if (s_inv < kSInvMin || s_inv >= kSInvMax) return QFLASH_ERR_PARAM;
    const int64_t m = round_half_up(-sk * 4294967296.0);           // Algorithm 2: round(-s * 2^N)
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
    if (!params_ok(p)) return QFLASH_ERR_PARAM;
    *out = p;
    return QFLASH_OK;
}

extern "C" int qflash_create(qflash_ctx** out, int device_id) {
    if (!out) return QFLASH_ERR_NULL;
    *out = nullptr;
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || device_id < 0 || device_id >= n) {
        (void)hipGetLastError();
        return QFLASH_ERR_DEVICE;
    }
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device_id) != hipSuccess) {
        (void)hipGetLastError();
        return QFLASH_ERR_DEVICE;
    }
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return QFLASH_ERR_DEVICE;
    qflash_ctx* c = new (std::nothrow) qflash_ctx;
    if (!c) return QFLASH_ERR_DEVICE;
    c->device = device_id;
    int lds = 0;
    if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, device_id) != hipSuccess) {
        (void)hipGetLastError();
        lds = 64 * 1024;
    }
    c->lds_limit = lds;
    c->use_table = 1;
    c->n_slots = 0;
    c->tables = nullptr;
    int cur = -1;
    const bool switched = hipGetDevice(&cur) == hipSuccess && cur != device_id && hipSetDevice(device_id) == hipSuccess;
    if (hipMalloc((void**)&c->tables, (size_t)kTableSlots * kTableMaxBytes) != hipSuccess) {
        (void)hipGetLastError();
        c->tables = nullptr;   // the arithmetic mode needs no tables
    }
    if (switched) (void)hipSetDevice(cur);
    {
        std::lock_guard<std::mutex> lk(g_mu);
        live_contexts().insert(c);
    }
    *out = c;
    return QFLASH_OK;
}

extern "C" int qflash_destroy(qflash_ctx* ctx) {
    if (!ctx) return QFLASH_OK;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        auto it = live_contexts().find(ctx);
        if (it == live_contexts().end()) return QFLASH_ERR_CTX;
        live_contexts().erase(it);
    }
    if (ctx->tables) {
        if (hipFree(ctx->tables) != hipSuccess) (void)hipGetLastError();
    }
    delete ctx;
    return QFLASH_OK;
}

extern "C" int qflash_configure(qflash_ctx* ctx, int key, int value) {
    if (!ctx) return QFLASH_ERR_NULL;
    std::lock_guard<std::mutex> lk(g_mu);
    if (live_contexts().find(ctx) == live_contexts().end()) return QFLASH_ERR_CTX;
    if (key != QFLASH_CFG_EXP_TABLE || (value != 0 && value != 1)) return QFLASH_ERR_PARAM;
    ctx->use_table = value;
    return QFLASH_OK;
}

namespace {

// Clamp point of the exponent: smallest multiple of 2^-k at or below -20.5 octaves.  Above it
// q <= 28 and every intermediate fits 24/32 bits; at and below it the numerator of Algorithm 2
// (< 2^20) is shifted right by >= 20, so the exact result is 0.  Returns false if the constants
// put it beyond 28.5 octaves.
bool fill_head_consts(const qflash_params& p, QflashHeadConsts* h) {
    h->x_shift = p.x_shift; h->s_inv = p.s_inv; h->exp_mul = p.exp_mul;
    h->p_mul = p.p_mul; h->p_shift = p.p_shift; h->a_mul = p.a_mul;
    const int64_t x0 = (41 * (int64_t)p.s_inv + ((int64_t)2 << p.x_shift) - 1) >> (p.x_shift + 1);
    if ((x0 << p.x_shift) * 2 > 57 * (int64_t)p.s_inv) return false;
    h->x_floor = (int)-x0;
    h->lut = nullptr; h->lut_bytes = 0; h->lut_xp = 0;
    return true;
}

// Shared by the per-tensor and the per-head entry points: n_p = 1 (p[0] serves every head) or H.
int attention_impl(qflash_ctx* ctx, const int8_t* Q, const int8_t* K, const int8_t* V, int8_t* O,
                   const int32_t* bias, int bias_B, int bias_H, int B, int H, int N, int d, int kv_tile,
                   const qflash_params* p, bool per_head, void* hip_stream) {
    if (!ctx) return QFLASH_ERR_NULL;
    int device, lds_limit;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        if (live_contexts().find(ctx) == live_contexts().end()) return QFLASH_ERR_CTX;
        device = ctx->device;
        lds_limit = ctx->lds_limit;
    }
    if (!Q || !K || !V || !O || !p) return QFLASH_ERR_NULL;
    if (d != 32 && d != 64) return QFLASH_ERR_SHAPE;
    if (B < 1 || H < 1 || N < 1 || N > QFLASH_MAX_N) return QFLASH_ERR_SHAPE;
    if ((int64_t)B * H * N * d >= ((int64_t)1 << 31)) return QFLASH_ERR_SHAPE;
    if (per_head && H > QFLASH_MAX_PARAM_HEADS) return QFLASH_ERR_SHAPE;
    if (bias) {
        if (bias_B < 1 || bias_H < 1) return QFLASH_ERR_SHAPE;
        if ((int64_t)bias_B * bias_H * N * N >= ((int64_t)1 << 31)) return QFLASH_ERR_SHAPE;
    }
    if (kv_tile != 64 && kv_tile != 128) return QFLASH_ERR_TILE;
    const int n_p = per_head ? H : 1;
    for (int h = 0; h < n_p; ++h) {
        if (!params_ok(p[h])) return QFLASH_ERR_PARAM;
        if (p[h].out_round != p[0].out_round) return QFLASH_ERR_PARAM;   // one rounding mode per call
    }
    if (((uintptr_t)Q | (uintptr_t)K | (uintptr_t)V | (uintptr_t)O) & 15u) return QFLASH_ERR_ALIGN;
    if (bias && ((uintptr_t)bias & 3u)) return QFLASH_ERR_ALIGN;

    static_assert(QFLASH_MAX_PARAM_HEADS == kQflashMaxParamHeads, "header and kernel arguments disagree");
    QflashKernelArgs a;
    a.Q = Q; a.K = K; a.V = V; a.O = O;
    a.bias = bias;
    a.bias_B = bias ? bias_B : 1;
    a.bias_H = bias ? bias_H : 1;
    a.B = B; a.H = H; a.N = N;
    a.out_round = p[0].out_round;
    a.per_head = per_head ? 1 : 0;
    bool all_k0 = true;
    for (int h = 0; h < n_p; ++h) {
        if (!fill_head_consts(p[h], &a.hc[h])) return QFLASH_ERR_PARAM;
        all_k0 = all_k0 && p[h].x_shift == 0;
    }
    a.exp_mode = all_k0 ? 1 : 0;
    a.lut_bytes_max = 0;
    if (qflash_plan_fwd(B * H, N, d, kv_tile, lds_limit, &a) != 0) return QFLASH_ERR_SHAPE;

    int cur = -1;
    if (hipGetDevice(&cur) != hipSuccess) { (void)hipGetLastError(); return QFLASH_ERR_DEVICE; }
    if (cur != device && hipSetDevice(device) != hipSuccess) {
        (void)hipGetLastError();
        return QFLASH_ERR_DEVICE;
    }
    // Look-up mode: find (or build, once, on this stream) the weight table of each set of
    // constants.  It is used only if every head gets one (the mode is uniform over a launch) and
    // the largest fits LDS beside K and V.  Workgroups that serve several pairs share one table,
    // which per-head constants cannot offer.
    int rc = 0;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        bool ok = ctx->use_table && ctx->tables && a.resident && !(per_head && a.heads_per_wg > 1);
        int xp[kQflashMaxParamHeads], np_[kQflashMaxParamHeads], max_bytes = 0;
        for (int h = 0; ok && h < n_p; ++h) {
            // weight is 0 at and below -8 octaves: x_p = ceil(8 s_inv / 2^k)
            const int64_t x_p = (8 * (int64_t)p[h].s_inv + ((int64_t)1 << p[h].x_shift) - 1) >> p[h].x_shift;
            xp[h] = (int)x_p;
            np_[h] = ((int)x_p + 1 + 15) & ~15;
            if (np_[h] > kTableMaxBytes) ok = false;
            if (np_[h] > max_bytes) max_bytes = np_[h];
        }
        ok = ok && qflash_table_fits(a, d, max_bytes, lds_limit);
        for (int h = 0; ok && rc == 0 && h < n_p; ++h) {
            const int32_t key[5] = {p[h].x_shift, p[h].s_inv, p[h].exp_mul, p[h].p_mul, p[h].p_shift};
            int slot = -1;
            for (int i = 0; i < ctx->n_slots; ++i)
                if (ctx->slots[i].stream == hip_stream && std::memcmp(ctx->slots[i].key, key, sizeof key) == 0) {
                    slot = i;
                    break;
                }
            if (slot < 0 && ctx->n_slots < kTableSlots) {
                // The builder is enqueued under the lock, so no other host thread can enqueue a
                // reader of this slot on the same stream ahead of it.
                uint8_t* tbl = ctx->tables + (size_t)ctx->n_slots * kTableMaxBytes;
                rc = qflash_launch_build_table(tbl, xp[h] + 1, np_[h], xp[h], a.hc[h], hip_stream);
                if (rc == 0) {
                    slot = ctx->n_slots++;
                    TableSlot& t = ctx->slots[slot];
                    std::memcpy(t.key, key, sizeof key);
                    t.stream = hip_stream; t.n = xp[h] + 1; t.n_padded = np_[h]; t.x_p = xp[h];
                }
            }
            if (slot < 0) { ok = false; break; }
            a.hc[h].lut = ctx->tables + (size_t)slot * kTableMaxBytes;
            a.hc[h].lut_bytes = np_[h];
            a.hc[h].lut_xp = xp[h];
        }
        if (ok && rc == 0) {
            a.exp_mode = 2;
            a.lut_bytes_max = max_bytes;
        }
    }
    if (rc == 0) rc = qflash_launch_fwd(a, d, kv_tile, lds_limit, hip_stream);
    if (cur != device) (void)hipSetDevice(cur);
    if (rc != 0) { (void)hipGetLastError(); return QFLASH_ERR_LAUNCH; }
    return QFLASH_OK;
}

}  // namespace

extern "C" int qflash_attention(qflash_ctx* ctx, const int8_t* Q, const int8_t* K, const int8_t* V,
                                int8_t* O, const int32_t* bias, int bias_B, int bias_H, int B, int H,
                                int N, int d, int kv_tile, const qflash_params* p, void* hip_stream) {
    return attention_impl(ctx, Q, K, V, O, bias, bias_B, bias_H, B, H, N, d, kv_tile, p, false, hip_stream);
}

extern "C" int qflash_attention_per_head(qflash_ctx* ctx, const int8_t* Q, const int8_t* K, const int8_t* V,
                                         int8_t* O, const int32_t* bias, int bias_B, int bias_H, int B,
                                         int H, int N, int d, int kv_tile, const qflash_params* p,
                                         void* hip_stream) {
    return attention_impl(ctx, Q, K, V, O, bias, bias_B, bias_H, B, H, N, d, kv_tile, p, true, hip_stream);
}

extern "C" const char* qflash_strerror(int code) {
    switch (code) {
        case QFLASH_OK: return "success";
        case QFLASH_ERR_NULL: return "a required pointer is NULL";
        case QFLASH_ERR_SHAPE: return "unsupported shape (d in {32,64}, 1 <= N <= 4096, sizes below 2^31, at most 64 heads with per-head constants)";
        case QFLASH_ERR_TILE: return "kv_tile must be 64 or 128";
        case QFLASH_ERR_PARAM: return "integer constants out of range or inconsistent";
        case QFLASH_ERR_DEVICE: return "no such GPU, not a gfx950 device, or HIP runtime error";
        case QFLASH_ERR_LAUNCH: return "kernel launch failed";
        case QFLASH_ERR_CTX: return "not a live qflash context";
        case QFLASH_ERR_ALIGN: return "Q, K, V, O must be 16-byte aligned and bias 4-byte aligned";
        default: return "unknown qflash error code";
    }
}
