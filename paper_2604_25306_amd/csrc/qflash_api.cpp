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
#include "qflash_derive.h"

// One weight table.  A slot is written by a kernel enqueued on `stream` and only ever read by
// launches on that same stream, so stream order alone makes the first use safe.  When all slots are
// taken, the least recently used one is rebuilt for new constants: the building kernel then waits,
// on the GPU, for everything enqueued so far on the stream that read the old table.  A slot that
// a stream under capture has used is never rebuilt: a captured graph keeps reading it.
struct TableSlot {
    int32_t key[5];   // x_shift, s_inv, exp_mul, p_mul, p_shift
    void* stream;
    int n, n_padded, x_p;
    uint64_t last_use;   // value of the context's launch counter at the last launch that read it
    bool pinned;         // read under stream capture
};

constexpr int kPlanQueryTableBytes = 32 * 1024;   // table size qflash_plan_query assumes (it is not given constants)
constexpr int kTableSlots = 32;
constexpr int kTableMaxBytes = 40 * 1024;

// Device memory of the entry point that allocates nothing (qflash_attention_static): room for one
// weight table.  Every GPU the library runs on holds its own copy until the process ends.  In host
// code this name is only a stand-in for the symbol: the address that kernels and copies may use is
// the one hipGetSymbolAddress reports for the current device (qflash_create, kept in the context).
constexpr int kScratchBytes = QFLASH_STATIC_TABLE_BYTES;
static_assert(kScratchBytes % 256 == 0 && kScratchBytes <= kTableMaxBytes, "one table at most");
static __device__ __align__(256) uint8_t scratch[kScratchBytes];

struct qflash_ctx {
    int device;
    int lds_limit;        // LDS bytes one workgroup may allocate on this device
    int n_cu;             // compute units
    int use_table;        // QFLASH_CFG_EXP_TABLE
    int qmax;             // QFLASH_CFG_QUANTISED_MAX
    uint8_t* tables;      // device, kTableSlots x kTableMaxBytes
    uint8_t* scratch_ptr; // device address of `scratch` on this context's GPU, or nullptr
    int n_slots;          // slots in use
    TableSlot slots[kTableSlots];
    std::mutex mu;        // guards the table cache and the options; held while a launch that reads the cache is enqueued
    uint64_t launches;    // launch counter (age of the slots)
    hipEvent_t evict_ev;  // marks "everything enqueued so far" on the stream of a slot about to be rebuilt
    int evictions;        // slots rebuilt for other constants so far
    int last_mode;        // weight mode of the last launch through the cache: QFLASH_WEIGHTS_*
    int last_kernel;      // kernel family of the last launch (as qflash_plan_info.kernel)
};

namespace {

std::mutex g_mu;
std::set<const qflash_ctx*>& live_contexts() {
    static std::set<const qflash_ctx*> s;
    return s;
}

}  // namespace

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
    c->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    c->use_table = 1;
    c->qmax = 0;
    c->n_slots = 0;
    c->tables = nullptr;
    c->launches = 0;
    c->evictions = 0;
    c->last_mode = QFLASH_WEIGHTS_ARITHMETIC;
    c->last_kernel = 0;
    c->evict_ev = nullptr;
    int cur = -1;
    const bool switched = hipGetDevice(&cur) == hipSuccess && cur != device_id && hipSetDevice(device_id) == hipSuccess;
    if (hipMalloc((void**)&c->tables, (size_t)kTableSlots * kTableMaxBytes) != hipSuccess) {
        (void)hipGetLastError();
        c->tables = nullptr;   // the arithmetic mode needs no tables
    }
    if (hipEventCreateWithFlags(&c->evict_ev, hipEventDisableTiming) != hipSuccess) {
        (void)hipGetLastError();
        c->evict_ev = nullptr;     // without it a full cache is never recycled
    }
    // Address of this device's copy of the static table memory (the context's device is current).
    c->scratch_ptr = nullptr;
    {
        void* sp = nullptr;
        if (hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch)) == hipSuccess) c->scratch_ptr = (uint8_t*)sp;
        else (void)hipGetLastError();
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
    if (ctx->evict_ev && hipEventDestroy(ctx->evict_ev) != hipSuccess) (void)hipGetLastError();
    delete ctx;
    return QFLASH_OK;
}

extern "C" int qflash_configure(qflash_ctx* ctx, int key, int value) {
    if (!ctx) return QFLASH_ERR_NULL;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        if (live_contexts().find(ctx) == live_contexts().end()) return QFLASH_ERR_CTX;
    }
    if ((key != QFLASH_CFG_EXP_TABLE && key != QFLASH_CFG_QUANTISED_MAX) || (value != 0 && value != 1)) return QFLASH_ERR_PARAM;
    std::lock_guard<std::mutex> lk(ctx->mu);
    if (key == QFLASH_CFG_EXP_TABLE) ctx->use_table = value;
    else ctx->qmax = value;
    return QFLASH_OK;
}

#ifdef QF_TRACE
static unsigned long long* g_trace = nullptr;
extern "C" void qflash_debug_trace(void* buf) { g_trace = (unsigned long long*)buf; }
#endif

namespace {

// The kernel family the plan chose.
int launch_attention(QflashKernelArgs& a, int d, int kv_tile, int lds_limit, void* hip_stream) {
    if (a.win_mode) return qflash_launch_fwd_win(a, lds_limit, hip_stream);
    if (a.cu_mode) return qflash_launch_fwd_cu(a, lds_limit, hip_stream);
    if (a.ring_dma) {
        a.ring_table_lds = (a.lut_bytes_max + 1023) & ~1023;
        return qflash_launch_fwd_ring(a, lds_limit, hip_stream);
    }
    return qflash_launch_fwd(a, d, kv_tile, lds_limit, hip_stream);
}

// Whether the planned launch can hold a weight table of table_bytes in LDS and copying it pays.
bool table_fits(const QflashKernelArgs& a, int d, int table_bytes, int lds_limit) {
    if (a.win_mode) return table_bytes <= a.win_table_lds;      // staged once per compute unit
    if (a.cu_mode) return table_bytes <= a.cu_table_lds && 4ll * a.cu_heads * a.N * d >= (long long)table_bytes;
    return qflash_table_fits(a, d, table_bytes, lds_limit) != 0;
}

// Shared by the per-tensor and the per-head entry points: n_p = 1 (p[0] serves every head) or H.
// hc_dev != nullptr: the constants are computed on the GPU (dynamic quantisation); p is then not
// used and out_round_dev gives the rounding mode.
int attention_impl(qflash_ctx* ctx, const int8_t* Q, const int8_t* K, const int8_t* V, int8_t* O,
                   const int32_t* bias, int bias_B, int bias_H, int B, int H, int N, int d, int kv_tile,
                   const qflash_params* p, bool per_head, void* hip_stream,
                   QflashHeadConsts* hc_dev = nullptr, int out_round_dev = 0, bool bias_packed = false,
                   uint8_t* dyn_table = nullptr, bool static_table = false) {
    if (!ctx) return QFLASH_ERR_NULL;
    int device, lds_limit, n_cu;
    uint8_t* scratch_ptr;
    bool table_wanted, qmax;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        if (live_contexts().find(ctx) == live_contexts().end()) return QFLASH_ERR_CTX;
        device = ctx->device;
        lds_limit = ctx->lds_limit;
        n_cu = ctx->n_cu;
        scratch_ptr = ctx->scratch_ptr;
    }
    {
        std::lock_guard<std::mutex> lk(ctx->mu);
        table_wanted = ctx->use_table != 0;
        qmax = ctx->qmax != 0;
    }
    // The quantised-maximum variant takes its constants from the host and needs x_shift = 0.
    if (qmax && (hc_dev || static_table)) return QFLASH_ERR_PARAM;
    {
        const int rc = qflash_check_call(Q, K, V, O, bias, bias_B, bias_H, bias_packed, B, H, N, d, kv_tile, p, per_head,
                                         hc_dev != nullptr, qmax);
        if (rc != QFLASH_OK) return rc;
    }
    const int n_p = hc_dev ? 0 : per_head ? H : 1;
    // The entry point that allocates nothing keeps its one weight table in the static device array:
    // constants whose table is larger than that are refused, not silently run another way.
    int static_xp = 0, static_np = 0;
    if (static_table && table_wanted) {
        const int64_t x_p = (8 * (int64_t)p[0].s_inv + ((int64_t)1 << p[0].x_shift) - 1) >> p[0].x_shift;
        if (x_p + 16 > kScratchBytes) return QFLASH_ERR_SCRATCH;
        if (!scratch_ptr) return QFLASH_ERR_DEVICE;
        static_xp = (int)x_p;
        static_np = ((int)x_p + 1 + 15) & ~15;
    }

    static_assert(QFLASH_MAX_PARAM_HEADS == kQflashMaxParamHeads, "header and kernel arguments disagree");
    QflashKernelArgs a;
    a.Q = Q; a.K = K; a.V = V; a.O = O;
    a.bias = bias;
    a.bias_B = bias ? bias_B : 1;
    a.bias_H = bias ? bias_H : 1;
    a.bias_packed = bias_packed ? 1 : 0;
    a.B = B; a.H = H; a.N = N;
    a.out_round = hc_dev ? out_round_dev : p[0].out_round;
    a.per_head = per_head ? 1 : 0;
    a.qmax = qmax ? 1 : 0;
    a.hc_dev = hc_dev;
    a.n_cu = n_cu;
#ifdef QF_TRACE
    a.trace = g_trace;
#endif
    bool all_k0 = hc_dev == nullptr;
    for (int h = 0; h < n_p; ++h) {
        if (!qflash_fill_head_consts(p[h], &a.hc[h])) return QFLASH_ERR_PARAM;
        all_k0 = all_k0 && p[h].x_shift == 0;
    }
    a.exp_mode = all_k0 ? 1 : 0;
    a.lut_bytes_max = 0;
    if (qflash_plan_fwd(B * H, N, d, kv_tile, lds_limit, &a) != 0) return QFLASH_ERR_SHAPE;
    a.ring_table_lds = 0;
    // The kernel that gives a whole compute unit to one workgroup, where the shape allows it: its LDS
    // budget depends on the size of the weight table the call would use.
    {
        int table_hint = 0;
        if (hc_dev) {
            table_hint = (table_wanted && dyn_table) ? kTableMaxBytes : 0;
        } else if (static_table) {
            table_hint = static_np;
        } else if (table_wanted && !per_head) {
            const int64_t x_p = (8 * (int64_t)p[0].s_inv + ((int64_t)1 << p[0].x_shift) - 1) >> p[0].x_shift;
            if (x_p + 16 <= kTableMaxBytes) table_hint = ((int)x_p + 1 + 15) & ~15;
        }
        // a table only pays while it is smaller than the Q, K, V, O bytes of the workgroup
        a.win_mode = 0;
        if (!qmax && qflash_plan_win(d, kv_tile, lds_limit, table_hint, &a) == 0 && table_hint > 0)
            qflash_plan_win(d, kv_tile, lds_limit, 0, &a);
        if (qmax || a.win_mode) a.cu_mode = 0;          // (the whole-compute-unit kernel exists for Algorithm 1 only)
        else if (!qflash_plan_cu(B * H, N, d, kv_tile, lds_limit, table_hint, &a) && table_hint > 0)
            qflash_plan_cu(B * H, N, d, kv_tile, lds_limit, 0, &a);
    }
    // wave priority by dispatch round: only for launches of two to four rounds (0 = off)
    if (a.n_units <= n_cu || a.n_units > 4 * n_cu) a.n_cu = 0;

    int cur = -1;
    if (hipGetDevice(&cur) != hipSuccess) { (void)hipGetLastError(); return QFLASH_ERR_DEVICE; }
    if (cur != device && hipSetDevice(device) != hipSuccess) {
        (void)hipGetLastError();
        return QFLASH_ERR_DEVICE;
    }
    // Look-up mode: find (or build, once, on this stream) the weight table of each set of
    // constants.  A head gets one if it is small enough and the largest of them fits LDS beside K
    // and V.  If every head has one the whole launch runs in table mode; if only some have, each
    // workgroup chooses by its head; otherwise the launch is arithmetic.  Workgroups that serve several pairs share one
    // table: with per-head constants their pairs are therefore one head of consecutive batch elements.
    int rc = 0;
    if (hc_dev) {
        // Constants made on the GPU: so is the table, by the quantising kernel ahead of this one on
        // the stream, which also decides whether there is one (mode 3 reads that decision per
        // workgroup; without mode 3 the table is simply not looked at).
        const bool use_table = table_wanted;
        if (use_table && dyn_table && a.resident && table_fits(a, d, kTableMaxBytes, lds_limit)) {
            a.exp_mode = 3;
            a.lut_bytes_max = kTableMaxBytes;
        }
    } else if (static_table) {
        // One table, rebuilt by every call in the static device array ahead of the attention kernel
        // on the same stream (the array keeps the last call's table and every byte the kernel
        // stages, [0, static_np), is rewritten).  No lock: nothing of the context is touched.
        if (static_np > 0 && a.resident && table_fits(a, d, static_np, lds_limit)) {
            rc = qflash_launch_build_table(scratch_ptr, static_xp + 1, static_np, static_xp, a.hc[0], hip_stream);
            a.hc[0].lut = scratch_ptr;
            a.hc[0].lut_bytes = static_np;
            a.hc[0].lut_xp = static_xp;
            a.exp_mode = 2;
            a.lut_bytes_max = static_np;
        }
    } else {
        // The context's lock is held until the attention kernel has been enqueued: a slot this launch
        // reads must not be handed to other constants by another host thread in between.
        std::unique_lock<std::mutex> lk(ctx->mu);
        const bool allowed = ctx->use_table && ctx->tables && a.resident && !(per_head && a.heads_per_wg > 1 && !a.same_head);
        // A stream under capture records the kernels instead of running them: a table built now would
        // be read, by eager launches with the same constants, before it has ever been written.  Such a
        // call only uses tables that already exist (and pins them, since the graph keeps reading them).
        bool capturing = false;
        {
            hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
            if (hipStreamIsCapturing((hipStream_t)hip_stream, &cs) != hipSuccess) { (void)hipGetLastError(); capturing = true; }
            else capturing = cs != hipStreamCaptureStatusNone;
        }
        const uint64_t now = ++ctx->launches;
        int xp[kQflashMaxParamHeads], np_[kQflashMaxParamHeads], max_bytes = 0, n_with = 0;
        bool has[kQflashMaxParamHeads];
        for (int h = 0; h < n_p; ++h) {
            // weight is 0 at and below -8 octaves: x_p = ceil(8 s_inv / 2^k)
            const int64_t x_p = (8 * (int64_t)p[h].s_inv + ((int64_t)1 << p[h].x_shift) - 1) >> p[h].x_shift;
            xp[h] = (int)x_p;
            np_[h] = ((int)x_p + 1 + 15) & ~15;
            has[h] = allowed && x_p + 16 <= kTableMaxBytes;
            if (has[h] && np_[h] > max_bytes) max_bytes = np_[h];
        }
        if (max_bytes == 0 || !table_fits(a, d, max_bytes, lds_limit))
            for (int h = 0; h < n_p; ++h) has[h] = false;
        for (int h = 0; rc == 0 && h < n_p; ++h) {
            if (!has[h]) continue;
            const int32_t key[5] = {p[h].x_shift, p[h].s_inv, p[h].exp_mul, p[h].p_mul, p[h].p_shift};
            int slot = -1;
            for (int i = 0; i < ctx->n_slots; ++i)
                if (ctx->slots[i].stream == hip_stream && std::memcmp(ctx->slots[i].key, key, sizeof key) == 0) {
                    slot = i;
                    break;
                }
            if (slot < 0 && !capturing) {
                int victim = -1;
                if (ctx->n_slots < kTableSlots) {
                    victim = ctx->n_slots;
                } else if (ctx->evict_ev) {
                    // least recently used slot that no graph reads and this launch does not need
                    for (int i = 0; i < kTableSlots; ++i)
                        if (!ctx->slots[i].pinned && ctx->slots[i].last_use < now &&
                            (victim < 0 || ctx->slots[i].last_use < ctx->slots[victim].last_use))
                            victim = i;
                    if (victim >= 0) {
                        // the builder must not overtake the launches that still read the old table
                        bool ordered = ctx->slots[victim].stream == hip_stream;
                        if (!ordered) {
                            hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
                            const hipStream_t old = (hipStream_t)ctx->slots[victim].stream;
                            if (hipStreamIsCapturing(old, &cs) == hipSuccess && cs == hipStreamCaptureStatusNone &&
                                hipEventRecord(ctx->evict_ev, old) == hipSuccess &&
                                hipStreamWaitEvent((hipStream_t)hip_stream, ctx->evict_ev, 0) == hipSuccess)
                                ordered = true;
                            else
                                (void)hipGetLastError();
                        }
                        if (!ordered) victim = -1;
                        else ++ctx->evictions;
                    }
                }
                if (victim >= 0) {
                    // The builder is enqueued under the lock, so no other host thread can enqueue a
                    // reader of this slot on the same stream ahead of it.
                    uint8_t* tbl = ctx->tables + (size_t)victim * kTableMaxBytes;
                    rc = qflash_launch_build_table(tbl, xp[h] + 1, np_[h], xp[h], a.hc[h], hip_stream);
                    if (rc == 0) {
                        slot = victim;
                        if (victim == ctx->n_slots) ++ctx->n_slots;
                        TableSlot& t = ctx->slots[slot];
                        std::memcpy(t.key, key, sizeof key);
                        t.stream = hip_stream; t.n = xp[h] + 1; t.n_padded = np_[h]; t.x_p = xp[h];
                        t.pinned = false;
                    }
                }
            }
            if (slot < 0) { has[h] = false; continue; }     // no slot to be had: this head computes
            ctx->slots[slot].last_use = now;
            if (capturing) ctx->slots[slot].pinned = true;
            a.hc[h].lut = ctx->tables + (size_t)slot * kTableMaxBytes;
            a.hc[h].lut_bytes = np_[h];
            a.hc[h].lut_xp = xp[h];
            ++n_with;
        }
        if (rc == 0 && n_with == n_p) {
            a.exp_mode = 2;
            a.lut_bytes_max = max_bytes;
        } else if (rc == 0 && n_with > 0) {
            a.exp_mode = 3;
            a.lut_bytes_max = max_bytes;
        } else {
            for (int h = 0; h < n_p; ++h) { a.hc[h].lut = nullptr; a.hc[h].lut_bytes = 0; a.hc[h].lut_xp = 0; }
        }
        if (rc == 0) rc = launch_attention(a, d, kv_tile, lds_limit, hip_stream);
        ctx->last_mode = a.exp_mode == 2 ? QFLASH_WEIGHTS_TABLE : a.exp_mode == 3 ? QFLASH_WEIGHTS_MIXED : QFLASH_WEIGHTS_ARITHMETIC;
        ctx->last_kernel = a.win_mode ? 4 : a.cu_mode ? 3 : !a.resident ? 0 : a.ring ? 2 : 1;   // (2 also for the direct-load ring)
        lk.unlock();
        if (cur != device) (void)hipSetDevice(cur);
        if (rc != 0) { (void)hipGetLastError(); return QFLASH_ERR_LAUNCH; }
        return QFLASH_OK;
    }
    if (rc == 0) rc = launch_attention(a, d, kv_tile, lds_limit, hip_stream);
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

extern "C" int qflash_attention_static(qflash_ctx* ctx, const int8_t* Q, const int8_t* K, const int8_t* V,
                                       int8_t* O, const int32_t* bias, int bias_B, int bias_H, int B, int H,
                                       int N, int d, int kv_tile, const qflash_params* p, void* hip_stream) {
    return attention_impl(ctx, Q, K, V, O, bias, bias_B, bias_H, B, H, N, d, kv_tile, p, false, hip_stream,
                          nullptr, 0, false, nullptr, true);
}

extern "C" int qflash_attention_per_head(qflash_ctx* ctx, const int8_t* Q, const int8_t* K, const int8_t* V,
                                         int8_t* O, const int32_t* bias, int bias_B, int bias_H, int B,
                                         int H, int N, int d, int kv_tile, const qflash_params* p,
                                         void* hip_stream) {
    return attention_impl(ctx, Q, K, V, O, bias, bias_B, bias_H, B, H, N, d, kv_tile, p, true, hip_stream);
}

extern "C" int qflash_plan_query(qflash_ctx* ctx, int B, int H, int N, int d, int kv_tile, int bias_B,
                                 int bias_H, qflash_plan_info* out) {
    if (!out) return QFLASH_ERR_NULL;
    int lds_limit = 160 * 1024, n_cu = 256;
    bool qmax = false;
    if (ctx) {
        {
            std::lock_guard<std::mutex> lk(g_mu);
            if (live_contexts().find(ctx) == live_contexts().end()) return QFLASH_ERR_CTX;
            lds_limit = ctx->lds_limit;
            n_cu = ctx->n_cu;
        }
        std::lock_guard<std::mutex> lk(ctx->mu);
        qmax = ctx->qmax != 0;
    }
    if (d != 32 && d != 64) return QFLASH_ERR_SHAPE;
    if (B < 1 || H < 1 || N < 1 || N > QFLASH_MAX_N) return QFLASH_ERR_SHAPE;
    if ((int64_t)B * H * N * d >= ((int64_t)1 << 31)) return QFLASH_ERR_SHAPE;
    if (kv_tile != 64 && kv_tile != 128) return QFLASH_ERR_TILE;
    const bool has_bias = bias_B != 0 || bias_H != 0;
    if (has_bias && (bias_B < 1 || bias_H < 1)) return QFLASH_ERR_SHAPE;
    QflashKernelArgs a;
    std::memset(&a, 0, sizeof a);
    static const int32_t some_bias = 0;
    a.bias = has_bias ? &some_bias : nullptr;    // the plan only asks whether there is one
    a.bias_B = has_bias ? bias_B : 1;
    a.bias_H = has_bias ? bias_H : 1;
    a.B = B; a.H = H; a.N = N;
    a.n_cu = n_cu;
    a.qmax = qmax ? 1 : 0;
    if (qflash_plan_fwd(B * H, N, d, kv_tile, lds_limit, &a) != 0) return QFLASH_ERR_SHAPE;
    std::memset(out, 0, sizeof *out);
    a.bias_packed = has_bias ? 1 : 0;      // (a bias is taken to be in the packed layout, the only one kernel 4 reads)
    if (!qmax && qflash_plan_win(d, kv_tile, lds_limit, kPlanQueryTableBytes, &a)) {
        out->kernel = 4;
        out->pairs_per_workgroup = a.win_streams * a.win_chunk;
        out->wavefronts_per_pair = 2;
        out->query_blocks = 2;
        out->units = a.win_groups;
        out->workgroups = a.win_groups;
        return QFLASH_OK;
    }
    if (!qmax && qflash_plan_cu(B * H, N, d, kv_tile, lds_limit, kPlanQueryTableBytes, &a)) {
        out->kernel = 3;
        out->pairs_per_workgroup = a.cu_heads;
        out->wavefronts_per_pair = a.cu_waves;
        out->query_blocks = (N + 31) / 32;
        out->units = a.cu_groups;
        out->workgroups = a.cu_groups;
        return QFLASH_OK;
    }
    out->kernel = !a.resident ? 0 : a.ring ? 2 : 1;
    out->pairs_per_workgroup = a.heads_per_wg;
    out->wavefronts_per_pair = a.waves_per_head;
    out->query_blocks = a.n_qtiles;
    out->units = a.n_units;
    out->workgroups = 8 * a.units_per_xcd;
    out->tile_by_tile = a.resident && a.pipelined && d == 64 && (kv_tile == 64 || N > 256) ? 1 : 0;
    out->bias_period_units = a.xcd_period;
    out->units_per_xcd = a.units_per_xcd;
    return QFLASH_OK;
}

extern "C" int qflash_cache_query(qflash_ctx* ctx, qflash_cache_info* out) {
    if (!ctx || !out) return QFLASH_ERR_NULL;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        if (live_contexts().find(ctx) == live_contexts().end()) return QFLASH_ERR_CTX;
    }
    std::lock_guard<std::mutex> lk(ctx->mu);
    std::memset(out, 0, sizeof *out);
    out->slots_total = ctx->tables ? kTableSlots : 0;
    out->slots_in_use = ctx->n_slots;
    for (int i = 0; i < ctx->n_slots; ++i) out->slots_pinned += ctx->slots[i].pinned ? 1 : 0;
    out->evictions = ctx->evictions;
    out->last_weight_mode = ctx->last_mode;
    out->last_kernel = ctx->last_kernel;
    return QFLASH_OK;
}

extern "C" int qflash_plan_unit(const qflash_plan_info* plan, int workgroup) {
    if (!plan || workgroup < 0 || workgroup >= plan->workgroups) return -1;
    if (plan->kernel == 3 || plan->kernel == 4) return workgroup;
    const int unit = qflash_unit_of_workgroup(workgroup, plan->units_per_xcd, plan->bias_period_units);
    return unit < plan->units ? unit : -1;
}

extern "C" size_t qflash_packed_bias_bytes(int bias_B, int bias_H, int N) {
    if (bias_B < 1 || bias_H < 1 || N < 1 || N > QFLASH_MAX_N) return 0;
    if ((int64_t)bias_B * bias_H * N * N >= ((int64_t)1 << 31)) return 0;
    const long long words = qflash_packed_bias_words(bias_B * bias_H, N);
    if (words >= ((int64_t)1 << 29)) return 0;
    return (size_t)words * 16;
}

extern "C" int qflash_pack_bias(qflash_ctx* ctx, const int32_t* bias, int bias_B, int bias_H, int N,
                                int32_t* packed, size_t packed_bytes, void* hip_stream) {
    if (!ctx) return QFLASH_ERR_NULL;
    int device;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        if (live_contexts().find(ctx) == live_contexts().end()) return QFLASH_ERR_CTX;
        device = ctx->device;
    }
    if (!bias || !packed) return QFLASH_ERR_NULL;
    const size_t need = qflash_packed_bias_bytes(bias_B, bias_H, N);
    if (need == 0) return QFLASH_ERR_SHAPE;
    if (packed_bytes < need) return QFLASH_ERR_SHAPE;
    if (((uintptr_t)bias & 3u) || ((uintptr_t)packed & 15u)) return QFLASH_ERR_ALIGN;
    int cur = -1;
    if (hipGetDevice(&cur) != hipSuccess) { (void)hipGetLastError(); return QFLASH_ERR_DEVICE; }
    if (cur != device && hipSetDevice(device) != hipSuccess) {
        (void)hipGetLastError();
        return QFLASH_ERR_DEVICE;
    }
    const int rc = qflash_launch_pack_bias(bias, bias_B * bias_H, N, packed, hip_stream);
    if (cur != device) (void)hipSetDevice(cur);
    if (rc != 0) { (void)hipGetLastError(); return QFLASH_ERR_LAUNCH; }
    return QFLASH_OK;
}

extern "C" int qflash_attention_packed_bias(qflash_ctx* ctx, const int8_t* Q, const int8_t* K, const int8_t* V,
                                            int8_t* O, const int32_t* packed_bias, int bias_B, int bias_H,
                                            int B, int H, int N, int d, int kv_tile, const qflash_params* p,
                                            int n_params, void* hip_stream) {
    if (n_params != 1 && n_params != H) return QFLASH_ERR_PARAM;
    if (!packed_bias) return QFLASH_ERR_NULL;
    return attention_impl(ctx, Q, K, V, O, packed_bias, bias_B, bias_H, B, H, N, d, kv_tile, p,
                          n_params == H && H > 1, hip_stream, nullptr, 0, true);
}

// Workspace layout of the dynamic entry point: [int8 Q | int8 K | int8 V | constants | abs-max scratch | weight table]
namespace {
size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
size_t dyn_scratch_bytes(size_t n) {     // partial maxima of the abs-max kernel
    return align256(sizeof(float) * (4 + 3 * (size_t)qflash_dynamic_partials((long long)n)));
}
}

extern "C" size_t qflash_dynamic_workspace_bytes(int B, int H, int N, int d) {
    if (B < 1 || H < 1 || N < 1 || d < 1) return 0;
    const size_t n = (size_t)B * H * N * d;
    return 3 * align256(n) + align256(sizeof(QflashHeadConsts)) + dyn_scratch_bytes(n) + align256(kTableMaxBytes);
}

namespace {

int dynamic_impl(qflash_ctx* ctx, const float* Qf, const float* Kf, const float* Vf, int8_t* O, const float* bias_real,
                 const uint8_t* excluded, int bias_B, int bias_H, int B, int H, int N, int d, int kv_tile, int out_round,
                 qflash_dynamic_info* info, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!ctx) return QFLASH_ERR_NULL;
    int device, lds_limit, n_cu;
    {
        std::lock_guard<std::mutex> lk(g_mu);
        if (live_contexts().find(ctx) == live_contexts().end()) return QFLASH_ERR_CTX;
        device = ctx->device;
        lds_limit = ctx->lds_limit;
        n_cu = ctx->n_cu;
    }
    const bool with_bias = bias_real || excluded;
    if (!Qf || !Kf || !Vf || !O || !workspace) return QFLASH_ERR_NULL;
    if (d != 32 && d != 64) return QFLASH_ERR_SHAPE;
    if (B < 1 || H < 1 || N < 1 || N > QFLASH_MAX_N) return QFLASH_ERR_SHAPE;
    if ((int64_t)B * H * N * d >= ((int64_t)1 << 31)) return QFLASH_ERR_SHAPE;
    size_t need = qflash_dynamic_workspace_bytes(B, H, N, d);
    if (with_bias) {
        if (bias_B < 1 || bias_H < 1) return QFLASH_ERR_SHAPE;
        if ((int64_t)bias_B * bias_H * N * N >= ((int64_t)1 << 31)) return QFLASH_ERR_SHAPE;
        if (qflash_packed_bias_words(bias_B * bias_H, N) >= ((int64_t)1 << 29)) return QFLASH_ERR_SHAPE;
        need = qflash_dynamic_bias_workspace_bytes(B, H, N, d, bias_B, bias_H);
    }
    if (need == 0 || workspace_bytes < need) return QFLASH_ERR_SHAPE;
    if (kv_tile != 64 && kv_tile != 128) return QFLASH_ERR_TILE;
    if (out_round != 0 && out_round != 1) return QFLASH_ERR_PARAM;
    if (((uintptr_t)Qf | (uintptr_t)Kf | (uintptr_t)Vf | (uintptr_t)O | (uintptr_t)workspace) & 15u) return QFLASH_ERR_ALIGN;
    if (bias_real && ((uintptr_t)bias_real & 3u)) return QFLASH_ERR_ALIGN;
    if (info && ((uintptr_t)info & 7u)) return QFLASH_ERR_ALIGN;
    {
        // everything the attention launch would refuse is refused here, before the quantising kernels
        // are enqueued
        static const int32_t some_bias = 0;
        QflashKernelArgs probe;
        std::memset(&probe, 0, sizeof probe);
        probe.B = B; probe.H = H; probe.N = N; probe.n_cu = n_cu;
        probe.bias = with_bias ? &some_bias : nullptr;
        probe.bias_B = with_bias ? bias_B : 1;
        probe.bias_H = with_bias ? bias_H : 1;
        if (qflash_plan_fwd(B * H, N, d, kv_tile, lds_limit, &probe) != 0) return QFLASH_ERR_SHAPE;
    }

    const size_t n = (size_t)B * H * N * d;        // a multiple of 32
    int8_t* ws = (int8_t*)workspace;
    int8_t* Qo = ws;
    int8_t* Ko = Qo + align256(n);
    int8_t* Vo = Ko + align256(n);
    QflashHeadConsts* hc_dev = (QflashHeadConsts*)(Vo + align256(n));
    float* scratch = (float*)((int8_t*)hc_dev + align256(sizeof(QflashHeadConsts)));
    uint8_t* dyn_table = (uint8_t*)scratch + dyn_scratch_bytes(n);    // kTableMaxBytes: a weight table made on the GPU
    int32_t* packed = (int32_t*)(ws + qflash_dynamic_workspace_bytes(B, H, N, d));   // with_bias only

    int cur = -1;
    if (hipGetDevice(&cur) != hipSuccess) { (void)hipGetLastError(); return QFLASH_ERR_DEVICE; }
    if (cur != device && hipSetDevice(device) != hipSuccess) {
        (void)hipGetLastError();
        return QFLASH_ERR_DEVICE;
    }
    int rc = qflash_launch_dynamic_front(Qf, Kf, Vf, Qo, Ko, Vo, (long long)n, std::sqrt((double)d), out_round,
                                         scratch, hc_dev, info, dyn_table, kTableMaxBytes, hip_stream);
    if (rc == 0 && with_bias)
        rc = qflash_launch_dynamic_bias(bias_real, excluded, bias_B * bias_H, N, packed, scratch, (long long)n,
                                        std::sqrt((double)d), hip_stream);
    if (cur != device) (void)hipSetDevice(cur);
    if (rc != 0) { (void)hipGetLastError(); return QFLASH_ERR_LAUNCH; }
    return attention_impl(ctx, Qo, Ko, Vo, O, with_bias ? packed : nullptr, with_bias ? bias_B : 0, with_bias ? bias_H : 0,
                          B, H, N, d, kv_tile, nullptr, false, hip_stream, hc_dev, out_round, with_bias, dyn_table);
}

}  // namespace

extern "C" int qflash_attention_dynamic(qflash_ctx* ctx, const float* Qf, const float* Kf, const float* Vf,
                                        int8_t* O, int B, int H, int N, int d, int kv_tile, int out_round,
                                        qflash_dynamic_info* info, void* workspace, size_t workspace_bytes,
                                        void* hip_stream) {
    return dynamic_impl(ctx, Qf, Kf, Vf, O, nullptr, nullptr, 0, 0, B, H, N, d, kv_tile, out_round, info, workspace,
                        workspace_bytes, hip_stream);
}

extern "C" size_t qflash_dynamic_bias_workspace_bytes(int B, int H, int N, int d, int bias_B, int bias_H) {
    const size_t base = qflash_dynamic_workspace_bytes(B, H, N, d);
    if (base == 0 || bias_B < 1 || bias_H < 1) return 0;
    if ((int64_t)bias_B * bias_H * N * N >= ((int64_t)1 << 31)) return 0;
    const long long words = qflash_packed_bias_words(bias_B * bias_H, N);
    if (words >= (1ll << 29)) return 0;
    return base + 16 * (size_t)words;
}

extern "C" int qflash_attention_dynamic_bias(qflash_ctx* ctx, const float* Qf, const float* Kf, const float* Vf,
                                             int8_t* O, const float* bias_real, const uint8_t* excluded, int bias_B,
                                             int bias_H, int B, int H, int N, int d, int kv_tile, int out_round,
                                             qflash_dynamic_info* info, void* workspace, size_t workspace_bytes,
                                             void* hip_stream) {
    if (!bias_real && !excluded) return QFLASH_ERR_NULL;
    return dynamic_impl(ctx, Qf, Kf, Vf, O, bias_real, excluded, bias_B, bias_H, B, H, N, d, kv_tile, out_round, info,
                        workspace, workspace_bytes, hip_stream);
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
        case QFLASH_ERR_SCRATCH: return "the weight table of these constants exceeds the static device memory of qflash_attention_static";
        default: return "unknown qflash error code";
    }
}
