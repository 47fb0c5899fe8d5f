// Sanitizer harness (CPU only): exercises the host-only translation unit of the library
// (constants from scales, argument checks, kernel plan) and the plain-C oracle under
// -fsanitize=address,undefined.  Built and run by tests/test_sanitizers.py:
//
//   gcc -std=c11 -O1 -g -fsanitize=address,undefined -fno-sanitize-recover=all -fopenmp -c oracle/qflash_oracle.c
//   g++ -std=c++17 -O1 -g -fsanitize=address,undefined -fno-sanitize-recover=all -fopenmp
//       -I include -I paper_2604_25306_amd/csrc tests/sanitize/host_sanitize.cpp
//       paper_2604_25306_amd/csrc/qflash_plan.cpp qflash_oracle.o -o host_sanitize && ./host_sanitize
//
// Every check is an invariant the code under test must keep for any input; a sanitizer report or a
// failed check ends the program with a non-zero status.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <limits>
#include <random>
#include <vector>

#include "qflash.h"
#include "qflash_internal.h"
#include "qflash_derive.h"

extern "C" {
typedef struct {
    int32_t x_shift, s_inv, exp_mul, exp_shift, p_mul, p_shift, a_mul, out_round;
} oracle_params;
int64_t oracle_shift_exp2(int64_t x, const oracle_params* p);
int64_t oracle_shift_exp2_scaled(int64_t xs, const oracle_params* p);
int64_t oracle_qmax_level(int64_t t, const oracle_params* p);
int64_t oracle_requant(int64_t y, const oracle_params* p);
int64_t oracle_alpha16(int64_t alpha_hat, const oracle_params* p);
int64_t oracle_scale_release(int64_t acc, int64_t alpha16);
int oracle_qflash_attention(const int8_t*, const int8_t*, const int8_t*, int8_t*, const int32_t*, int, int, int, int, int,
                            int, int, const oracle_params*, int64_t*, int64_t*, int64_t*, int64_t*, int);
int oracle_qflash_attention_per_head(const int8_t*, const int8_t*, const int8_t*, int8_t*, const int32_t*, int, int, int,
                                     int, int, int, int, const oracle_params*, int64_t*, int64_t*, int64_t*, int64_t*, int);
int oracle_qflash_attention_qmax(const int8_t*, const int8_t*, const int8_t*, int8_t*, const int32_t*, int, int, int, int,
                                 int, int, int, const oracle_params*, int64_t*, int64_t*, int64_t*, int64_t*, int);
}

static long g_checks = 0;
#define CHECK(cond)                                                                      \
    do {                                                                                 \
        ++g_checks;                                                                      \
        if (!(cond)) {                                                                   \
            std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
            std::exit(1);                                                                \
        }                                                                                \
    } while (0)

static oracle_params to_oracle(const qflash_params& p) {
    return oracle_params{p.x_shift, p.s_inv, p.exp_mul, p.exp_shift, p.p_mul, p.p_shift, p.a_mul, p.out_round};
}

static void constants_from_scales() {
    const double inf = std::numeric_limits<double>::infinity(), nan = std::numeric_limits<double>::quiet_NaN();
    qflash_params p;
    CHECK(qflash_params_from_scales(0.03, 0.03, 0.02, 64, nullptr) == QFLASH_ERR_NULL);
    CHECK(qflash_params_from_scales(0.03, 0.03, 0.02, 48, &p) == QFLASH_ERR_SHAPE);
    for (double bad : {0.0, -1.0, inf, nan}) {
        CHECK(qflash_params_from_scales(bad, 0.03, 0.02, 64, &p) == QFLASH_ERR_PARAM);
        CHECK(qflash_params_from_scales(0.03, bad, 0.02, 64, &p) == QFLASH_ERR_PARAM);
        CHECK(qflash_params_from_scales(0.03, 0.03, bad, 64, &p) == QFLASH_ERR_PARAM);
    }
    int ok = 0, refused = 0;
    for (int d : {32, 64})
        for (double e = -12.0; e <= 12.0; e += 0.037) {
            const double s = std::pow(2.0, e);
            const int rc = qflash_params_from_scales(s, 1.0, 1.0, d, &p);
            CHECK(rc == QFLASH_OK || rc == QFLASH_ERR_PARAM);
            if (rc != QFLASH_OK) { ++refused; continue; }
            ++ok;
            CHECK(qflash_params_ok(p));
            CHECK(p.s_inv >= 1024 && p.s_inv < (1 << 18) && p.x_shift >= 0 && p.x_shift <= 13 && p.exp_mul < 0);
            QflashHeadConsts hc;
            CHECK(qflash_fill_head_consts(p, &hc));
            CHECK(hc.x_floor <= 0);
            // the oracle's scalar functions on these constants: range and monotonicity
            const oracle_params op = to_oracle(p);
            int64_t prev = -1;
            for (int64_t x = -((int64_t)40 * p.s_inv >> p.x_shift); x <= 0; x += 1 + (p.s_inv >> (p.x_shift + 3))) {
                const int64_t y = oracle_shift_exp2(x, &op);
                CHECK(y >= 0 && y <= p.s_inv && y >= prev - 1);
                prev = y;
                const int64_t w = oracle_requant(y, &op);
                CHECK(w >= 0 && w <= 127);
                CHECK(oracle_alpha16(y, &op) <= 65536);
                CHECK(oracle_shift_exp2_scaled(x * ((int64_t)1 << p.x_shift), &op) == y);
            }
            CHECK(oracle_shift_exp2(-(1 << 22), &op) == 0);
            const int64_t L = oracle_qmax_level(-(1 << 21), &op);
            CHECK(L * p.s_inv >= -((int64_t)1 << (21 + p.x_shift)) && (L - 1) * p.s_inv < -((int64_t)1 << (21 + p.x_shift)));
        }
    CHECK(ok > 100 && refused > 10);
    CHECK(oracle_scale_release(-1, 65535) == -1 && oracle_scale_release(-(1 << 26), 65536) == -(1 << 26));
}

static void argument_checks() {
    qflash_params p;
    CHECK(qflash_params_from_scales(0.03, 0.03, 0.02, 64, &p) == QFLASH_OK);
    alignas(16) static int8_t buf[64];
    alignas(16) static int32_t bias[4];
    const void* q = buf;
    auto call = [&](const void* Q, const void* O, const int32_t* b, int bB, int bH, bool packed, int B, int H, int N, int d,
                    int tile, const qflash_params* pp, bool per_head, bool dev, bool qmax) {
        return qflash_check_call(Q, q, q, O, b, bB, bH, packed, B, H, N, d, tile, pp, per_head, dev, qmax);
    };
    CHECK(call(q, q, nullptr, 0, 0, false, 1, 1, 1, 64, 64, &p, false, false, false) == QFLASH_OK);
    CHECK(call(nullptr, q, nullptr, 0, 0, false, 1, 1, 1, 64, 64, &p, false, false, false) == QFLASH_ERR_NULL);
    CHECK(call(q, q, nullptr, 0, 0, false, 1, 1, 1, 64, 64, nullptr, false, false, false) == QFLASH_ERR_NULL);
    CHECK(call(q, q, nullptr, 0, 0, false, 1, 1, 1, 64, 64, nullptr, false, true, false) == QFLASH_OK);
    CHECK(call(q, q, nullptr, 0, 0, true, 1, 1, 1, 64, 64, &p, false, false, false) == QFLASH_ERR_NULL);
    CHECK(call(q, q, nullptr, 0, 0, false, 1, 1, 1, 48, 64, &p, false, false, false) == QFLASH_ERR_SHAPE);
    CHECK(call(q, q, nullptr, 0, 0, false, 0, 1, 1, 64, 64, &p, false, false, false) == QFLASH_ERR_SHAPE);
    CHECK(call(q, q, nullptr, 0, 0, false, 1, 1, QFLASH_MAX_N + 1, 64, 64, &p, false, false, false) == QFLASH_ERR_SHAPE);
    CHECK(call(q, q, nullptr, 0, 0, false, 1 << 15, 1 << 6, 4096, 64, 64, &p, false, false, false) == QFLASH_ERR_SHAPE);
    CHECK(call(q, q, nullptr, 0, 0, false, 1, QFLASH_MAX_PARAM_HEADS + 1, 8, 64, 64, &p, true, false, false) == QFLASH_ERR_SHAPE);
    CHECK(call(q, q, bias, 0, 1, false, 1, 1, 1, 64, 64, &p, false, false, false) == QFLASH_ERR_SHAPE);
    CHECK(call(q, q, bias, 1 << 10, 1 << 10, false, 1, 1, 4096, 64, 64, &p, false, false, false) == QFLASH_ERR_SHAPE);
    CHECK(call(q, q, bias, 1, 1, false, 1, 1, 1, 64, 96, &p, false, false, false) == QFLASH_ERR_TILE);
    CHECK(call(buf + 1, q, nullptr, 0, 0, false, 1, 1, 1, 64, 64, &p, false, false, false) == QFLASH_ERR_ALIGN);
    CHECK(call(q, q, (const int32_t*)((const char*)bias + 4), 1, 1, true, 1, 1, 1, 64, 64, &p, false, false, false) == QFLASH_ERR_ALIGN);
    CHECK(call(q, q, (const int32_t*)((const char*)bias + 4), 1, 1, false, 1, 1, 1, 64, 64, &p, false, false, false) == QFLASH_OK);
    qflash_params bad = p;
    bad.s_inv = 17;
    CHECK(call(q, q, nullptr, 0, 0, false, 1, 1, 1, 64, 64, &bad, false, false, false) == QFLASH_ERR_PARAM);
    qflash_params two[2] = {p, p};
    two[1].out_round = 1;
    CHECK(call(q, q, nullptr, 0, 0, false, 1, 2, 1, 64, 64, two, true, false, false) == QFLASH_ERR_PARAM);
    qflash_params coarse;
    CHECK(qflash_params_from_scales(3.0, 4.0, 1.0, 64, &coarse) == QFLASH_OK && coarse.x_shift > 0);
    CHECK(call(q, q, nullptr, 0, 0, false, 1, 1, 1, 64, 64, &coarse, false, false, false) == QFLASH_OK);
    CHECK(call(q, q, nullptr, 0, 0, false, 1, 1, 1, 64, 64, &coarse, false, false, true) == QFLASH_ERR_PARAM);
}

// Every unit of work is handed to exactly one workgroup of the launch grid.
static void grid_covers_units(const QflashKernelArgs& a) {
    std::vector<char> seen((size_t)a.n_units, 0);
    const int grid = 8 * a.units_per_xcd;
    for (int wg = 0; wg < grid; ++wg) {
        const int u = qflash_unit_of_workgroup(wg, a.units_per_xcd, a.xcd_period);
        CHECK(u >= 0);
        if (u < a.n_units) {
            CHECK(!seen[(size_t)u]);
            seen[(size_t)u] = 1;
        }
    }
    for (char c : seen) CHECK(c);
}

static void kernel_plans() {
    const int lds = 160 * 1024;
    static const int32_t some_bias = 0;
    std::mt19937 rng(7);
    long plans = 0;
    auto one = [&](int B, int H, int N, int d, int tile, int bias_B, int bias_H, bool per_head, int n_cu) {
        QflashKernelArgs a;
        std::memset(&a, 0, sizeof a);
        a.bias = bias_B ? &some_bias : nullptr;
        a.bias_B = bias_B ? bias_B : 1;
        a.bias_H = bias_B ? bias_H : 1;
        a.B = B; a.H = H; a.N = N;
        a.per_head = per_head;
        a.n_cu = n_cu;
        const int rc = qflash_plan_fwd(B * H, N, d, tile, lds, &a);
        CHECK(rc == 0 || (long long)B * H * ((N + 31) / 32) >= (1ll << 30));
        if (rc != 0) return;
        ++plans;
        CHECK(a.waves_per_head >= 1 && a.waves_per_head <= kResidentMaxWavesWide);
        CHECK(a.heads_per_wg >= 1 && a.heads_per_wg * a.waves_per_head <= kResidentMaxWavesWide);
        CHECK(a.rows_per_wg == 32 * a.waves_per_head && (long long)a.rows_per_wg * a.n_qtiles >= N);
        CHECK(a.heads_per_wg == 1 || a.n_qtiles == 1);
        CHECK(!a.ring || (a.pipelined && d == 64 && a.heads_per_wg == 1 && (a.waves_per_head >= 4 || a.ring_dma)));
        CHECK(!a.ring_dma || (a.ring && !a.bias && a.waves_per_head <= 4 &&
                              qflash_ring_lds_bytes(a.waves_per_head, tile, 40 * 1024) <= (size_t)lds));
        CHECK(!a.pipelined || (a.resident && (a.waves_per_head >= 4 || a.ring_dma) && N > tile));
        if (a.resident) {
            const size_t bytes = a.ring_dma ? qflash_ring_lds_bytes(a.waves_per_head, tile, 0)
                                            : qflash_resident_lds_bytes(N, d, a.heads_per_wg, 0, lds, a.ring ? tile : 0);
            CHECK(bytes > 0 && bytes <= (size_t)lds);
        }
        const long long pairs = (long long)B * H;
        const long long served = a.same_head ? (long long)a.n_units / H * a.heads_per_wg * H
                                 : a.heads_per_wg > 1 ? (long long)a.n_units * a.heads_per_wg : (long long)a.n_units / a.n_qtiles;
        CHECK(served >= pairs);
        CHECK(a.xcd_period == 0 || (a.xcd_period % 8 == 0 && a.bias != nullptr));
        if (a.n_units <= (1 << 16)) grid_covers_units(a);
        for (int table : {0, 4096, 29 * 1024, 40 * 1024}) {
            const int fits = qflash_table_fits(a, d, table, lds);
            CHECK(fits == 0 || fits == 1);
            QflashKernelArgs c = a;
            if (qflash_plan_cu(B * H, N, d, tile, lds, table, &c)) {
                CHECK(d == 64 && tile == 64 && !c.bias && !c.per_head && N <= 256);
                CHECK((long long)c.cu_heads * c.cu_groups >= pairs && (long long)(c.cu_heads - 1) * c.cu_groups < pairs + c.cu_groups);
                CHECK(c.cu_groups <= (n_cu > 0 ? n_cu : 256) && c.cu_waves >= 1 && c.cu_waves <= 16);
                CHECK(qflash_cu_lds_bytes(N, c.cu_heads, table) <= (size_t)lds && c.cu_table_lds >= table);
            } else {
                CHECK(c.cu_mode == 0);
            }
        }
    };
    for (int d : {32, 64})
        for (int tile : {64, 128})
            for (int N : {1, 5, 31, 32, 33, 49, 64, 65, 127, 128, 129, 197, 255, 256, 257, 300, 577, 640, 1030, 2100, 4096})
                for (int BH : {1, 2, 3, 7, 8, 36, 255, 256, 257, 768, 769, 6144, 12288}) {
                    one(BH, 1, N, d, tile, 0, 0, false, 256);
                    one(1, BH > 64 ? 64 : BH, N, d, tile, 0, 0, true, 256);
                    one(BH, 3, N, d, tile, BH > 64 ? 64 : BH, 3, false, 256);
                    one(BH, 3, N, d, tile, 1, 1, true, 0);
                }
    for (int it = 0; it < 3000; ++it) {
        const int B = 1 + (int)(rng() % 300), H = 1 + (int)(rng() % 24), N = 1 + (int)(rng() % 4096);
        const int bB = (rng() & 1) ? 1 + (int)(rng() % B) : 0;
        one(B, H, N, (rng() & 1) ? 32 : 64, (rng() & 1) ? 64 : 128, bB, bB ? ((rng() & 1) ? H : 1) : 0, (rng() & 1) && H <= 64,
            (rng() & 1) ? 256 : 0);
    }
    CHECK(plans > 5000);
    CHECK(qflash_packed_bias_words(192, 49) == 192ll * 4 * 256);
}

static void oracle_runs() {
    std::mt19937 rng(11);
    for (int it = 0; it < 40; ++it) {
        const int B = 1 + (int)(rng() % 2), H = 1 + (int)(rng() % 3), N = 1 + (int)(rng() % 150), d = (rng() & 1) ? 32 : 64;
        const int tile = (rng() & 1) ? 64 : (rng() & 1) ? 128 : 16;
        const size_t n = (size_t)B * H * N * d;
        std::vector<int8_t> Q(n), K(n), V(n), O(n), O2(n);
        for (size_t i = 0; i < n; ++i) {
            Q[i] = (int8_t)((int)(rng() % 255) - 127);
            K[i] = (int8_t)((int)(rng() % 255) - 127);
            V[i] = (int8_t)((int)(rng() % 256) - 128);
        }
        std::vector<qflash_params> ps((size_t)H);
        std::vector<oracle_params> ops((size_t)H);
        for (int h = 0; h < H; ++h) {
            CHECK(qflash_params_from_scales(0.02 + 0.01 * h, 0.03, 0.02, d, &ps[(size_t)h]) == QFLASH_OK);
            ops[(size_t)h] = to_oracle(ps[(size_t)h]);
        }
        const bool with_bias = rng() & 1;
        const int bB = with_bias ? 1 + (int)(rng() % B) : 0, bH = with_bias ? ((rng() & 1) ? H : 1) : 0;
        std::vector<int32_t> bias(with_bias ? (size_t)bB * bH * N * N : 1);
        for (auto& b : bias) b = (rng() % 7 == 0) ? INT32_MIN : (int32_t)(rng() % 4001) - 2000;
        std::vector<int64_t> acc(n), l((size_t)B * H * N), m((size_t)B * H * N);
        int64_t viol = -1;
        CHECK(oracle_qflash_attention(Q.data(), K.data(), V.data(), O.data(), with_bias ? bias.data() : nullptr, bB, bH, B, H, N,
                                      d, tile, &ops[0], acc.data(), l.data(), m.data(), &viol, 2) == 0);
        CHECK(viol == 0);
        for (size_t i = 0; i < l.size(); ++i) CHECK(l[i] >= 0 && l[i] <= 127ll * N && m[i] >= -(1 << 21));
        CHECK(oracle_qflash_attention_per_head(Q.data(), K.data(), V.data(), O2.data(), with_bias ? bias.data() : nullptr, bB, bH,
                                               B, H, N, d, tile, ops.data(), nullptr, nullptr, nullptr, &viol, 1) == 0);
        CHECK(viol == 0);
        if (H == 1) CHECK(std::memcmp(O.data(), O2.data(), n) == 0);
        CHECK(oracle_qflash_attention_qmax(Q.data(), K.data(), V.data(), O2.data(), with_bias ? bias.data() : nullptr, bB, bH, B, H,
                                           N, d, tile, &ops[0], acc.data(), l.data(), m.data(), &viol, 0) == 0);
        CHECK(viol == 0);
    }
    int8_t x = 0;
    oracle_params op{};
    CHECK(oracle_qflash_attention(&x, &x, &x, &x, nullptr, 0, 0, 0, 1, 1, 32, 64, &op, nullptr, nullptr, nullptr, nullptr, 0) == -1);
    CHECK(oracle_qflash_attention(nullptr, &x, &x, &x, nullptr, 0, 0, 1, 1, 1, 32, 64, &op, nullptr, nullptr, nullptr, nullptr, 0) == -1);
}

int main() {
    constants_from_scales();
    argument_checks();
    kernel_plans();
    oracle_runs();
    std::printf("host_sanitize: %ld checks passed\n", g_checks);
    return 0;
}
