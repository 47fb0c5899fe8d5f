/*
 * QFlash CPU oracle -- TEST INFRASTRUCTURE, NOT A PRODUCT PATH.
 *
 * A plain, slow, scalar implementation of the fused integer-only attention
 * forward pass (Algorithm 1) with the division-free base-2 exponential
 * (Algorithm 2).  It exists only so that tests, the smoke check and the
 * benchmark's cpu_baseline leg can compare the GPU library against it.  It
 * shares no code, header, table or constant generator with the GPU library
 * and must never be linked or called from it.
 *
 * Every intermediate is an int64_t.  Wherever the GPU kernel keeps a value in
 * 32 bits the oracle checks that the int64 value fits and counts a violation
 * otherwise (returned through `violations`), so a silent wrap can never pass
 * as agreement.
 *
 * The steps follow Algorithm 1 in the paper's order, one query row at a time
 * (rows are independent, so the query block size B_r does not enter).  No
 * blocking, fusion or reordering beyond the KV tiling the algorithm states.
 *
 * Readings of points the paper leaves open are marked [Rn] below; the list
 * with reasons lives in the design document of this repository.
 *
 * Parity pins: every function here is pinned by tests that run without a
 * GPU (closed forms of 2^x, exact integer matmul, brute-force full-row
 * integer softmax for the single-tile and the early-maximum cases, the
 * two-tile composition rule, floor division, scaling identities, the
 * exclusion rule).  No function is "parity unpinned".
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Integer constants of one call; derived on the host from the real scales
 * (Algorithm 1 "Require", Algorithm 2, Eq. 9-10).  Field order is private to
 * the oracle and its Python wrapper. */
typedef struct {
    int32_t x_shift;   /* k: scores are multiplied by 2^k before Algorithm 2 [R5] */
    int32_t s_inv;     /* round(2^k / s), s = sQ*sK*d^-1/2*log2(e)  (Alg. 2)     */
    int32_t exp_mul;   /* M = round(-(s/2^k) * 2^exp_shift), negative (Alg. 2)   */
    int32_t exp_shift; /* N of the mul+shift quotient (Appendix B.2) [R1]        */
    int32_t p_mul;     /* M_r of Eq. 10 for the ratio 127/s_inv [R7]             */
    int32_t p_shift;   /* r   of Eq. 9                                           */
    int32_t a_mul;     /* ceil(2^30 / s_inv): alpha -> 16 fractional bits [R6]   */
    int32_t out_round; /* 0: floor as printed in Alg. 1; 1: nearest (extension)  */
} oracle_params;

#define EXCLUDED INT32_MIN        /* bias sentinel: column takes no part [R12] */
#define M_INIT   (-(1 << 21))     /* initial running maximum (Alg. 1)          */

/* floor(v / 2^n) for any sign: the paper's ">>" on integers. */
static int64_t asr(int64_t v, int n)
{
    int64_t den = (int64_t)1 << n;
    int64_t q = v / den;
    if ((v % den) != 0 && v < 0) q -= 1;
    return q;
}

/* floor(a / b), b > 0. */
static int64_t floor_div(int64_t a, int64_t b)
{
    int64_t q = a / b;
    if ((a % b) != 0 && ((a < 0) != (b < 0))) q -= 1;
    return q;
}

static int fits32(int64_t v) { return v >= INT32_MIN && v <= INT32_MAX; }

/* Algorithm 2 (integer base-2 exponential, mul+shift quotient), for x <= 0.
 * Returns y with 1.0 represented by s_inv.
 *   x' = x * 2^k                                   [R5]
 *   q  = (x' * M) >> N                             (quotient, q >= 0 [R2])
 *   r  = x' + q * s_inv                            (remainder, not clamped [R3])
 *   y  = ((r >> 1) + s_inv) >> q,  0 when q > 31   [R4]
 */
int64_t oracle_shift_exp2(int64_t x, const oracle_params *p)
{
    int64_t xs = x * ((int64_t)1 << p->x_shift);
    int64_t q = asr(xs * (int64_t)p->exp_mul, p->exp_shift);
    int64_t r = xs + q * (int64_t)p->s_inv;
    if (q > 31) return 0;
    return asr(asr(r, 1) + (int64_t)p->s_inv, (int)q);
}

/* The quotient alone, for the test that compares it with the division form
 * q = floor(x' / -s_inv) of Appendix B.2. */
int64_t oracle_shift_exp2_quotient(int64_t x, const oracle_params *p)
{
    int64_t xs = x * ((int64_t)1 << p->x_shift);
    return asr(xs * (int64_t)p->exp_mul, p->exp_shift);
}

/* Eq. 10 applied to the exponential: int32 -> [0,127] with 1.0 <-> 127 [R7]. */
int64_t oracle_requant(int64_t y, const oracle_params *p)
{
    int64_t v = asr(y * (int64_t)p->p_mul, p->p_shift);
    return v > 127 ? 127 : v;
}

/* Max-offset factor in 16 fractional bits, 1.0 <-> 65536 [R6]. */
int64_t oracle_alpha16(int64_t alpha_hat, const oracle_params *p)
{
    int64_t a = asr(alpha_hat * (int64_t)p->a_mul, 14);
    return a > 65536 ? 65536 : a;
}

/* ScaleRelease: rescale a running accumulator by alpha and drop alpha's scale
 * again, so the accumulator keeps its own scale (Appendix B.1) [R6]. */
int64_t oracle_scale_release(int64_t acc, int64_t alpha16)
{
    return asr(acc * alpha16, 16);
}

/*
 * Algorithm 1 for tensors Q,K,V,O of shape [B,H,N,d] (row-major, int8).
 *
 *   bias       NULL, or int32 [bias_B, bias_H, N, N] indexed
 *              [b % bias_B][h % bias_H][i][c]; the value INT32_MIN excludes
 *              the column from the maximum and gives it weight 0 [R12].
 *   kv_tile    B_c of Algorithm 1.
 *   O_acc      optional int64 [B,H,N,d]: numerator after the last tile.
 *   l_out      optional int64 [B,H,N]  : denominator after the last tile.
 *   m_out      optional int64 [B,H,N]  : running maximum after the last tile.
 *   violations optional int64[1]: number of intermediate values that would
 *              not fit the 32-bit registers a GPU kernel keeps them in.
 *   nthreads   OpenMP threads over (b,h); <= 0 means the OpenMP default.
 * Returns 0, or -1 on an invalid argument.
 */
static int attention_impl(const int8_t *Q, const int8_t *K, const int8_t *V,
                          int8_t *O, const int32_t *bias, int bias_B, int bias_H,
                          int B, int H, int N, int d, int kv_tile,
                          const oracle_params *p_all, int p_per_head,
                          int64_t *O_acc, int64_t *l_out, int64_t *m_out,
                          int64_t *violations, int nthreads)
{
    if (!Q || !K || !V || !O || !p_all) return -1;
    if (B < 1 || H < 1 || N < 1 || d < 1 || kv_tile < 1) return -1;
    if (bias && (bias_B < 1 || bias_H < 1)) return -1;

    const int Tc = (N + kv_tile - 1) / kv_tile;
    int64_t bad_total = 0;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif

#pragma omp parallel for schedule(dynamic, 1) reduction(+ : bad_total)
    for (int bh = 0; bh < B * H; ++bh) {
        const int b = bh / H, h = bh % H;
        /* per-tensor constants, or those of head h (Section 3.3 / Appendix B.3: per-head scales) */
        const oracle_params *p = p_per_head ? p_all + h : p_all;
        const int8_t *Qh = Q + (size_t)bh * N * d;
        const int8_t *Kh = K + (size_t)bh * N * d;
        const int8_t *Vh = V + (size_t)bh * N * d;
        int8_t *Oh = O + (size_t)bh * N * d;
        const int32_t *bias_h =
            bias ? bias + ((size_t)(b % bias_B) * bias_H + (size_t)(h % bias_H)) * N * N : NULL;

        int64_t *S = (int64_t *)malloc(sizeof(int64_t) * (size_t)kv_tile);
        int64_t *P = (int64_t *)malloc(sizeof(int64_t) * (size_t)kv_tile);
        char *excl = (char *)malloc((size_t)kv_tile);
        int64_t *acc = (int64_t *)malloc(sizeof(int64_t) * (size_t)d);
        int64_t bad = 0;

        for (int i = 0; i < N; ++i) {
            /* initial on-chip state of Algorithm 1 */
            for (int t = 0; t < d; ++t) acc[t] = 0;
            int64_t l = 0;
            int64_t m = M_INIT;

            for (int j = 0; j < Tc; ++j) {
                const int c0 = j * kv_tile;
                const int nc = (c0 + kv_tile <= N) ? kv_tile : N - c0;

                /* step 1: S = Q_i K_j^T (+ bias) */
                for (int c = 0; c < nc; ++c) {
                    int64_t s = 0;
                    for (int t = 0; t < d; ++t)
                        s += (int64_t)Qh[(size_t)i * d + t] * (int64_t)Kh[(size_t)(c0 + c) * d + t];
                    excl[c] = 0;
                    if (bias_h) {
                        int32_t bv = bias_h[(size_t)i * N + (c0 + c)];
                        if (bv == EXCLUDED) excl[c] = 1;
                        else s += (int64_t)bv;
                    }
                    S[c] = s;
                    if (!excl[c] && !fits32(s)) bad++;
                }

                /* steps 2,3: row maximum, running maximum */
                int64_t m_new = m;
                for (int c = 0; c < nc; ++c)
                    if (!excl[c] && S[c] > m_new) m_new = S[c];

                /* step 4: max-offset factor */
                int64_t alpha_hat = oracle_shift_exp2(m - m_new, p);
                int64_t alpha16 = oracle_alpha16(alpha_hat, p);
                if (alpha_hat < 0 || !fits32(alpha_hat * (int64_t)p->a_mul)) bad++;

                /* steps 5,6: score intensity, requantisation to int8 */
                int64_t rowsum = 0;
                for (int c = 0; c < nc; ++c) {
                    if (excl[c]) { P[c] = 0; continue; }
                    int64_t y = oracle_shift_exp2(S[c] - m_new, p);
                    if (y < 0 || !fits32(y * (int64_t)p->p_mul)) bad++;
                    P[c] = oracle_requant(y, p);
                    if (P[c] < 0) bad++;
                    rowsum += P[c];                       /* step 7 */
                }

                /* step 9: denominator */
                l = oracle_scale_release(l, alpha16) + rowsum;
                if (!fits32(l)) bad++;

                /* steps 8,10: P V and numerator */
                for (int t = 0; t < d; ++t) {
                    int64_t pv = 0;
                    for (int c = 0; c < nc; ++c)
                        pv += P[c] * (int64_t)Vh[(size_t)(c0 + c) * d + t];
                    acc[t] = oracle_scale_release(acc[t], alpha16) + pv;
                    if (!fits32(acc[t])) bad++;
                }
                m = m_new;
            }

            /* step 11: integer normalisation, output scale s_V */
            for (int t = 0; t < d; ++t) {
                int64_t o;
                if (l == 0) o = 0;                                        /* [R11] */
                else if (p->out_round) o = floor_div(2 * acc[t] + l, 2 * l);
                else o = floor_div(acc[t], l);                            /* [R10] */
                if (o < -128) o = -128;
                if (o > 127) o = 127;
                Oh[(size_t)i * d + t] = (int8_t)o;
                if (O_acc) O_acc[((size_t)bh * N + i) * d + t] = acc[t];
            }
            if (l_out) l_out[(size_t)bh * N + i] = l;
            if (m_out) m_out[(size_t)bh * N + i] = m;
        }
        free(S); free(P); free(excl); free(acc);
        bad_total += bad;
    }
    if (violations) *violations = bad_total;
    return 0;
}

int oracle_qflash_attention(const int8_t *Q, const int8_t *K, const int8_t *V,
                            int8_t *O, const int32_t *bias, int bias_B, int bias_H,
                            int B, int H, int N, int d, int kv_tile,
                            const oracle_params *p,
                            int64_t *O_acc, int64_t *l_out, int64_t *m_out,
                            int64_t *violations, int nthreads)
{
    return attention_impl(Q, K, V, O, bias, bias_B, bias_H, B, H, N, d, kv_tile, p, 0,
                          O_acc, l_out, m_out, violations, nthreads);
}

/*
 * The same with one set of integer constants per head: p[h] serves every (b, h) pair of head h
 * (per-head quantisation, Section 3.3 and Appendix B.3: Q, K and V of a head share one scale
 * each, so the running maximum still compares like with like).  The output of head h has scale
 * s_V of that head.  Everything else as above.
 */
int oracle_qflash_attention_per_head(const int8_t *Q, const int8_t *K, const int8_t *V,
                                     int8_t *O, const int32_t *bias, int bias_B, int bias_H,
                                     int B, int H, int N, int d, int kv_tile,
                                     const oracle_params *p /* H entries */,
                                     int64_t *O_acc, int64_t *l_out, int64_t *m_out,
                                     int64_t *violations, int nthreads)
{
    return attention_impl(Q, K, V, O, bias, bias_B, bias_H, B, H, N, d, kv_tile, p, 1,
                          O_acc, l_out, m_out, violations, nthreads);
}

/*
 * ---------------------------------------------------------------------------
 * NOT THE PAPER'S ALGORITHM 1: the "quantised maximum" variant.
 *
 * Algorithm 1 rescales the running numerator and denominator by
 * alpha = 2^((m_old - m_new) s), an arbitrary factor in (0, 1], through
 * ScaleRelease (Appendix B.1).  This variant keeps, instead of the running
 * maximum itself, the smallest whole number of octaves at or above it: with
 * one octave = s_inv units of the scaled score x' = x 2^k (Algorithm 2),
 *
 *     level(t) = ceil(t 2^k / s_inv),      L_new = max(L_old, level(rowmax)),
 *
 * and every score is referred to L_new s_inv instead of to the maximum:
 * x' = S 2^k - L_new s_inv <= 0 goes through the remaining steps of
 * Algorithm 2 and through Eq. 10 unchanged.  The reference level only moves
 * by whole octaves, n = L_new - L_old >= 0, so alpha = 2^-n exactly and
 * ScaleRelease is the arithmetic shift X <- X >> n (floor), for numerator and
 * denominator alike.  Everything else (steps 1, 5-9, 11, bias, exclusion,
 * initial maximum -2^21, output rule) is as in Algorithm 1.
 *
 * What it costs: the largest weight of a row is 127 2^-f with f in [0, 1)
 * instead of 127, i.e. up to one bit of the 7-bit weights.  What it buys:
 * no multiplication in the rescale, and tiles that leave the level alone
 * (most of them) need no rescale at all.
 *
 * Pins (tests without a GPU): single tile == brute force over the whole row
 * with the same reference level; level invariants (multiple of s_inv,
 * at or above the maximum, less than one octave above it); exact
 * re-composition of 2..10 tiles from the state after each tile with plain
 * shifts; independence of the tiling when the level is settled in the first
 * tile; exact invariance under adding a whole number of octaves to every
 * score; uniform scores = floor(mean V); exclusion = deleted key; cosine
 * against float64 softmax on tiny inputs.
 */

/* ceil(a / b) for b > 0 and any sign of a. */
static int64_t ceil_div(int64_t a, int64_t b)
{
    return -floor_div(-a, b);
}

/* level(t): the smallest L with L * s_inv >= t * 2^k. */
int64_t oracle_qmax_level(int64_t t, const oracle_params *p)
{
    return ceil_div(t * ((int64_t)1 << p->x_shift), (int64_t)p->s_inv);
}

/* Algorithm 2 from its quotient step on, for an argument xs <= 0 that is
 * already in units of the scaled score (x 2^k): quotient by multiply and
 * shift, unclamped remainder, linear fraction, shift; 0 when q > 31. */
int64_t oracle_shift_exp2_scaled(int64_t xs, const oracle_params *p)
{
    int64_t q = asr(xs * (int64_t)p->exp_mul, p->exp_shift);
    int64_t r = xs + q * (int64_t)p->s_inv;
    if (q > 31) return 0;
    return asr(asr(r, 1) + (int64_t)p->s_inv, (int)q);
}

/* X >> n for n >= 0 of any size (floor(X / 2^n)). */
static int64_t shift_release(int64_t x, int64_t n)
{
    return asr(x, n > 62 ? 62 : (int)n);
}

/* Arguments as oracle_qflash_attention; m_out receives the final LEVEL L of every row
 * (the reference is L * s_inv in units of the scaled score). */
static int attention_qmax_impl(const int8_t *Q, const int8_t *K, const int8_t *V,
                               int8_t *O, const int32_t *bias, int bias_B, int bias_H,
                               int B, int H, int N, int d, int kv_tile,
                               const oracle_params *p_all, int p_per_head,
                               int64_t *O_acc, int64_t *l_out, int64_t *m_out,
                               int64_t *violations, int nthreads)
{
    if (!Q || !K || !V || !O || !p_all) return -1;
    if (B < 1 || H < 1 || N < 1 || d < 1 || kv_tile < 1) return -1;
    if (bias && (bias_B < 1 || bias_H < 1)) return -1;

    const int Tc = (N + kv_tile - 1) / kv_tile;
    int64_t bad_total = 0;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif

#pragma omp parallel for schedule(dynamic, 1) reduction(+ : bad_total)
    for (int bh = 0; bh < B * H; ++bh) {
        const int b = bh / H, h = bh % H;
        const oracle_params *p = p_per_head ? p_all + h : p_all;
        const int8_t *Qh = Q + (size_t)bh * N * d;
        const int8_t *Kh = K + (size_t)bh * N * d;
        const int8_t *Vh = V + (size_t)bh * N * d;
        int8_t *Oh = O + (size_t)bh * N * d;
        const int32_t *bias_h =
            bias ? bias + ((size_t)(b % bias_B) * bias_H + (size_t)(h % bias_H)) * N * N : NULL;

        int64_t *S = (int64_t *)malloc(sizeof(int64_t) * (size_t)kv_tile);
        int64_t *P = (int64_t *)malloc(sizeof(int64_t) * (size_t)kv_tile);
        char *excl = (char *)malloc((size_t)kv_tile);
        int64_t *acc = (int64_t *)malloc(sizeof(int64_t) * (size_t)d);
        int64_t bad = 0;
        const int64_t two_k = (int64_t)1 << p->x_shift;

        for (int i = 0; i < N; ++i) {
            for (int t = 0; t < d; ++t) acc[t] = 0;
            int64_t l = 0;
            int64_t L = oracle_qmax_level(M_INIT, p);      /* level of the initial maximum */

            for (int j = 0; j < Tc; ++j) {
                const int c0 = j * kv_tile;
                const int nc = (c0 + kv_tile <= N) ? kv_tile : N - c0;

                /* step 1 as in Algorithm 1 */
                for (int c = 0; c < nc; ++c) {
                    int64_t s = 0;
                    for (int t = 0; t < d; ++t)
                        s += (int64_t)Qh[(size_t)i * d + t] * (int64_t)Kh[(size_t)(c0 + c) * d + t];
                    excl[c] = 0;
                    if (bias_h) {
                        int32_t bv = bias_h[(size_t)i * N + (c0 + c)];
                        if (bv == EXCLUDED) excl[c] = 1;
                        else s += (int64_t)bv;
                    }
                    S[c] = s;
                    if (!excl[c] && !fits32(s)) bad++;
                }

                /* the tile's maximum decides the new level */
                int64_t L_new = L;
                for (int c = 0; c < nc; ++c) {
                    if (excl[c]) continue;
                    int64_t Lc = oracle_qmax_level(S[c], p);
                    if (Lc > L_new) L_new = Lc;
                }
                const int64_t n = L_new - L;               /* alpha = 2^-n */
                const int64_t ref = L_new * (int64_t)p->s_inv;

                int64_t rowsum = 0;
                for (int c = 0; c < nc; ++c) {
                    if (excl[c]) { P[c] = 0; continue; }
                    int64_t xs = S[c] * two_k - ref;       /* <= 0, > -s_inv for the maximum */
                    if (xs > 0) bad++;
                    int64_t y = oracle_shift_exp2_scaled(xs, p);
                    if (y < 0 || !fits32(y * (int64_t)p->p_mul)) bad++;
                    P[c] = oracle_requant(y, p);
                    if (P[c] < 0) bad++;
                    rowsum += P[c];
                }

                l = shift_release(l, n) + rowsum;
                if (!fits32(l)) bad++;
                for (int t = 0; t < d; ++t) {
                    int64_t pv = 0;
                    for (int c = 0; c < nc; ++c)
                        pv += P[c] * (int64_t)Vh[(size_t)(c0 + c) * d + t];
                    acc[t] = shift_release(acc[t], n) + pv;
                    if (!fits32(acc[t])) bad++;
                }
                L = L_new;
            }

            for (int t = 0; t < d; ++t) {
                int64_t o;
                if (l == 0) o = 0;
                else if (p->out_round) o = floor_div(2 * acc[t] + l, 2 * l);
                else o = floor_div(acc[t], l);
                if (o < -128) o = -128;
                if (o > 127) o = 127;
                Oh[(size_t)i * d + t] = (int8_t)o;
                if (O_acc) O_acc[((size_t)bh * N + i) * d + t] = acc[t];
            }
            if (l_out) l_out[(size_t)bh * N + i] = l;
            if (m_out) m_out[(size_t)bh * N + i] = L;
        }
        free(S); free(P); free(excl); free(acc);
        bad_total += bad;
    }
    if (violations) *violations = bad_total;
    return 0;
}

int oracle_qflash_attention_qmax(const int8_t *Q, const int8_t *K, const int8_t *V,
                                 int8_t *O, const int32_t *bias, int bias_B, int bias_H,
                                 int B, int H, int N, int d, int kv_tile,
                                 const oracle_params *p,
                                 int64_t *O_acc, int64_t *l_out, int64_t *m_out,
                                 int64_t *violations, int nthreads)
{
    return attention_qmax_impl(Q, K, V, O, bias, bias_B, bias_H, B, H, N, d, kv_tile, p, 0,
                               O_acc, l_out, m_out, violations, nthreads);
}

int oracle_qflash_attention_qmax_per_head(const int8_t *Q, const int8_t *K, const int8_t *V,
                                          int8_t *O, const int32_t *bias, int bias_B, int bias_H,
                                          int B, int H, int N, int d, int kv_tile,
                                          const oracle_params *p /* H entries */,
                                          int64_t *O_acc, int64_t *l_out, int64_t *m_out,
                                          int64_t *violations, int nthreads)
{
    return attention_qmax_impl(Q, K, V, O, bias, bias_B, bias_H, B, H, N, d, kv_tile, p, 1,
                               O_acc, l_out, m_out, violations, nthreads);
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
