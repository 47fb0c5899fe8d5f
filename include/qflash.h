/*
 * qflash.h -- C ABI of the MI355X (gfx950) integer-only fused attention forward library.
 *
 * The library computes Algorithm 1 ("QFlash") of arxiv 2604.25306: tile-wise attention on int8
 * Q, K, V with an online softmax carried out entirely in integers (Algorithm 2, the division-free
 * base-2 exponential; Eq. 9-10 requantisation; ScaleRelease of Appendix B.1; integer
 * normalisation, Section 4.7).  Output is int8 with scale s_O = s_V (Algorithm 1, Return).
 *
 * Conventions for every function:
 *   - returns QFLASH_OK (0) or a negative QFLASH_ERR_* code; never throws, aborts or synchronises;
 *   - "device" pointers are HIP device memory on the context's GPU, "host" pointers ordinary memory;
 *   - the caller owns every buffer it passes; the library owns only the opaque context.
 */
#ifndef QFLASH_H
#define QFLASH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define QFLASH_OK           0
#define QFLASH_ERR_NULL    (-1)  /* a required pointer is NULL                                   */
#define QFLASH_ERR_SHAPE   (-2)  /* B,H,N,d or the bias extents are outside the supported range  */
#define QFLASH_ERR_TILE    (-3)  /* kv_tile is not 64 or 128                                      */
#define QFLASH_ERR_PARAM   (-4)  /* an integer constant in qflash_params is out of range          */
#define QFLASH_ERR_DEVICE  (-5)  /* no such GPU, not a gfx950, or a HIP runtime error             */
#define QFLASH_ERR_LAUNCH  (-6)  /* the kernel launch was rejected by the runtime                 */
#define QFLASH_ERR_CTX     (-7)  /* the context is not a live context of this library             */
#define QFLASH_ERR_ALIGN   (-8)  /* Q, K, V or O is not 16-byte aligned, bias not 4-byte aligned  */
#define QFLASH_ERR_SCRATCH (-9)  /* qflash_attention_static: table larger than its static memory  */

#define QFLASH_MAX_N       4096  /* 128*127*N must stay below 2^31 with margin                    */
#define QFLASH_MAX_PARAM_HEADS 64 /* most heads qflash_attention_per_head accepts                 */
#define QFLASH_EXCLUDED    INT32_MIN  /* bias value that removes a (query, key) pair              */

typedef struct qflash_ctx qflash_ctx;   /* opaque; created and destroyed by the library */

/*
 * Integer constants of one call.  They depend only on the real scales and are computed outside
 * the kernel (Section 4.3 below Eq. 7; Section 4.4 below Eq. 10; Algorithm 1 "Require").
 * Caller-owned, read during the call only.  With s = sQ*sK*d^(-1/2)*log2(e) (Algorithm 1):
 */
typedef struct {
    int32_t x_shift;    /* k in [0,13]: scores are multiplied by 2^k before Algorithm 2 and s is
                           divided by 2^k; 0 is the paper as printed, k > 0 keeps s_inv usable when
                           s is coarse                                                          */
    int32_t s_inv;      /* round(2^k / s), in [2^10, 2^18)                  (Algorithm 2)         */
    int32_t exp_mul;    /* M = round(-(s/2^k) * 2^exp_shift), negative      (Algorithm 2)         */
    int32_t exp_shift;  /* N of q = (x*M) >> N; must be 32                  (Appendix B.2)        */
    int32_t p_mul;      /* M_r = round(127/s_inv * 2^p_shift)               (Eq. 10)              */
    int32_t p_shift;    /* r = 8 - floor(log2(127/s_inv))                   (Eq. 9)               */
    int32_t a_mul;      /* ceil(2^30 / s_inv): brings alpha to 16 fractional bits for ScaleRelease
                           (Appendix B.1)                                                         */
    int32_t out_round;  /* 0: floor in the final division (Algorithm 1, last step); 1: nearest    */
} qflash_params;

/*
 * Derive every field of *out from the real per-tensor scales of Q and K and the head size d
 * (host only, no GPU work).  sV does not enter the kernel (it is the output scale) and is only
 * checked for being positive and finite.  out_round is set to 0.
 * Errors: NULL, PARAM (scales not positive/finite, or s outside the representable window),
 * SHAPE (d not 32 or 64).
 */
int qflash_params_from_scales(double sQ, double sK, double sV, int d, qflash_params* out /*host*/);

/*
 * Create a context bound to GPU `device_id`.  *out (host) receives the context.
 * Errors: NULL, DEVICE (no such device / not gfx950).
 */
int qflash_create(qflash_ctx** out, int device_id);

/*
 * Context options.  QFLASH_CFG_EXP_TABLE (default 1): 1 lets the kernel read the int8 weight of a
 * score (Algorithm 2 followed by Eq. 10) from a table of that same function held in LDS when the
 * table is small enough (about 8 * s_inv / 2^x_shift bytes, up to 40 KiB); 0 always evaluates
 * Algorithm 2 arithmetically.  Both give identical bits.  A table is built on the GPU, once per
 * set of constants and stream (first call with them) and kept in one of 32 slots of the context.
 * When all are taken, the least recently used one is rebuilt for the new constants; the building
 * kernel waits on the GPU (never on the host) for what has been enqueued so far on the stream that
 * read the old table.  A call on a stream that is being captured into a HIP graph builds nothing:
 * it uses a table only if an earlier call on that stream has built it (such a table is then kept
 * for good, because the graph reads it on every replay) and computes arithmetically otherwise.
 *
 * QFLASH_CFG_QUANTISED_MAX (default 0).  1 switches the context to a variant that is NOT the
 * paper's Algorithm 1 and gives different (slightly less accurate) results; never on by default.
 * Instead of the running maximum it keeps the maximum rounded up to a whole octave (a multiple of
 * s_inv score units) as the reference of the integer softmax; the reference then only moves by
 * whole octaves, the max-offset factor alpha of Algorithm 1 (step 4) is an exact power of two, and
 * ScaleRelease (Appendix B.1) is an arithmetic shift of numerator and denominator, skipped for
 * tiles that move no reference.  The largest weight of a row is 127 * 2^-f, 0 <= f < 1, instead of
 * 127.  Everything else (Algorithm 2, Eq. 10, bias, exclusion, normalisation, output scale) is
 * unchanged.  Requires x_shift == 0 in every qflash_params of the call (PARAM otherwise); not
 * available through qflash_attention_static and qflash_attention_dynamic (PARAM).
 * Errors: NULL, CTX, PARAM (unknown key or value).
 */
#define QFLASH_CFG_EXP_TABLE 1
#define QFLASH_CFG_QUANTISED_MAX 2
int qflash_configure(qflash_ctx* ctx, int key, int value);

/*
 * State of the context's table cache and what the last call through it did (host only; for
 * callers who want to know whether their constants keep the look-up mode, and for tests).
 *   slots_total, slots_in_use, slots_pinned (read by a captured graph: never rebuilt), evictions
 *   (slots rebuilt for other constants so far); last_weight_mode: QFLASH_WEIGHTS_ARITHMETIC, _TABLE
 *   (every head read its table) or _MIXED (per-head constants of which only some had a table) of the
 *   last qflash_attention / _per_head / _packed_bias call; last_kernel: as qflash_plan_info.kernel.
 * Errors: NULL, CTX.
 */
#define QFLASH_WEIGHTS_ARITHMETIC 0
#define QFLASH_WEIGHTS_TABLE      1
#define QFLASH_WEIGHTS_MIXED      2
typedef struct {
    int32_t slots_total, slots_in_use, slots_pinned, evictions;
    int32_t last_weight_mode, last_kernel, reserved[2];
} qflash_cache_info;
int qflash_cache_query(qflash_ctx* ctx, qflash_cache_info* out /* host */);

/*
 * One fused attention forward pass (Algorithm 1), enqueued on `hip_stream`; returns without
 * waiting for the GPU.
 *
 *   Q, K, V  device, int8, [B,H,N,d] contiguous row-major, 16-byte aligned; read only.
 *   O        device, int8, [B,H,N,d], same layout; every element is written.  Scale s_V.
 *   bias     device int32 [bias_B,bias_H,N,N] or NULL.  Element [b % bias_B][h % bias_H][i][c] is
 *            added to the integer score of query i and key c before the row maximum; it is in
 *            units of the score Q_hat.K_hat (real bias * sqrt(d)/(sQ*sK)).  The value
 *            QFLASH_EXCLUDED removes the pair: it takes no part in the maximum and gets weight 0.
 *            Contract: every non-excluded score+bias lies in (-2^21, 2^21) (the initial running
 *            maximum of Algorithm 1 is -2^21).  A row with every key excluded yields zeros.
 *            With bias == NULL, bias_B and bias_H are ignored.
 *   B,H,N,d  1 <= N <= QFLASH_MAX_N, d in {32,64}, B,H >= 1, B*H*N*d < 2^31.
 *   kv_tile  B_c of Algorithm 1: 64 or 128.  The result depends on it (the running maximum and
 *            the rescaling of past accumulators happen per KV tile); it does not depend on the
 *            query block size or on any launch parameter.
 *            Cost: 64 is the tile the kernels are tuned for.  Measured on MI355X: with short
 *            sequences (N <= 256) tile 128 takes 1.3 times the time of tile 64 (ViT-B/16
 *            B=64: 24.9 against 19.2 us; the variant runs short of registers, and the library
 *            computes its weights arithmetically there because the look-up variant is slower
 *            still); on long sequences with d = 64 the two are within 1 % (N = 577: 43.7 against
 *            43.9 us).  A d = 32 sequence
 *            too long for LDS (N above about 1000) takes the streamed kernel, which stages one
 *            tile at a time with two barriers per tile and computes weights arithmetically:
 *            about 0.65 of the ring kernel's rate per score with tile 64 (B*H = 64, N = 2100:
 *            150 us), 0.43 with tile 128 (228 us).
 *   p        host; validated on every call.
 *   hip_stream  a hipStream_t of the context's device (NULL = the default stream).
 *
 * All buffers must stay valid until the stream has executed the work.  Calls on one context
 * from several host threads are allowed (the context's table cache is guarded by a lock of its own;
 * contexts do not wait for one another).  The first call with new constants on a stream also
 * enqueues a small table-building kernel on that stream; a stream handle must not be reused for a
 * new stream while its context lives.
 * Errors: CTX, NULL, SHAPE, TILE, PARAM, ALIGN, DEVICE, LAUNCH.  On error nothing is enqueued.
 */
int qflash_attention(qflash_ctx* ctx,
                     const int8_t* Q, const int8_t* K, const int8_t* V, int8_t* O,
                     const int32_t* bias, int bias_B, int bias_H,
                     int B, int H, int N, int d, int kv_tile,
                     const qflash_params* p, void* hip_stream);

/*
 * qflash_attention for callers that must not allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same result bits.  The
 * only device memory the library needs beyond inputs and outputs, the weight table of the look-up
 * mode (see qflash_configure), lives here in a static device array of QFLASH_STATIC_TABLE_BYTES
 * that each GPU holds from the moment the library is loaded until the process ends; its address is
 * looked up once per context in qflash_create.  Every call rebuilds the table there (one small
 * kernel ahead of the attention kernel on hip_stream), so nothing is cached, nothing is allocated
 * or freed, and the context's table cache is not touched.
 *   - Constants whose table (about 8 * s_inv / 2^x_shift bytes) does not fit the array are
 *     refused with QFLASH_ERR_SCRATCH; with QFLASH_CFG_EXP_TABLE set to 0 the call computes
 *     arithmetically, uses no such memory and accepts every constant qflash_attention accepts.
 *   - All calls on one GPU share the one array: calls on different streams (or from different
 *     contexts of the same GPU) that overlap in time race on it.  Calls on one stream are safe.
 * Errors: as qflash_attention, plus SCRATCH; DEVICE also if the array's address was not available.
 */
#define QFLASH_STATIC_TABLE_BYTES (32 * 1024)
int qflash_attention_static(qflash_ctx* ctx,
                            const int8_t* Q, const int8_t* K, const int8_t* V, int8_t* O,
                            const int32_t* bias, int bias_B, int bias_H,
                            int B, int H, int N, int d, int kv_tile,
                            const qflash_params* p, void* hip_stream);

/*
 * The same pass with per-head quantisation (Section 3.3 and Appendix B.3: per-tensor and per-head
 * are the granularities under which the integer running maximum still compares like with like).
 * p points to H entries (host); head h of every batch element uses p[h], and its output has the
 * scale s_V of that head.  All entries must share out_round.  H <= QFLASH_MAX_PARAM_HEADS.
 * bias, if given, is added to the integer score of each head as is, i.e. it has to be expressed
 * in that head's score unit.  Everything else as for qflash_attention.
 * Errors: as qflash_attention; SHAPE also for H > QFLASH_MAX_PARAM_HEADS, PARAM also for
 * entries that differ in out_round.
 */
int qflash_attention_per_head(qflash_ctx* ctx,
                              const int8_t* Q, const int8_t* K, const int8_t* V, int8_t* O,
                              const int32_t* bias, int bias_B, int bias_H,
                              int B, int H, int N, int d, int kv_tile,
                              const qflash_params* p /* host, H entries */, void* hip_stream);

/*
 * Bias in the layout the kernels read fastest.  The additive integer bias of windowed attention
 * (Section 5: Swin; relative-position bias plus the mask of shifted windows, step 1 of
 * Algorithm 1 with the bias added to S) is fixed per layer, while the plain [N,N] layout makes
 * every lane of a wavefront read its own row.  qflash_pack_bias rewrites it once so that the 64
 * lanes of a wavefront read 1 KiB in a row; qflash_attention_packed_bias then computes exactly
 * what qflash_attention / qflash_attention_per_head compute from the plain bias.
 *
 * Layout of `packed` (int32): [bias_B*bias_H][R][R][4][64][4] with R = ceil(N/32); the element
 * [s][rb][cb][a][l][b] is bias[s][min(32*rb + l%32, N-1)][c] with c = 32*cb + 8*a + 4*(l/32) + b,
 * or QFLASH_EXCLUDED where c >= N.  It depends on N only, not on kv_tile or d.
 *
 *   qflash_packed_bias_bytes  size of `packed` in bytes; 0 if the extents are not supported.
 *   qflash_pack_bias          bias: device int32 [bias_B,bias_H,N,N], 4-byte aligned, read only;
 *                             packed: device, 16-byte aligned, packed_bytes >= the size above,
 *                             caller-owned.  Enqueues one kernel on hip_stream; allocates nothing.
 *                             Errors: CTX, NULL, SHAPE (also: packed_bytes too small), ALIGN,
 *                             DEVICE, LAUNCH.
 *   qflash_attention_packed_bias  as qflash_attention with n_params == 1 (p[0] serves every head)
 *                             or as qflash_attention_per_head with n_params == H; packed_bias must
 *                             not be NULL and must have been written for the same bias_B, bias_H, N.
 *                             Errors: as those; PARAM also for another n_params.
 */
size_t qflash_packed_bias_bytes(int bias_B, int bias_H, int N);

int qflash_pack_bias(qflash_ctx* ctx, const int32_t* bias, int bias_B, int bias_H, int N,
                     int32_t* packed /* device */, size_t packed_bytes, void* hip_stream);

int qflash_attention_packed_bias(qflash_ctx* ctx,
                                 const int8_t* Q, const int8_t* K, const int8_t* V, int8_t* O,
                                 const int32_t* packed_bias, int bias_B, int bias_H,
                                 int B, int H, int N, int d, int kv_tile,
                                 const qflash_params* p /* host, n_params entries */, int n_params,
                                 void* hip_stream);

/*
 * Dynamic quantisation (Section 5, evaluation set-up: activation scales computed on the fly;
 * Eq. 1-2 with b = 8) in front of the same pass, entirely on the GPU and without waiting for it:
 * per-tensor abs-max of the float32 tensors Qf, Kf, Vf, scales s_X = max|X| / 127, quantisation
 * X_hat = clip(rint(X * r), -127, 127) with r = float32(127) / max|X| (one float32 multiplication
 * per element, round half to even), derivation of the integer constants from s_Q and s_K exactly
 * as qflash_params_from_scales does, then Algorithm 1.  An all-zero tensor gets scale 1.
 *
 *   Qf, Kf, Vf  device, float32, [B,H,N,d] contiguous, 16-byte aligned, finite values; read only.
 *   O           device, int8, [B,H,N,d]; scale s_V as reported in *info.
 *   info        device or NULL; receives the scales, the constants used and a status: QFLASH_OK,
 *               or QFLASH_ERR_PARAM when the scales fall outside the supported window (O is then
 *               all zeros, with or without info).
 *   workspace   device scratch of at least qflash_dynamic_workspace_bytes(B,H,N,d) bytes, 16-byte
 *               aligned, caller-owned; it holds the int8 copies of Q, K, V among other things and
 *               must stay untouched until the stream has executed the work.  The call allocates
 *               nothing.
 *   out_round, kv_tile, hip_stream  as for qflash_attention.  No integer bias in these entry
 *               points (it is expressed in a score unit that is only known on the GPU here);
 *               qflash_attention_dynamic_bias takes one in real units.
 * The weight table of the look-up mode, if the constants allow one, is built on the GPU as well
 * (in the workspace).
 * Errors: CTX, NULL, SHAPE (also: workspace too small), TILE, PARAM (out_round), ALIGN, DEVICE,
 * LAUNCH.
 */
typedef struct {
    double sQ, sK, sV;       /* Eq. 1: max|X| / 127                                             */
    qflash_params params;    /* the constants the attention kernel used                         */
    int32_t status;          /* QFLASH_OK or QFLASH_ERR_PARAM                                   */
    int32_t reserved;
} qflash_dynamic_info;

size_t qflash_dynamic_workspace_bytes(int B, int H, int N, int d);

int qflash_attention_dynamic(qflash_ctx* ctx,
                             const float* Qf, const float* Kf, const float* Vf, int8_t* O,
                             int B, int H, int N, int d, int kv_tile, int out_round,
                             qflash_dynamic_info* info /* device or NULL */,
                             void* workspace /* device */, size_t workspace_bytes,
                             void* hip_stream);

/*
 * The same with an additive bias given in real units and an exclusion mask (windowed attention:
 * relative-position bias, shifted-window mask), for callers whose scales are only found on the fly.
 * The paper adds the bias to S inside Algorithm 1 (step 1) and leaves its quantisation open; here
 * the GPU brings it to the unit of the integer score with the scales it has just computed:
 *   unit = (s_Q * s_K) / sqrt(d),   b_hat = clip(floor(double(b) / unit + 0.5), -(2^20-1), 2^20-1)
 * in float64, one rounding per operation; excluded pairs take no part in the maximum and get
 * weight 0 (QFLASH_EXCLUDED).  The converted bias is written to the workspace in the packed layout
 * (see qflash_pack_bias) and the attention kernel reads it from there.
 *
 *   bias_real  device or NULL, float32 [bias_B,bias_H,N,N] contiguous, 4-byte aligned, finite;
 *              NULL means a bias of zeros (mask only).
 *   excluded   device or NULL, uint8 [bias_B,bias_H,N,N]; nonzero excludes the pair.
 *              At least one of the two must be given (NULL otherwise); indexing as for qflash_attention.
 *   workspace  at least qflash_dynamic_bias_workspace_bytes(B,H,N,d,bias_B,bias_H) bytes (0: the
 *              extents are not supported).
 * Everything else, and the errors, as qflash_attention_dynamic; SHAPE also for bias extents.
 */
size_t qflash_dynamic_bias_workspace_bytes(int B, int H, int N, int d, int bias_B, int bias_H);

int qflash_attention_dynamic_bias(qflash_ctx* ctx,
                                  const float* Qf, const float* Kf, const float* Vf, int8_t* O,
                                  const float* bias_real /* device or NULL */,
                                  const uint8_t* excluded /* device or NULL */, int bias_B, int bias_H,
                                  int B, int H, int N, int d, int kv_tile, int out_round,
                                  qflash_dynamic_info* info /* device or NULL */,
                                  void* workspace /* device */, size_t workspace_bytes,
                                  void* hip_stream);

/*
 * How a call would be laid out on the GPU (host only; nothing is enqueued and no GPU is touched
 * when ctx is NULL, in which case an MI355X is assumed: 256 compute units, 160 KiB of LDS per
 * workgroup).  For callers who want to know the occupancy of a shape, and for tests of the host
 * logic: the work decomposition of Algorithm 1 over (batch, head, query block) is the library's
 * own choice and does not change a single output bit.
 *
 *   bias_B, bias_H   extents of the bias the call would be given, or 0, 0 for none.
 *   kernel           0: KV tiles streamed through LDS, 128 query rows per workgroup;
 *                    1: K and V of a (batch, head) pair resident in LDS; 2: two KV tiles in LDS (long
 *                    sequences with d = 64; without a bias they are fed by direct global-to-LDS loads and
 *                    workgroups are four wavefronts);
 *                    3: one workgroup per compute unit holds Q, K, V of several pairs in LDS (short
 *                    sequences, d = 64, kv_tile 64, no bias, one set of constants, few enough pairs for
 *                    a single round of workgroups; assumes a weight table of 32 KiB).  For kernel 3:
 *                    wavefronts_per_pair is the number of wavefronts of a workgroup, query_blocks the
 *                    32-row blocks of a pair, units = workgroups, and workgroup w takes pairs
 *                    [w * pairs_per_workgroup, (w + 1) * pairs_per_workgroup).
 *                    4: windowed attention (33 <= N <= 64, d = 32, one KV tile, no bias or a bias
 *                    in the packed layout whose extents divide B and H, one set of constants,
 *                    Algorithm 1 only): persistent workgroups, one per compute unit, whose wavefronts
 *                    each work through a run of pairs that share a bias slice (the query assumes
 *                    that a bias would be packed).  For kernel 4: pairs_per_workgroup = pairs a
 *                    workgroup works through, wavefronts_per_pair = 2 (one per half of the rows),
 *                    units = workgroups.
 *   pairs_per_workgroup, wavefronts_per_pair, query_blocks (workgroups a pair is split over),
 *   units (pieces of work = workgroups that have rows), workgroups (launched; a few may be idle),
 *   tile_by_tile (1: KV tiles staged one ahead of their use), bias_period_units (0, or the number of
 *   units after which the bias slices repeat and by which workgroups are dealt to the 8 XCDs).
 * qflash_plan_unit: the unit that workgroup `workgroup` of such a launch takes, or -1 if it is one
 * of the idle ones (or out of range).  Every unit in [0, units) is taken by exactly one workgroup.
 * Errors: NULL, CTX, SHAPE, TILE.
 */
typedef struct {
    int32_t kernel, pairs_per_workgroup, wavefronts_per_pair, query_blocks;
    int32_t units, workgroups, tile_by_tile, bias_period_units;
    int32_t units_per_xcd, reserved[3];
} qflash_plan_info;

int qflash_plan_query(qflash_ctx* ctx /* or NULL */, int B, int H, int N, int d, int kv_tile,
                      int bias_B, int bias_H, qflash_plan_info* out);

int qflash_plan_unit(const qflash_plan_info* plan, int workgroup);

/*
 * Destroy a context.  NULL is accepted (returns QFLASH_OK).  Destroying a context twice, or a
 * pointer that never was a context, returns QFLASH_ERR_CTX and touches nothing.
 */
int qflash_destroy(qflash_ctx* ctx);

/* Static, NUL-terminated description of an error code (host). */
const char* qflash_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* QFLASH_H */
