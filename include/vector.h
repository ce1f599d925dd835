/*
 * libvector: VECTOR three-way KV-cache routing on one MI355X (gfx950).
 *
 * The compression pass at prefill -- importance score, reconstruction residual,
 * retain / approximate / evict routing, compaction into a packed cache -- and
 * the decode attention that rebuilds approximated values from their kept keys.
 *
 * Conventions shared by every entry point
 *   - Plain C ABI.  Every pointer marked "device" is device memory owned by the
 *     caller; "host" pointers are ordinary host memory.  The library never
 *     allocates, frees or synchronises: work is enqueued on `stream` (a
 *     hipStream_t passed as void*, NULL = the default stream) and the call
 *     returns at once.  Inputs are never modified.
 *   - Return value: VECTOR_OK or a negative VECTOR_ERR_* code.  Arguments are
 *     validated on the host before anything is launched, so a failing call
 *     writes nothing.
 *   - Row convention: v_hat = k . W with W [d, d]; this W is the transpose of
 *     the column-convention W_OLS of the paper (Section 3.1, footnote).
 *   - The innermost dimension (head_dim) is contiguous; device tensors must be
 *     16-byte aligned.  head_dim is 64 or 128.
 *   - `ws` is caller-owned device scratch of at least vector_workspace_bytes()
 *     bytes (256-byte aligned); calls sharing one workspace must be ordered on
 *     one stream.
 */
#ifndef VECTOR_H_
#define VECTOR_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VECTOR_API __attribute__((visibility("default")))

#define VECTOR_OK              0
#define VECTOR_ERR_ARG        (-1)  /* null pointer, bad count or flag            */
#define VECTOR_ERR_SHAPE      (-2)  /* shape outside what the kernels support     */
#define VECTOR_ERR_WORKSPACE  (-3)  /* ws too small or misaligned                 */
#define VECTOR_ERR_DTYPE      (-4)  /* unknown element type                       */
#define VECTOR_ERR_HIP        (-5)  /* a HIP call or launch failed                */

typedef enum { VECTOR_F32 = 0, VECTOR_BF16 = 1 } vector_dtype;

/* tiers written by vector_route */
#define VECTOR_TIER_EVICT   0
#define VECTOR_TIER_APPROX  1
#define VECTOR_TIER_RETAIN  2

/* how the base scorer smooths the attention mass along the token axis */
#define VECTOR_POOL_AVG 0
#define VECTOR_POOL_MAX 1

/* One layer of one sequence. */
typedef struct {
  int32_t n_q_heads;      /* Hq, a multiple of n_kv_heads                              */
  int32_t n_kv_heads;     /* Hkv                                                       */
  int32_t head_dim;       /* d: 64 or 128                                              */
  int32_t seq_len;        /* n                                                         */
  int32_t window;         /* w: the observation window is the last w positions, 1<=w<=n */
  int32_t pool_kernel;    /* odd k >= 1: pooling window, stride 1                      */
  int32_t dtype;          /* vector_dtype of q, k, v, W; score and eps are always fp32 */
  int32_t pool_mode;      /* VECTOR_POOL_AVG (zero pad, divisor k) or VECTOR_POOL_MAX   */
  int64_t k_stride_head, k_stride_tok;   /* element strides of k [Hkv, n, d]; 0,0 = packed */
  int64_t v_stride_head, v_stride_tok;   /* element strides of v [Hkv, n, d]; 0,0 = packed */
  int64_t w_stride_head;                 /* element stride between per-head W; 0 with
                                            w_shared != 0 means one W for all heads      */
  int32_t w_shared;
  int32_t reserved2;
} vector_shape;

/* ---- host-only helpers ------------------------------------------------- */

/* Section 3.2: with compression ratio p_c and approximation ratio p_a the
 * retained fraction is 1-p_c-p_a and the approximated fraction 2 p_a.
 * Counts are floors of fraction * n, where a product within 1e-9 of an integer counts as that
 * integer (p_c = 0.9, p_a = 0.05, n = 1000 gives 50 retained, not 49);
 * n_pool = n_retain + n_approx. */
VECTOR_API int vector_budget_counts(int32_t n, double p_c, double p_a, int32_t* n_pool, int32_t* n_approx);
/* Same, from token fractions directly. */
VECTOR_API int vector_budget_counts_frac(int32_t n, double f_retain, double f_approx, int32_t* n_pool, int32_t* n_approx);
/* Section 4, deployment formula: min(p_c/2, (1-p_c-eps)/2). */
VECTOR_API double vector_pa_deploy(double p_c, double eps);
/* Scratch bytes sufficient for any entry point on this shape (batch applies to
 * vector_decode_attn; pass 1 for the compression pass). */
VECTOR_API size_t vector_workspace_bytes(const vector_shape* shape, int32_t n_pool, int32_t n_approx, int32_t batch);
VECTOR_API const char* vector_strerror(int code);

/* ---- the compression pass ---------------------------------------------- */

/* Base importance scorer (Section 3.2 Step 1 needs one; the paper plugs into
 * SnapKV-style scorers).  Per KV head h and token t < n-w:
 *   mass[h,t]  = mean over the G = Hq/Hkv query heads of h and the w window rows
 *                of softmax_t( q . k_t / sqrt(d) ), causal (window row r sees
 *                keys <= n-w+r);
 *   score[h,t] = (1/k) sum_{|j|<=k/2, 0<=t+j<n-w} mass[h,t+j]      (VECTOR_POOL_AVG), or
 *   score[h,t] = max_{|j|<=k/2, 0<=t+j<n-w} mass[h,t+j]            (VECTOR_POOL_MAX);
 * tokens t >= n-w get +inf.
 * q_win: device [Hq, w, d] packed.  k: device, strides from shape.
 * score: device fp32 [Hkv, n] packed (output).
 * The query rows of a KV head are staged in LDS, up to 288 rows (bf16) or 160 rows (fp32) at
 * d = 128, 384 or 288 rows at d = 64.  With more than that (G*w = 512 for 8 query heads per KV
 * head and a 64-token window) the query heads go through the two passes in groups of as many
 * heads as fit, each group adding its share to the column mass: one more read of K per group.
 * VECTOR_ERR_SHAPE only when a single head's w rows exceed the limit. */
VECTOR_API int vector_score(const vector_shape* shape, const void* q_win, const void* k,
                 float* score, void* ws, size_t ws_bytes, void* stream);

/* A query-agnostic scorer (Section 5 pairs VECTOR with scorers that rank tokens by the geometric
 * diversity of their keys and gives no formula; this is one such score): with a_h the direction of
 * the mean of head h's unit-normalised keys, score[h,t] = - cos(k[h,t], a_h); a zero key scores 0.
 * No observation window is involved (shape->window and pool_kernel are ignored).  The result feeds
 * vector_route like any other score.  ws: vector_score_key_diversity_workspace_bytes(shape). */
VECTOR_API size_t vector_score_key_diversity_workspace_bytes(const vector_shape* shape);
VECTOR_API int vector_score_key_diversity(const vector_shape* shape, const void* k, float* score, void* ws,
                               size_t ws_bytes, void* stream);

/* Reconstruction residual (Section 3.2 Step 2), for every token:
 *   eps[h,t] = || v[h,t] - k[h,t] . W[h] ||_2^2, fp32 accumulation.
 * W: device [Hkv, d, d] (or one [d, d] when w_shared).  eps: device fp32 [Hkv, n]. */
VECTOR_API int vector_residual(const vector_shape* shape, const void* k, const void* v, const void* W,
                    float* eps, void* ws, size_t ws_bytes, void* stream);

/* Score and residual in one pass over k (same outputs as the two calls above,
 * within floating-point tolerance; k is streamed once less). */
VECTOR_API int vector_score_residual(const vector_shape* shape, const void* q_win, const void* k, const void* v,
                          const void* W, float* score, float* eps, void* ws, size_t ws_bytes, void* stream);

/* Three-way routing (Section 3.2 Steps 1 and 3), independently per KV head:
 *   pool    = the n_pool tokens of highest score,
 *   approx  = the n_approx pool tokens of lowest eps,
 *   retain  = pool minus approx;  everything else is evicted.
 * Ties go to the lower token index in both selections.  NaN inputs are not
 * supported; -0 and +0 compare equal.
 * score, eps: device fp32 [Hkv, n].  tier: device u8 [Hkv, n] (VECTOR_TIER_*).
 * idx_retain: device i32 [Hkv, n_pool-n_approx], idx_approx: device i32
 * [Hkv, n_approx], both ascending token indices.
 * Requires 0 <= n_approx <= n_pool <= n, n <= 2^20 and n_kv_heads <= 65535 (VECTOR_ERR_SHAPE beyond). */
VECTOR_API int vector_route(int32_t n_kv_heads, int32_t seq_len, const float* score, const float* eps,
                 int32_t n_pool, int32_t n_approx,
                 uint8_t* tier, int32_t* idx_retain, int32_t* idx_approx,
                 void* ws, size_t ws_bytes, void* stream);

/* vector_route for callers that cannot allocate device memory or size a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, outputs
 * and errors as vector_route, without ws: the routing kernels' scratch is a device array of
 * VECTOR_ROUTE_STATIC_SCRATCH_BYTES that lives inside the library (one copy per GPU, held until the
 * process ends; its address is looked up on the first call on a device, on the device that is
 * current then).  The call allocates and frees nothing.  VECTOR_ERR_WORKSPACE when
 * the shape needs more scratch than the array holds (what vector_route would ask its caller for;
 * 8 heads of 131072 tokens fit).  Every call on a GPU uses that GPU's one array: calls on different
 * streams of one GPU must not overlap; calls on one stream are ordered and safe.  Nothing in the
 * array has to be cleared between calls (every call rewrites what it reads). */
#define VECTOR_ROUTE_STATIC_SCRATCH_BYTES (16u << 20)
VECTOR_API size_t vector_route_static_scratch_bytes(void);
VECTOR_API int vector_route_static(int32_t n_kv_heads, int32_t seq_len, const float* score, const float* eps,
                        int32_t n_pool, int32_t n_approx,
                        uint8_t* tier, int32_t* idx_retain, int32_t* idx_approx, void* stream);

/* Packed cache (Section 3.2: keys of the whole pool, values of retained tokens
 * only).  Row gather by the index lists:
 *   k_ret[h,s,:] = k[h, idx_retain[h,s], :],  v_ret likewise,
 *   k_apx[h,s,:] = k[h, idx_approx[h,s], :].
 * k_ret, v_ret: device [Hkv, cap_retain, d] with cap_retain >= n_retain (rows
 * beyond n_retain are left untouched for decode-time appends);
 * k_apx: device [Hkv, n_approx, d]. */
VECTOR_API int vector_compact(const vector_shape* shape, const void* k, const void* v,
                   const int32_t* idx_retain, const int32_t* idx_approx,
                   int32_t n_retain, int32_t n_approx,
                   void* k_ret, void* v_ret, void* k_apx, int32_t cap_retain, void* stream);

/* The whole compression pass of one layer in one call: vector_score_residual, vector_route
 * and vector_compact with the same arguments and the same outputs, bit for bit; everything is
 * validated before the first launch.  ws: vector_compress_workspace_bytes(shape, n_pool, n_approx)
 * bytes. */
VECTOR_API size_t vector_compress_workspace_bytes(const vector_shape* shape, int32_t n_pool, int32_t n_approx);
VECTOR_API int vector_compress(const vector_shape* shape, const void* q_win, const void* k, const void* v, const void* W,
                    int32_t n_pool, int32_t n_approx, float* score, float* eps, uint8_t* tier,
                    int32_t* idx_retain, int32_t* idx_approx, void* k_ret, void* v_ret, void* k_apx,
                    int32_t cap_retain, void* ws, size_t ws_bytes, void* stream);

/* vector_score_residual and vector_compress for callers that already hold the log-sum-exp of the
 * window queries' attention rows (Section 3.2 Step 1's scorer attends from the last w positions; the
 * attention kernel of the prefill has computed exactly these rows and returns their log-sum-exp).
 * Then the first of the two passes over k is not needed.
 *   lse   device fp32: lse[hq * lse_stride_head + r] = log sum_{t <= n - w + r} exp(q[hq,r] . k[hq / G, t] / sqrt(d))
 *         (natural logarithm, causal, r = 0 .. w-1 the last w positions); lse_stride_head in elements,
 *         0 meaning w (a slice of a [Hq, n] array has stride n).
 * Same outputs as the calls without it, to the tolerance of the fp32 log-sum-exp given; a wrong
 * lse gives wrong scores, nothing checks it.  Other arguments, layouts and errors as there. */
VECTOR_API int vector_score_residual_lse(const vector_shape* shape, const void* q_win, const void* k, const void* v,
                              const void* W, const float* lse, int64_t lse_stride_head, float* score, float* eps,
                              void* ws, size_t ws_bytes, void* stream);
VECTOR_API int vector_compress_lse(const vector_shape* shape, const void* q_win, const void* k, const void* v, const void* W,
                        const float* lse, int64_t lse_stride_head,
                        int32_t n_pool, int32_t n_approx, float* score, float* eps, uint8_t* tier,
                        int32_t* idx_retain, int32_t* idx_approx, void* k_ret, void* v_ret, void* k_apx,
                        int32_t cap_retain, void* ws, size_t ws_bytes, void* stream);

/* The compression pass of one layer for a batch of sequences of unequal length (Section 3.2 applies
 * per sequence: every sequence is scored, routed and packed on its own, with its own counts).
 * Sizes are host arrays of `batch` entries; shape->seq_len is ignored.  With
 * T_b = seq_len[0] + .. + seq_len[b-1], R_b and A_b the same running sums of n_pool - n_approx and of
 * n_approx, and C_b that of cap_retain:
 *   k, v        device, ragged along tokens: sequence b owns rows T_b .. T_b + seq_len[b] - 1 of every
 *               head; strides from shape, packed (0, 0) meaning [Hkv, T, d] with T the total;
 *   q_win       device [batch, Hq, w, d];  W as in vector_compress (shared by the sequences);
 *   score, eps, tier   sequence after sequence: block b is [Hkv, seq_len[b]] and starts at element Hkv * T_b;
 *   idx_retain  block b is [Hkv, n_pool[b] - n_approx[b]] at element Hkv * R_b, idx_approx block b is
 *               [Hkv, n_approx[b]] at element Hkv * A_b; token indices count from the sequence's first row;
 *   k_ret, v_ret   block b is [Hkv, cap_retain[b], d] at row Hkv * C_b;  k_apx block b is
 *               [Hkv, n_approx[b], d] at row Hkv * A_b
 * (the blocks of a vector_cache with per-sequence capacities, below).  Each sequence gives exactly
 * what vector_compress gives for it alone.  Every sequence must satisfy vector_compress's
 * conditions (window <= seq_len[b], n_approx[b] <= n_pool[b] <= seq_len[b],
 * cap_retain[b] >= n_pool[b] - n_approx[b]); everything is validated before the first launch.
 * Sequences share their launches, whatever their lengths: consecutive sequences with the same length,
 * counts and capacity have their heads stacked into one problem; up to 64 consecutive sequences that
 * differ go through one set of launches in which every workgroup looks up its own sequence's
 * parameters (which are those vector_compress would compute for it, so the results do not change;
 * the parameter tables live at the start of ws and are written by small copy launches, nothing is
 * read from host memory after the call returns).  Parts follow each other on `stream` and share ws:
 * vector_compress_batch_workspace_bytes(shape, batch) bytes (the sequences of a part each have their
 * own piece of it).  A sequence with n_pool = 0, or a shape whose G * w query rows need more than one
 * pair of passes, is taken on its own. */
typedef struct {
  int32_t batch;
  const int32_t* seq_len;      /* host [batch] */
  const int32_t* n_pool;       /* host [batch] */
  const int32_t* n_approx;     /* host [batch] */
  const int32_t* cap_retain;   /* host [batch] */
} vector_batch;
VECTOR_API size_t vector_compress_batch_workspace_bytes(const vector_shape* shape, const vector_batch* batch);
VECTOR_API int vector_compress_batch(const vector_shape* shape, const vector_batch* batch, const void* q_win, const void* k,
                          const void* v, const void* W, float* score, float* eps, uint8_t* tier,
                          int32_t* idx_retain, int32_t* idx_approx, void* k_ret, void* v_ret, void* k_apx,
                          void* ws, size_t ws_bytes, void* stream);


/* ---- decode attention over packed caches -------------------------------- */

typedef struct {
  int32_t batch, n_q_heads, n_kv_heads, head_dim;
  int32_t dtype;                  /* vector_dtype of the cache, q, W and out            */
  int32_t cap_retain, n_approx;   /* capacities: of every sequence, or (per-sequence
                                     capacities below) the largest of the batch         */
  int32_t w_shared;               /* non-zero: W is one [d, d] for all heads            */
  const int32_t* len_retain;      /* device [batch]: live rows of the retained segment
                                     (compressed + appended), 0 <= len <= capacity      */
  const void* k_ret;              /* device [batch, Hkv, cap_retain, d]                 */
  const void* v_ret;              /* device [batch, Hkv, cap_retain, d]                 */
  const void* k_apx;              /* device [batch, Hkv, n_approx, d]                   */
  const void* W;                  /* device [Hkv, d, d]                                 */
  /* Per-sequence capacities (sequences compressed at their own lengths): all four null, or all
   * four device arrays of `batch` entries.  Then sequence b's retained block is
   * [Hkv, cap_retain_seq[b], d] starting at row ret_row_start[b] of k_ret / v_ret, its
   * approximated block [Hkv, n_approx_seq[b], d] starting at row apx_row_start[b] of k_apx, with
   * cap_retain and n_approx above then only steer how the work is split: give the largest of the batch. */
  const int32_t* cap_retain_seq;
  const int32_t* n_approx_seq;
  const int64_t* ret_row_start;
  const int64_t* apx_row_start;
  /* Paged retained segments (the segment that grows during generation): ret_block_table null, or a
   * device array [batch, Hkv, ret_blocks_per_seq] of block ids.  Then k_ret / v_ret are pools of
   * blocks of ret_block_rows rows each ([n_blocks, ret_block_rows, d]; ret_block_rows a power of two,
   * at least 16), row r of sequence b and KV head h is row r % ret_block_rows of block
   * ret_block_table[b][h][r / ret_block_rows], and cap_retain <= ret_blocks_per_seq * ret_block_rows is
   * the capacity of every sequence (table entries up to that capacity must name blocks that exist).
   * The per-sequence arrays above must be null with a block table; the approximated segment stays
   * contiguous ([batch, Hkv, n_approx, d]). */
  const int32_t* ret_block_table;
  int32_t ret_block_rows;
  int32_t ret_blocks_per_seq;
} vector_cache;

/* One query token per sequence (Section 3.2 Step 3: discarded values are
 * rebuilt from their keys during generation).  Per sequence b and query head
 * qh (KV head h = qh / G): one softmax over the live retained rows and the
 * approximated rows together, logits q . k_t * scale, and
 *   out = sum_ret p_t v_t + sum_apx p_t (k_t . W[h]).
 * q: device [batch, Hq, d]; out: device [batch, Hq, d], same dtype as the cache.
 * Hq / Hkv may be 1 .. 8, 10, 12 or 16 (VECTOR_ERR_SHAPE otherwise).
 * flags: 0, or VECTOR_DECODE_LITERAL to rebuild v_hat = k . W for every approximated row on
 * the matrix cores before weighting it (bf16 caches only); by default the weighted keys are
 * summed first and W is applied once, (sum p_t k_t) . W, which is the same sum in another
 * order and far less work.  A sequence with no live token yields zeros. */
#define VECTOR_DECODE_LITERAL 1
/* flags: VECTOR_DECODE_OUT_F32 stores out as fp32 [batch, Hq, d] whatever the cache dtype (the
 * kernels accumulate in fp32; without the flag a bf16 cache rounds the result to bf16 on store). */
#define VECTOR_DECODE_OUT_F32 2
VECTOR_API int vector_decode_attn(const vector_cache* cache, const void* q, float scale, void* out,
                       int32_t flags, void* ws, size_t ws_bytes, void* stream);

/* One decode step with its append (Section 3.2 keeps what generation adds exactly): the new
 * token's key and value (k_new, v_new: device [batch, Hkv, d], cache dtype) join the retained
 * segment of their sequence as row len_retain[b], the query attends over the cache with that row
 * included, and len_retain[b] grows by one, all inside the two launches of vector_decode_attn
 * (the workgroup whose rows include the new one stores it; the step itself reads it from k_new /
 * v_new).  Same arguments, flags, outputs and errors as vector_decode_attn otherwise.  The call
 * writes cache->k_ret, v_ret (one row per sequence and KV head) and cache->len_retain, although the
 * struct declares them const.  A sequence whose retained block is already full (len_retain[b] equal
 * to its capacity) still attends over its new token, but the token is not stored and the length
 * stays: give the blocks room for the tokens to come.  VECTOR_ERR_ARG if cap_retain < 1. */
VECTOR_API int vector_decode_step(const vector_cache* cache, const void* q, const void* k_new, const void* v_new,
                       float scale, void* out, int32_t flags, void* ws, size_t ws_bytes, void* stream);

/* ---- measurement ---------------------------------------------------------- */

/* Optional per-kernel timing for benchmarks.  While enabled, every kernel launch
 * of the library is bracketed by HIP events recorded on the launch stream
 * (events are created on demand on the host; no device memory is involved).
 * vector_timing_read waits for the recorded launches of one kernel, returns
 * their summed duration in milliseconds and their count, and resets that
 * kernel's record.  kernel_id runs from 0 to vector_timing_kernels()-1;
 * vector_timing_name gives the kernel's name.  Single host thread only. */
VECTOR_API int vector_timing_enable(int on);
VECTOR_API int vector_timing_kernels(void);
VECTOR_API const char* vector_timing_name(int kernel_id);
VECTOR_API int vector_timing_read(int kernel_id, double* total_ms, int64_t* launches);

/* ---- keys cached after rotary position embedding -------------------------- */

/* Section 3.1, "RoPE Decoupling": the value map is fitted on keys as projected, while a
 * cache holds them after the rotary embedding of their position.  Wherever a value is
 * rebuilt from a cached key (the residual of Step 2, the approximated rows of decode
 * attention), the key is first turned back by its position; attention logits and
 * importance scores use the cached keys unchanged.
 * The rotation of a row at position m turns pair i by the angle m * inv_freq[i]:
 * (a, b) -> (a cos - b sin, a sin + b cos). */
typedef struct {
  const double* inv_freq;    /* HOST memory, head_dim/2 values, radians per position;
                                read during the call, not kept                          */
  int32_t interleaved;       /* 0: pair i = (x[i], x[i + d/2]); 1: pair i = (x[2i], x[2i+1]) */
  int32_t pos_offset;        /* added to every position; positions (offset included)
                                must lie in [0, 2^24)                                   */
  const int32_t* positions;  /* device memory or NULL.  vector_*residual_rope: [n], the
                                position of each row of k (NULL: the row index).
                                vector_decode_attn_rope: [batch, Hkv, n_approx] (one per
                                row of k_apx, also with per-sequence capacities), the
                                original position of each approximated row (NULL: the
                                row index).                                             */
} vector_rope;

/* vector_residual / vector_score_residual on post-RoPE keys: same arguments, layouts,
 * workspace and errors; eps[h,t] = || v[h,t] - (R^-1 k[h,t]) . W[h] ||^2, the score is
 * that of vector_score on the same k.  VECTOR_ERR_ARG for a NULL rope or inv_freq. */
VECTOR_API int vector_residual_rope(const vector_shape* shape, const void* k, const void* v, const void* W,
                         const vector_rope* rope, float* eps, void* ws, size_t ws_bytes, void* stream);
VECTOR_API int vector_score_residual_rope(const vector_shape* shape, const void* q_win, const void* k, const void* v,
                               const void* W, const vector_rope* rope, float* score, float* eps, void* ws,
                               size_t ws_bytes, void* stream);
/* vector_compress on post-RoPE keys: vector_score_residual_rope, vector_route and vector_compact in
 * one call, the same outputs bit for bit (the packed cache holds the keys as cached, rotated: the
 * decode-time entry points turn approximated rows back).  ws: vector_compress_workspace_bytes. */
VECTOR_API int vector_compress_rope(const vector_shape* shape, const vector_rope* rope, const void* q_win, const void* k,
                         const void* v, const void* W, int32_t n_pool, int32_t n_approx, float* score, float* eps,
                         uint8_t* tier, int32_t* idx_retain, int32_t* idx_approx, void* k_ret, void* v_ret, void* k_apx,
                         int32_t cap_retain, void* ws, size_t ws_bytes, void* stream);
/* vector_compress_batch on post-RoPE keys (vector_compress_rope per sequence).  rope->positions is
 * NULL (every sequence's positions are its row indices, plus pos_offset) or a device array ragged
 * along the token axis like k: [T], sequence b owning entries T_b .. T_b + seq_len[b] - 1. */
VECTOR_API int vector_compress_batch_rope(const vector_shape* shape, const vector_batch* batch, const vector_rope* rope,
                               const void* q_win, const void* k, const void* v, const void* W, float* score, float* eps,
                               uint8_t* tier, int32_t* idx_retain, int32_t* idx_approx, void* k_ret, void* v_ret,
                               void* k_apx, void* ws, size_t ws_bytes, void* stream);

/* The compression pass with any combination of the two variants above: keys cached after RoPE
 * (rope) and the window rows' log-sum-exp handed in (lse), as a production prefill has them.
 * options NULL, or with both members NULL, is vector_compress / vector_compress_batch.
 *   rope             as in vector_compress_rope / vector_compress_batch_rope, or NULL
 *   lse              as in vector_compress_lse, or NULL; for a batch: device [batch, Hq, lse_stride_head]
 *   lse_stride_head  floats between two query heads' rows (0: w); must be 0 when lse is NULL */
typedef struct {
  const vector_rope* rope;
  const float* lse;
  int64_t lse_stride_head;
} vector_compress_options;
VECTOR_API int vector_compress_ex(const vector_shape* shape, const vector_compress_options* options, const void* q_win,
                       const void* k, const void* v, const void* W, int32_t n_pool, int32_t n_approx, float* score,
                       float* eps, uint8_t* tier, int32_t* idx_retain, int32_t* idx_approx, void* k_ret, void* v_ret,
                       void* k_apx, int32_t cap_retain, void* ws, size_t ws_bytes, void* stream);
VECTOR_API int vector_compress_batch_ex(const vector_shape* shape, const vector_batch* batch, const vector_compress_options* options,
                             const void* q_win, const void* k, const void* v, const void* W, float* score, float* eps,
                             uint8_t* tier, int32_t* idx_retain, int32_t* idx_approx, void* k_ret, void* v_ret,
                             void* k_apx, void* ws, size_t ws_bytes, void* stream);
/* vector_decode_attn on a post-RoPE cache: out = sum_ret p_t v_t + sum_apx p_t ((R^-1 k_t) . W[h]),
 * logits from the cached keys.  VECTOR_DECODE_LITERAL is not available here (VECTOR_ERR_DTYPE). */
VECTOR_API int vector_decode_attn_rope(const vector_cache* cache, const vector_rope* rope, const void* q, float scale,
                            void* out, int32_t flags, void* ws, size_t ws_bytes, void* stream);
/* vector_decode_step on a post-RoPE cache: k_new is the new token's key as cached (after its rotary
 * embedding); retained rows are never un-rotated, so the append itself is the same. */
VECTOR_API int vector_decode_step_rope(const vector_cache* cache, const vector_rope* rope, const void* q, const void* k_new,
                            const void* v_new, float scale, void* out, int32_t flags, void* ws, size_t ws_bytes,
                            void* stream);

/* ---- calibration of the value map ---------------------------------------- */

/* Section 3.1: the least-squares map from keys to values, per KV head and without intercept,
 *   W[h] = argmin_W || k[h] W - v[h] ||_F^2      (v_hat = k . W; the transpose of the paper's W_OLS),
 * from shape->seq_len calibration tokens (k, v: device [Hkv, seq_len, d] with the shape's
 * strides and dtype; keys as projected, i.e. before any rotary embedding).  Solved through
 * the normal equations: the two d x d products are accumulated on the matrix cores in
 * fp32 per chunk of tokens and summed in fp64; Cholesky and the triangular solves run in fp64.
 * W: device [Hkv, d, d] (output, shape dtype).  ws: vector_calibrate_workspace_bytes(shape)
 * bytes of device scratch, 256-byte aligned.  VECTOR_ERR_ARG if seq_len < head_dim.  A head
 * whose K^T K is not positive definite gets NaN in its W. */
VECTOR_API size_t vector_calibrate_workspace_bytes(const vector_shape* shape);
VECTOR_API int vector_calibrate(const vector_shape* shape, const void* k, const void* v, void* W, void* ws,
                     size_t ws_bytes, void* stream);

/* Section 3.1: how well the map predicts the values of a token set (the paper reports it on
 * held-out sequences), per KV head:
 *   out[h][0] r2_centered    1 - sse / sst_centered   (coefficient of determination, all value
 *                                                      dimensions pooled)
 *   out[h][1] r2_uncentered  1 - sse / sst_raw        (one minus the relative error of Section 4)
 *   out[h][2] sse            sum_t || v_t - k_t . W[h] ||^2
 *   out[h][3] sst_centered   sum_t || v_t - mean_t v ||^2        out[h][4] sst_raw  sum_t || v_t ||^2
 * k, v, W as for vector_residual; out: device fp64 [Hkv, VECTOR_R2_FIELDS]; ws:
 * vector_r2_workspace_bytes(shape) bytes.  Residuals in fp32 as in vector_residual, sums in fp64. */
#define VECTOR_R2_FIELDS 5
VECTOR_API size_t vector_r2_workspace_bytes(const vector_shape* shape);
VECTOR_API int vector_r2(const vector_shape* shape, const void* k, const void* v, const void* W, double* out, void* ws,
              size_t ws_bytes, void* stream);

/* ---- distortion diagnostics ------------------------------------------------ */

/* Section 4: with importance weights w (device fp32 [Hkv, n], summing to one per head), the
 * routing (tier), the residuals (eps) and the values v [Hkv, n, d] (shape strides, dtype):
 *   out[h][0] E          sum_evicted w_i + sum_approx w_i eps_i / ||v_i||^2
 *   out[h][1] w_evict    sum of w over evicted tokens        out[h][2] w_approx  same, approximated
 *   out[h][3] mu_approx  mean of eps_i / ||v_i||^2 over approximated tokens
 *   out[h][4] r2_approx  1 - mu_approx
 *   out[h][5] w_bar      (1 - w_evict) / (fraction of tokens in the pool)
 *   out[h][6] w_star     n * largest weight among evicted tokens (0 if none)
 *   out[h][7] threshold  w_bar / (w_star + w_bar): Proposition 1's bound on r2_approx
 *   out[h][8] n_approx   out[h][9] n_evict
 * out: device fp64 [Hkv, VECTOR_DISTORTION_FIELDS].  Sums run in fp64 in a fixed order.
 * ws: vector_distortion_workspace_bytes(shape) bytes, 256-byte aligned. */
#define VECTOR_DISTORTION_FIELDS 10
VECTOR_API size_t vector_distortion_workspace_bytes(const vector_shape* shape);
VECTOR_API int vector_distortion(const vector_shape* shape, const float* weights, const uint8_t* tier, const float* eps,
                      const void* v, double* out, void* ws, size_t ws_bytes, void* stream);

/* Diagnostic: the reconstruction contraction of Section 3.2 Step 2 (v_hat = k W, then the
 * squared distance to v) with memory out of the picture.  Same arguments, layout and
 * arithmetic as vector_residual for bf16 inputs, but every workgroup runs the arithmetic
 * of each tile `repeat` times on the operands it already holds in registers and LDS, so
 * (time(repeat = r) - time(repeat = 1)) / (r - 1) is one pass of the contraction code at
 * the rate the matrix cores sustain when they are not waiting for HBM.  eps receives the
 * same values as vector_residual.  VECTOR_ERR_DTYPE for fp32 inputs. */
VECTOR_API int vector_probe_residual_mfma(const vector_shape* shape, const void* k, const void* v, const void* W,
                               float* eps, int32_t repeat, void* stream);

/* Diagnostic: the matrix-core ceiling as measured on this chip.  Launches 256 workgroups of 16 waves
 * that each run `iters` rounds of four independent 32x32x16 bf16 MFMAs on register operands, and
 * writes the flop count of the launch to *flops (host).  out: device fp32 [262144] (a sink that
 * keeps the loop alive; its contents mean nothing).  Time the launch on `stream` to get FLOP/s. */
VECTOR_API int vector_probe_mfma_loop(float* out, int32_t iters, int64_t* flops, void* stream);

/* Diagnostic: the rate at which this chip streams a buffer that is only read (what the compression
 * pass and the decode step mostly do), next to the device copy that reads and writes.  1024
 * workgroups each read a contiguous slice of src (device, 16-byte aligned, `bytes` long) with 16-byte
 * loads, eight in flight per thread; *bytes_read (host) receives what the launch reads (`bytes`
 * rounded down to whole rounds of loads of 64 KiB per workgroup; VECTOR_ERR_ARG for a NULL or
 * misaligned pointer and for less than 64 MiB).  out: device fp32 [1024], a sink.  Time the launch on `stream`. */
VECTOR_API int vector_probe_read_stream(const void* src, size_t bytes, float* out, int64_t* bytes_read, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* VECTOR_H_ */
