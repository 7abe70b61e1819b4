/*
 * mixkv.h -- C ABI of libmixkv: MixKV's prefill-time KV-cache compression step
 * on one MI355X (gfx950).
 *
 * For every layer l and KV head h the library scores each cached key, mixes an
 * importance score with a diversity score according to the head's redundancy,
 * keeps the top-B entries and gathers the kept K/V rows into a compacted cache
 * (paper: Sec. 3.1 "KV Cache Compression" for the operator; Sec. 3.2 for the
 * importance and diversity scores; Sec. 3.3, Eq. 3-5 for the redundancy and the
 * head-wise mix; Appendix Algorithm 1 for the whole loop).
 *
 * Conventions
 *   Pointers   Members of mixkv_layer_in / mixkv_layer_out and `workspace` are
 *              DEVICE pointers owned by the caller.  The params struct and the
 *              arrays of layer structs are HOST memory, read during the call only.
 *   Ownership  The library allocates no device memory and keeps no state between
 *              calls.  Two calls may run concurrently on different streams if they
 *              use different workspaces and outputs.
 *   Ordering   All work is enqueued on `hip_stream` (a hipStream_t, NULL = the
 *              default stream).  Calls return without synchronising; outputs are
 *              valid once the stream has been synchronised.
 *   Errors     Every entry point returns a mixkv_status.  Arguments are validated
 *              on the host before anything is launched; on an argument error no
 *              output is touched.  HIP launch failures map to MIXKV_ERR_HIP.
 *   Notation   N cached tokens (the paper's T), D head dim, W window length,
 *              B budget per head (window included), B' = B - W (Algorithm 1),
 *              Nc = N - W candidates, G = n_q_heads / n_kv_heads.
 *   Layout     K, V: [batch, n_kv_heads, N, D], D contiguous, strides in elements.
 *              Qwin: [batch, n_q_heads, W, D] contiguous; query head g serves KV
 *              head g / G.  Row starts must be 16-byte aligned.
 */
#ifndef MIXKV_H
#define MIXKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MIXKV_VERSION 10
#define MIXKV_MAX_LAYERS 128      /* layers per call */
#define MIXKV_MAX_WINDOW 64
#define MIXKV_MAX_GROUP_ROWS 512  /* G * W */

typedef enum {
  MIXKV_OK = 0,
  MIXKV_ERR_INVALID_ARG = 1,
  MIXKV_ERR_UNSUPPORTED = 2,
  MIXKV_ERR_WORKSPACE_TOO_SMALL = 3,
  MIXKV_ERR_HIP = 4
} mixkv_status;

typedef enum { MIXKV_F32 = 0, MIXKV_BF16 = 1 } mixkv_dtype;
typedef enum { MIXKV_POOL_NONE = 0, MIXKV_POOL_AVG = 1, MIXKV_POOL_MAX = 2 } mixkv_pool;
/* How many rows a head keeps (Sec. 3.1: the budget B; Algorithm 1, budget line).
 *   FIXED          every head of every layer keeps params->budget rows
 *   HEAD_ADAPTIVE  the heads of one (layer, batch item) share a pool of n_kv_heads * budget rows, split by score
 *   PER_HEAD       the caller gives the rows kept by every (layer, KV head) in params->head_budgets: layer-wise
 *                  (pyramid) and static head-wise allocation schemes (Sec. 4.1, Table 1) compute such tables */
typedef enum { MIXKV_BUDGET_FIXED = 0, MIXKV_BUDGET_HEAD_ADAPTIVE = 1, MIXKV_BUDGET_PER_HEAD = 2 } mixkv_budget_mode;
/* Intrinsic importance (Sec. 3.2): none, the value norm |V_i| (the method's choice), or the negative
 * key norm -|K_i| (the KNorm alternative of the ablation, Sec. 4.3 / Table 4). */
typedef enum { MIXKV_INTRINSIC_NONE = 0, MIXKV_INTRINSIC_VNORM = 1, MIXKV_INTRINSIC_KNORM = 2 } mixkv_intrinsic;
/* How importance and diversity are combined into s_comp (Sec. 3.3, Eq. 5 and the ablation rows of
 * Table 4).  s_div_scaled is the diversity after min-max and mean matching in every mode.
 *   HEAD_ADAPTIVE  (1 - r) s_imp + r s_div_scaled with the head's own redundancy r (Eq. 4, Eq. 5)
 *   SUM            s_imp + s_div_scaled, no head weights
 *   DIV_ONLY       s_div_scaled
 *   IMP_ONLY       s_imp
 *   GIVEN_R        Eq. 5 with the caller's weight mixkv_layer_in.r_given in place of r (head weights
 *                  measured offline and shared by all samples) */
typedef enum {
  MIXKV_MIX_HEAD_ADAPTIVE = 0, MIXKV_MIX_SUM = 1, MIXKV_MIX_DIV_ONLY = 2, MIXKV_MIX_IMP_ONLY = 3, MIXKV_MIX_GIVEN_R = 4
} mixkv_mix;

typedef struct {
  mixkv_dtype dtype;         /* element type of K, V, Qwin and of K_out, V_out */
  int32_t batch;
  int32_t n_q_heads;         /* multiple of n_kv_heads */
  int32_t n_kv_heads;
  int32_t head_dim;          /* D: 64 or 128 */
  int32_t seq_len;           /* N >= 2, window included */
  int32_t window;            /* 1 <= W <= MIXKV_MAX_WINDOW and W < N; the queries are the last W positions */
  int32_t budget;            /* W <= B <= N rows kept per head (fixed mode) / on average (adaptive mode) / on average
                                at most (per-head mode: n_kv_heads * B rows is the capacity of one batch item's outputs) */
  mixkv_pool pool;           /* 1-D pooling of the window attention over candidates */
  int32_t pool_kernel;       /* odd, 1..63; ignored for MIXKV_POOL_NONE */
  int32_t causal_window;     /* 1: window query w (position Nc+w) attends to keys 0..Nc+w; 0: to all N keys */
  float softmax_scale;       /* multiplies Q.K before the softmax; the library never rescales Q itself */
  float eps;                 /* the epsilon of the paper's min-max and mean-matching formulas, > 0 */
  mixkv_intrinsic intrinsic; /* VNORM: importance = attention + scaled value norm (Sec. 3.2, Eq. 2); see the enum */
  mixkv_mix mix;             /* HEAD_ADAPTIVE: (1 - r) * importance + r * diversity (Sec. 3.3, Eq. 5); see the enum */
  mixkv_budget_mode budget_mode;
  int32_t budget_floor;      /* adaptive mode: minimum non-window rows per head, 0 <= floor <= B - W */
  const int32_t *head_budgets; /* HOST, per-head mode only (else ignored, may be NULL): [n_layers, n_kv_heads], rows
                                kept by KV head h of layer l (the l-th layer struct of the call), window included,
                                the same for every batch item; W <= b <= N and sum_h b[l][h] <= n_kv_heads * B */
} mixkv_params;

/* One layer of the cache to compress. */
typedef struct {
  const void *K;             /* [batch, n_kv_heads, N, D] */
  const void *V;             /* same shape and strides as K */
  int64_t kv_stride_b, kv_stride_h, kv_stride_n;   /* in elements; kv_stride_n >= D */
  const void *Qwin;          /* [batch, n_q_heads, W, D] contiguous, post-RoPE observation-window queries */
  const float *r_given;      /* [batch, n_kv_heads] head weights for MIXKV_MIX_GIVEN_R, finite; ignored (may be
                                NULL) in every other mix mode */
  const float *window_lse;   /* optional [batch, n_q_heads, W]: for every window query row the natural logarithm of
                                sum_i exp(softmax_scale * Q.K_i) over the keys the row attends to (all N, or 0..Nc+w
                                with causal_window), as the prefill attention kernel already produced it for these
                                rows.  When given (then for every layer of the call) the first pass computes no
                                window logits and the softmax is normalised by these values; NULL: computed here */
} mixkv_layer_in;

/* Outputs for one layer.  Which members are required is stated per entry point. */
typedef struct {
  float *scores;             /* [batch, n_kv_heads, N]: the mixed score s_comp at candidates, +inf at the W window slots */
  float *redundancy;         /* [batch, n_kv_heads]: the head's redundancy r (Eq. 4) */
  int32_t *indices;          /* kept positions, ascending per head, the W window positions last.
                                fixed: [batch, n_kv_heads, B]; adaptive and per-head: [batch, n_kv_heads * B], heads packed
                                back to back (per-head mode may leave the tail of a batch item's slots untouched) */
  int32_t *counts;           /* [batch, n_kv_heads] rows kept per head (B in fixed mode) */
  int32_t *offsets;          /* adaptive and per-head: [batch, n_kv_heads + 1] exclusive prefix sums of counts; may be
                                NULL in fixed mode */
  void *K_out, *V_out;       /* rows of K / V at `indices`, copied bit for bit, D contiguous.
                                fixed: [batch, n_kv_heads, B, D]; adaptive and per-head: [batch, n_kv_heads * B, D] packed
                                like indices */
} mixkv_layer_out;

/*
 * Bytes of device workspace mixkv_score / mixkv_compress need for `n_layers`
 * layers of this shape.  mixkv_select needs none and accepts NULL, except in
 * per-head budget mode, where it stages the budget table there and needs
 * n_layers * n_kv_heads * 4 bytes.  In head-adaptive mode mixkv_select uses a
 * workspace of n_layers * batch * n_kv_heads * 8192 bytes if it is given one
 * (two 1024-entry candidate lists per head) and a head's candidates fit them,
 * M = floor + n_kv_heads * (budget - window - floor) <= 1024 and n_kv_heads * M
 * <= 4096: every head is then ranked by a
 * workgroup of its own and a small kernel splits the pool, about ten times
 * faster on long caches than without, where one workgroup per batch item ranks
 * the scores of all heads; the results are the same.  This function's figure
 * is always enough for mixkv_select.
 * Host only; touches no GPU (head_budgets is not read).  The workspace needs no
 * initialisation and 256-byte alignment.
 */
mixkv_status mixkv_workspace_size(const mixkv_params *params, int32_t n_layers, size_t *bytes);

/*
 * Score every cached key (Algorithm 1, step 1 and the mixing half of step 2).
 * Per (layer, batch item, KV head):
 *   s_ex   mean over the G*W window queries of softmax attention on key i (Sec. 3.2,
 *          extrinsic importance), pooled over candidates; the rows' normalisers are computed
 *          here or taken from in[l].window_lse;
 *   s_imp  s_ex + min-max normalised value norm scaled to mean(s_ex) (Sec. 3.2, Eq. 2);
 *   s_div  -Khat_i . mean_j Khat_j with Khat the L2-normalised keys, all N keys in the mean
 *          (Sec. 3.2, diversity metrics), min-max normalised and scaled to mean(s_imp) (Sec. 3.3);
 *   r      (N^2 |mean Khat|^2 - N) / (N (N-1))   (Sec. 3.3, Eq. 3-4);
 *   s_comp (1 - r) s_imp + r s_div_scaled         (Sec. 3.3, Eq. 5).
 * All minima, maxima and means are over the Nc candidates.  params->intrinsic and params->mix
 * switch to the ablation's variants (Sec. 4.3, Table 4): with KNORM, -|K_i| takes the place of
 * |V_i| in s_imp; the mix modes change the last line only.
 * Writes out[l].scores (required) and out[l].redundancy (optional, may be NULL; always the head's
 * own r of Eq. 4, whatever the mix mode).
 */
mixkv_status mixkv_score(const mixkv_params *params, const mixkv_layer_in *in, mixkv_layer_out *out,
                         int32_t n_layers, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * TopB on caller-provided scores (Sec. 3.1; Algorithm 1, TopB step with B' = B - W and the
 * window excluded from ranking and always kept).  Reads out[l].scores (only the Nc candidate
 * slots are read); writes out[l].indices, out[l].counts and, if non-NULL, out[l].offsets
 * (required in adaptive mode).  Ties go to the smaller position.  NaN scores are not supported.
 * Fixed mode: each head keeps its B' best candidates.  Head-adaptive mode, per (layer, batch
 * item): every head keeps its budget_floor best candidates, then the remaining
 * n_kv_heads * (B' - budget_floor) slots go to the best remaining candidates of all heads
 * together (ties: smaller head, then smaller position).  Per-head mode: head h of layer l keeps its
 * head_budgets[l][h] - W best candidates.
 */
mixkv_status mixkv_select(const mixkv_params *params, mixkv_layer_out *out, int32_t n_layers,
                          void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The whole step (Algorithm 1): score, select, and gather the kept K/V rows (Sec. 3.1,
 * Khat, Vhat = TopB(K, V, {s_i})).  Writes indices, counts, K_out, V_out (all required),
 * offsets (required in adaptive mode), and scores / redundancy when non-NULL.
 * K_out / V_out must not overlap K / V.
 */
mixkv_status mixkv_compress(const mixkv_params *params, const mixkv_layer_in *in, mixkv_layer_out *out,
                            int32_t n_layers, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * mixkv_compress for callers that can neither allocate device memory nor hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * workspace is an array of MIXKV_STATIC_SCRATCH_BYTES inside the library's own device data (every
 * GPU the library runs on holds one from load until the process ends); inputs and outputs are the
 * caller's as in mixkv_compress, and so are the results, bit for bit.  The call allocates and
 * frees nothing.  Shapes whose workspace (mixkv_workspace_size) exceeds the array return
 * MIXKV_ERR_WORKSPACE_TOO_SMALL and touch nothing: 32 MiB hold the whole 28-layer 8K cache of the
 * 28Q/4KV shape in one call; larger caches go layer group by layer group.  Nothing in the array has
 * to start at zero (every word is written before it is read within a call) and it keeps the last
 * call's contents.  All calls on one GPU share the array: calls that overlap in time on one GPU
 * (different streams, or different host threads) race; serialise them or use mixkv_compress with
 * separate workspaces.  The first call on a device looks the array's address up once
 * (hipGetSymbolAddress); make that call outside a graph capture.
 */
#define MIXKV_STATIC_SCRATCH_BYTES (32u << 20)
mixkv_status mixkv_compress_static(const mixkv_params *params, const mixkv_layer_in *in, mixkv_layer_out *out,
                                   int32_t n_layers, void *hip_stream);

/*
 * Profiling aid: mixkv_compress with every kernel launch bracketed by a pair of HIP events on
 * `hip_stream`.  Synchronises the stream before returning and writes the milliseconds each
 * pipeline stage took to the HOST array stage_ms[MIXKV_N_STAGES] (summed over launch groups when
 * n_layers exceeds one group).  Stage names come from mixkv_stage_name.  Outputs are those of
 * mixkv_compress (Algorithm 1).
 */
#define MIXKV_N_STAGES 5
mixkv_status mixkv_compress_profiled(const mixkv_params *params, const mixkv_layer_in *in, mixkv_layer_out *out,
                                     int32_t n_layers, void *workspace, size_t workspace_bytes, void *hip_stream,
                                     float *stage_ms);
const char *mixkv_stage_name(int32_t stage);

/*
 * Redundancy analysis of cached keys or values (Sec. 1, the figures that show the cosine similarity
 * of keys inside one head, and the average similarity of keys and of values per layer and head;
 * Sec. 3.3, Eq. 3-4 for the similarity matrix and its off-diagonal mean).  For every (batch item,
 * head) of every layer, with R the N x N matrix of cosine similarities between the rows of X
 * (a row of norm below 1e-30 counts as the zero vector):
 *   redundancy  the mean of the off-diagonal entries of R (for X = K this is the r of mixkv_score);
 *   block_map   [nb, nb], nb = ceil(N / block): the mean of R over the rows of block a and the
 *               columns of block b, blocks being `block` consecutive positions (the last one may be
 *               shorter; diagonal entries belong to the diagonal blocks): the heat-map of R at a
 *               resolution of `block` tokens.
 * Only dtype, batch, n_kv_heads (the number of heads of X), head_dim and seq_len of `params` are
 * used; the rest must merely be valid.  1 <= block <= N.  Either output may be NULL, not both.
 * Workspace: mixkv_similarity_workspace_size bytes, 256-byte aligned, no initialisation.
 */
typedef struct {
  const void *X;             /* DEVICE [batch, n_kv_heads, N, D], D contiguous: keys or values */
  int64_t stride_b, stride_h, stride_n;   /* in elements; stride_n >= D; row starts 16-byte aligned */
} mixkv_rows_in;
typedef struct {
  float *redundancy;         /* DEVICE [batch, n_kv_heads] */
  float *block_map;          /* DEVICE [batch, n_kv_heads, nb, nb] */
} mixkv_similarity_out;
mixkv_status mixkv_similarity_workspace_size(const mixkv_params *params, int32_t n_layers, int32_t block, size_t *bytes);
mixkv_status mixkv_similarity(const mixkv_params *params, const mixkv_rows_in *in, const mixkv_similarity_out *out,
                              int32_t n_layers, int32_t block, void *workspace, size_t workspace_bytes,
                              void *hip_stream);

/*
 * Attention of one new token over the compacted cache (Sec. 3.1: the compressed K, V are what the
 * attention of the decoding phase reads).  Per layer, batch item and query head g (KV head
 * h = g / G): out_g = sum_j softmax_j(softmax_scale * Q_g . k_j) v_j over the rows of head h: the
 * counts[b][h] kept rows in K_cache / V_cache, laid out as mixkv_compress wrote them for
 * params->budget_mode and params->budget (fixed: [batch, n_kv_heads, B, D]; otherwise packed
 * [batch, n_kv_heads * B, D] with `offsets`), followed by the first tail_len rows of K_tail / V_tail
 * ([batch, n_kv_heads, tail_capacity, D]: the rows appended since the compression, the new token's
 * own row included; the caller's projection kernel writes them there).  fp32 accumulation; `out` has
 * the dtype of the inputs (bf16: rounded to nearest even).  All pointers are DEVICE pointers, rows
 * 16-byte aligned; K_tail / V_tail may be NULL when tail_len is 0, offsets when the layout is fixed.
 * counts / offsets are clamped to the capacity of the layout before use.
 * Workspace: long caches (more than 384 rows per head at params->budget + tail_len) are split over
 * several workgroups per head whose partial results pass through `workspace`:
 * mixkv_decode_workspace_size bytes (0 for short caches, then NULL is accepted), 256-byte aligned,
 * no initialisation.
 */
typedef struct {
  const void *K_cache, *V_cache;
  const int32_t *counts;     /* [batch, n_kv_heads] */
  const int32_t *offsets;    /* [batch, n_kv_heads + 1], packed layouts */
  const void *K_tail, *V_tail;
  const void *Q;             /* [batch, n_q_heads, D] the new token's queries */
  void *out;                 /* [batch, n_q_heads, D] */
} mixkv_decode_layer;
mixkv_status mixkv_decode_workspace_size(const mixkv_params *params, int32_t n_layers, int32_t tail_len, size_t *bytes);
mixkv_status mixkv_decode_attention(const mixkv_params *params, const mixkv_decode_layer *layers, int32_t n_layers,
                                    int32_t tail_len, int32_t tail_capacity, void *workspace, size_t workspace_bytes,
                                    void *hip_stream);

/*
 * Appends one token to the tails that mixkv_decode_attention reads (Sec. 3.1: the compressed cache
 * is what decoding continues on, so it grows again by one row per decoded token).  Per layer,
 * batch item b and KV head h: K_tail[b][h][position][:] = K_new[b][h][:], and the same for V:
 * verbatim copies in the dtype of params.  K_new / V_new are [batch, n_kv_heads, D] contiguous (the
 * new token's post-RoPE key and value rows), K_tail / V_tail [batch, n_kv_heads, tail_capacity, D]
 * contiguous; DEVICE pointers owned by the caller, 16-byte aligned; a tail may not overlap the new
 * rows.  0 <= position < tail_capacity, else MIXKV_ERR_INVALID_ARG (nothing is launched); the rows
 * before `position` are not touched.  After the call on the same stream,
 * mixkv_decode_attention with tail_len = position + 1 sees the new row.  No workspace.
 */
typedef struct {
  const void *K_new, *V_new;
  void *K_tail, *V_tail;
} mixkv_append_layer;
mixkv_status mixkv_append(const mixkv_params *params, const mixkv_append_layer *layers, int32_t n_layers,
                          int32_t position, int32_t tail_capacity, void *hip_stream);

const char *mixkv_status_string(mixkv_status status);
int32_t mixkv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MIXKV_H */
