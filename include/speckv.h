/*
 * speckv.h - C ABI of the MI355X (gfx950) SpecKV hot path.
 *
 * SpecKV (Sec. 4.1, Alg. 1) decides which prompt KV pairs a long-context model keeps
 * after prefill: the queries of the last n_window prompt tokens and of n_lookahead
 * draft tokens attend to every prompt key; the attention probabilities (Sec. 3.1,
 * Eq. 1) are reduced over queries and over the query heads of each GQA group
 * (App. C.2), smoothed by local pooling with kernel k, and the best-scoring keys plus
 * the whole window are kept; K and V are then gathered into a compact cache.
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - All data pointers are DEVICE pointers owned by the caller unless a comment says
 *    HOST.  The library allocates no device memory and keeps no state between calls;
 *    scratch comes from the caller's workspace (size from *_workspace_bytes).  The one
 *    exception is speckv_compress_static, which uses a fixed array inside the library.
 *  - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default
 *    stream) and the call returns without synchronising.  Outputs are valid once the
 *    stream reaches that point.  Inputs are never modified.
 *  - The return value is the only error channel.  Arguments are validated on the host
 *    before anything is launched: a call that returns INVALID_ARG, UNSUPPORTED or WORKSPACE has
 *    launched nothing.  SPECKV_ERR_RUNTIME means the HIP runtime refused a launch; kernels of
 *    the same call that were enqueued before it still run, and the outputs are undefined.
 *  - Element strides are in ELEMENTS of `dtype`; the head dimension is contiguous and
 *    every row (d elements) must start on a 16-byte boundary.
 *  - Readings of the paper fixed by this library: by default the reduction over queries and
 *    group is a SUM and pooling is MAX pooling (stride 1, same length, clipped to the
 *    non-window candidates [0, m), m = n_in - n_window); reduce_op / pool_op select the
 *    listing's max reduction and average pooling; `c_max` counts NON-window keys, so
 *    n_keep = min(c_max, m) + n_window rows are kept (pass C_max - n_window to get the
 *    paper's total budget); ties go to the smaller index; indices come out ascending.
 *
 * Layouts (S = n_seqs, L = n_layers, R = n_window + n_lookahead, T = total tokens)
 * ---------------------------------------------------------------------------------
 *  q       element (l, s, i, h, c) at l*q_stride_layer + s*q_stride_seq + i*q_stride_row
 *          + h*q_stride_head + c.  Rows 0..n_window-1 are the queries of prompt
 *          positions m..n_in-1 (causally masked), rows n_window..R-1 the lookahead
 *          queries (they see the whole prompt).            (Alg. 1: Q from [X_{m:}; Y])
 *  k, v    element (l, t, g, c) at l*kv_stride_layer + t*kv_stride_token
 *          + g*kv_stride_head + c, t = cu_seqlens[s] + j the packed token index.
 *  scores  (raw / pooled) fp32, per layer T*H_kv values: sequence s starts at
 *          H_kv*cu_seqlens[s] and holds [H_kv][n_in_s]; layer stride H_kv*T.
 *          pooled[j] is defined for j < m; entries j >= m are written as 0.
 *  idx     int32, per layer H_kv*KT values (KT = sum over s of n_keep_s): sequence s
 *          starts at H_kv*ck[s] (ck = prefix sums of n_keep_s) and holds
 *          [H_kv][n_keep_s] sequence-local token indices, ascending, window last.
 *  k_out,  same as idx with d contiguous elements per entry:
 *  v_out   [L][S packed][H_kv][n_keep_s][d].
 */
#ifndef SPECKV_H
#define SPECKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SPECKV_OK = 0,
  SPECKV_ERR_INVALID_ARG = -1, /* null pointer, bad dimension, misaligned pointer/stride    */
  SPECKV_ERR_UNSUPPORTED = -2, /* valid request outside what the kernels are built for      */
  SPECKV_ERR_WORKSPACE = -3,   /* workspace missing, misaligned or smaller than required    */
  SPECKV_ERR_RUNTIME = -4      /* the HIP runtime refused a launch                          */
} speckv_status;

/* Number type of q, k and v.  Products are exact in fp32 for all three; accumulation, softmax and
 * scores are fp32 (the paper does not fix a precision). */
typedef enum { SPECKV_BF16 = 0, SPECKV_F32 = 1, SPECKV_F16 = 2 } speckv_dtype;

/* Reduction over the observation rows of one query head (Alg. 1 reduce step).  SUM is Eq. 1's
 * mean times a constant; MAX is the listing's MaxReduce (hyper-parameter table "Reduction =
 * Max").  Either way the per-head results of a GQA group are added (App. C.2 averages them). */
typedef enum { SPECKV_REDUCE_SUM = 0, SPECKV_REDUCE_MAX = 1 } speckv_reduce_op;

/* Local pooling with kernel pool_k (Alg. 1 pooling step).  The window of key j is
 * j - pool_k/2 .. j + (pool_k-1)/2 (integer division): symmetric for odd kernels; an even kernel
 * (hyper-parameter table, SpecPC column: 64 / 32) reaches one position further back than ahead,
 * which is the usual library call with padding pool_k/2 keeping the first m outputs.
 * MAX: neighbourhood clipped to the candidates [0, m) (hyper-parameter table).  AVG: mean over the
 * pool_k positions with zeros outside [0, m), i.e. the divisor is always pool_k (the listing's
 * AvgPool1D with the usual library padding convention). */
typedef enum { SPECKV_POOL_MAX = 0, SPECKV_POOL_AVG = 1 } speckv_pool_op;

/* Limits (a request beyond them returns SPECKV_ERR_UNSUPPORTED):
 *  - sequences per call: the per-sequence tables travel to the kernels by value in the kernel
 *    argument block, which bounds their length; batch larger sets over several calls;
 *  - observation rows of one KV group, (n_q_heads / n_kv_heads) * R: bounds the row-statistics
 *    workspace per key chunk;
 *  - n_layers * n_kv_heads * (row super-blocks per group) <= 2^24 and total tokens <= 2^30. */
#define SPECKV_MAX_SEQS 128
#define SPECKV_MAX_GROUP_ROWS 4096
#define SPECKV_MAX_POOL_K 255

/* Problem statement of Alg. 1 (sequence lengths, n_lookahead, C_max, n_window, k) plus
 * the tensor geometry.  Plain data, read during the call only. */
typedef struct {
  int32_t n_seqs;      /* 1..SPECKV_MAX_SEQS                                                 */
  int32_t n_layers;    /* >= 1                                                               */
  int32_t n_q_heads;   /* multiple of n_kv_heads; query head h uses KV head h / group        */
  int32_t n_kv_heads;
  int32_t head_dim;    /* 64 or 128                                                          */
  int32_t n_window;    /* >= 0; every sequence needs n_in >= max(1, n_window)                */
  int32_t n_lookahead; /* >= 0; n_window + n_lookahead >= 1                                  */
  int32_t pool_k;      /* 1..SPECKV_MAX_POOL_K; window j - k/2 .. j + (k-1)/2                */
  int32_t c_max;       /* >= 0: non-window keys kept per KV head (clamped to m)              */
  float sm_scale;      /* > 0, multiplies q.k (1/sqrt(d), or 1 if folded into q)             */
  int32_t dtype;       /* speckv_dtype of q, k, v                                            */
  const int32_t *cu_seqlens; /* HOST, n_seqs+1 non-decreasing token prefix sums starting at 0;
                                NULL means one sequence of n_in tokens                       */
  int64_t n_in;        /* used only when cu_seqlens == NULL                                  */
  int64_t q_stride_layer, q_stride_seq, q_stride_row, q_stride_head;
  int64_t kv_stride_layer, kv_stride_token, kv_stride_head;
  int32_t reduce_op;   /* speckv_reduce_op; 0 (SUM) is the default                           */
  int32_t pool_op;     /* speckv_pool_op; 0 (MAX) is the default                             */
  const int32_t *n_in_dev; /* DEVICE, optional (NULL: unused).  One int32 holding the number of
                          prompt tokens that really exist, read by the kernels when they run; it
                          lets a call follow another that produced the count on the device (the
                          cascade of Sec. 4.3: prompt compression, then cache compression) without
                          a host round trip and inside one HIP graph.  Needs n_seqs == 1.  The
                          host length (n_in / cu_seqlens) is then an UPPER BOUND that sizes grids,
                          workspace, row strides and output shapes; values outside
                          [max(1, n_window), host length] are clamped.  With a live length n',
                          m' = n' - n_window: scores at j >= n' are written as 0, idx holds
                          min(c_max, m') candidates, the window m'..n'-1 and then -1 up to the
                          host-sized row; compaction writes zero rows for the -1 entries.
                          With per-head budgets head_off[Hkv] = Hkv * (min(c_max, m') + n_window)
                          and the rows behind it hold -1 / zeros.
                          Supported by speckv_score(_lse), speckv_select(_ada), speckv_compact(_ada)
                          and speckv_compress(_lse, _events, _static, _ada); the prompt-token entry
                          points (specpc_*) return SPECKV_ERR_UNSUPPORTED. */
} speckv_params;

/* Human-readable name of a status code (static storage). */
const char *speckv_status_string(speckv_status status);

/* Rows of the compacted cache of sequence `seq`: min(c_max, n_in_s - n_window) + n_window
 * (Alg. 1 "Select KVs": top-k plus the window).  Returns -1 on invalid arguments. */
int64_t speckv_n_keep(const speckv_params *p, int32_t seq);

/* Sum of speckv_n_keep over all sequences (KT in the layouts above); -1 if invalid. */
int64_t speckv_total_keep(const speckv_params *p);

/* Bytes of 256-byte-aligned device workspace that speckv_score, speckv_select and
 * speckv_compress need for these parameters (the maximum over the three).  Returns 0 if
 * the parameters are invalid. */
size_t speckv_workspace_bytes(const speckv_params *p);

/* Launch plan the host derives for these parameters, for diagnostics and tests (no GPU needed):
 * info[0] waves per scoring workgroup, [1] 32-row blocks per wave, [2] row super-blocks per KV group,
 * [3] keys per chunk of the scoring sweeps, [4] unmasked chunks over all sequences, [5] keys per LDS
 * tile, [6] parts a row is split into for selection (1: one workgroup per row), [7] keys per such
 * part, [8] kernels of the unmasked scoring sweeps: bit 0 set when the row-statistics sweep, bit 1
 * when the column-reduction sweep keeps the query rows stationary in LDS (clear: key tiles streamed
 * through LDS), [9] 1 for max reduction, [10] 1 when the key-tile row-statistics sweep sums
 * against fixed reference exponents and is followed by a repair launch (sweeps of several rounds of
 * workgroups), 0 when it takes the online maximum step on every key block.  Returns SPECKV_OK or
 * the reason the parameters are rejected. */
#define SPECKV_PLAN_INFO_WORDS 11
speckv_status speckv_plan_info(const speckv_params *p, int64_t info[SPECKV_PLAN_INFO_WORDS]);

/* Importance scores (Eq. 1; Alg. 1 CrossAttention, reduce and pooling steps).
 * For every (layer, sequence, KV head): softmax over the visible prompt keys of
 * sm_scale*q.k for each observation row of each query head of the group, summed over
 * rows and heads into raw[j] (all n_in keys), then max-pooled with kernel pool_k over
 * the candidates j < m into pooled[j].  `raw` may be NULL.  Layout: "scores" above. */
speckv_status speckv_score(const speckv_params *p, const void *q, const void *k,
                           float *pooled, float *raw, void *workspace,
                           size_t workspace_bytes, void *stream);

/* speckv_score with row normalisers supplied by the caller: ONE sweep over K instead of two.
 * lse_in (fp32, contiguous [L][S][R][n_q_heads]) is the natural-log sum over keys of
 * exp(sm_scale*q.k) per observation row, for example the log-sum-exp the prefill attention
 * kernel already produced for these rows (that one also counts the draft keys a lookahead row
 * attends to, so the probabilities are those of the real forward pass rather than renormalised
 * over the prompt: Alg. 1's attention matrix A taken from the forward pass).  With lse_in equal
 * to the row log-sum-exp over the visible prompt keys the result equals speckv_score's. */
speckv_status speckv_score_lse(const speckv_params *p, const void *q, const void *k,
                               const float *lse_in, float *pooled, float *raw, void *workspace,
                               size_t workspace_bytes, void *stream);

/* Selection (Alg. 1 "Select KVs"; Fig. 2: window always retained).  For every (layer,
 * sequence, KV head) writes the min(c_max, m) candidates with the largest pooled score
 * (equal scores: smaller index first), in ascending order, followed by m..n_in-1.
 * `pooled` must not contain NaN.  Layout: "idx" above.  The workspace is optional: with NULL every
 * row is ranked by one workgroup; with a 256-byte-aligned workspace of at least
 * speckv_select_workspace_bytes (a few MiB; 0 when the call would not use it), calls with few
 * and very long rows spread each row over several workgroups (same result). */
size_t speckv_select_workspace_bytes(const speckv_params *p);
speckv_status speckv_select(const speckv_params *p, const float *pooled, int32_t *idx,
                            void *workspace, size_t workspace_bytes, void *stream);

/* Compaction (Alg. 1 last step: cache <- K[i_cache], V[i_cache]).  Bit copy of the rows
 * named by idx into k_out / v_out.  `v` and `v_out` may both be NULL (keys only).  An
 * index outside [0, n_in_s) yields a zero row instead of a read.  Needs no workspace. */
speckv_status speckv_compact(const speckv_params *p, const void *k, const void *v,
                             const int32_t *idx, void *k_out, void *v_out, void *stream);

/* Fused path: score, select and compact in one call on one stream (Alg. 1 loop body for
 * every layer, head and sequence).  Pooled scores live in the workspace. */
speckv_status speckv_compress(const speckv_params *p, const void *q, const void *k,
                              const void *v, int32_t *idx, void *k_out, void *v_out,
                              void *workspace, size_t workspace_bytes, void *stream);

/* speckv_compress for callers that cannot allocate or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels and bit-identical
 * results; the scratch is a fixed array of SPECKV_STATIC_SCRATCH_BYTES inside the library's device
 * code (one copy per GPU, held until the process ends; its address is looked up on the first call
 * on each device).  The call allocates nothing and frees nothing.  Parameters whose
 * speckv_workspace_bytes exceeds SPECKV_STATIC_SCRATCH_BYTES are rejected with
 * SPECKV_ERR_WORKSPACE before anything is launched (32 MiB covers one layer of 8 KV heads at
 * 256K tokens, or a few layers of shorter prompts).  Every call on a GPU shares that GPU's array:
 * calls that overlap on one GPU (two streams, two threads) race and must be serialised by the
 * caller.  The array keeps the previous call's contents; the kernels never read what they have
 * not written in the same call, and the counters that must start at zero are zeroed by a kernel of
 * the same call (no memset). */
#define SPECKV_STATIC_SCRATCH_BYTES (32u << 20)
speckv_status speckv_compress_static(const speckv_params *p, const void *q, const void *k,
                                     const void *v, int32_t *idx, void *k_out, void *v_out,
                                     void *stream);

/* speckv_compress with caller-supplied row normalisers (see speckv_score_lse). */
speckv_status speckv_compress_lse(const speckv_params *p, const void *q, const void *k,
                                  const void *v, const float *lse_in, int32_t *idx, void *k_out,
                                  void *v_out, void *workspace, size_t workspace_bytes, void *stream);

/* speckv_compress with per-stage timing marks, for benchmarks and profilers.  `events` is a
 * HOST array of SPECKV_N_STAGE_EVENTS hipEvent_t handles created by the caller; the call
 * records them on `stream` around its kernels and does not synchronise:
 *   [0] start  [1] after scoring pass 1 (row statistics)  [2] after the row-statistics merge
 *   [3] after scoring pass 2 (column sums)  [4] after pooling  [5] after selection
 *   [6] after compaction.  Same results as speckv_compress (Alg. 1 loop body). */
#define SPECKV_N_STAGE_EVENTS 7
speckv_status speckv_compress_events(const speckv_params *p, const void *q, const void *k,
                                     const void *v, int32_t *idx, void *k_out, void *v_out,
                                     void *workspace, size_t workspace_bytes, void *stream,
                                     void **events, int32_t n_events);

/* Per-head budgets (App. "Integration and Comparison with the AdaKV Baseline": a different
 * budget per attention head, applied to SpecKV).  The paper gives no formula; the rule here is:
 * per (layer, sequence), with C = min(c_max, m) and f = min(c_floor, C), every KV head keeps
 * its own f best candidates, and the remaining Hkv*(C - f) slots go to the best remaining
 * candidates of the whole layer whatever their head (equal scores: smaller head, then smaller
 * index).  A layer keeps Hkv*C non-window keys, as with equal budgets, so idx, k_out and v_out
 * have the sizes of the equal-budget calls; only the split between heads moves.
 *   head_off  int32 device, [n_layers][n_seqs][n_kv_heads + 1]: row offsets of the heads inside
 *             their (layer, sequence) block; head g owns rows head_off[g] .. head_off[g+1]-1,
 *             its kept candidates ascending followed by the window; head_off[Hkv] = Hkv*n_keep_s.
 *   idx       per layer: sequence s starts at Hkv*KT_before(s) as in the "idx" layout; inside
 *             the block the heads follow each other at head_off.
 *   k_out / v_out  rows in the same order as idx, each d elements.
 * c_floor >= c_max gives exactly speckv_select's result.  Needs n_kv_heads <=
 * SPECKV_MAX_ADA_HEADS and a workspace of speckv_ada_workspace_bytes (0 if the parameters are
 * invalid), which covers all three calls.  `pooled` must not hold NaN. */
#define SPECKV_MAX_ADA_HEADS 128
size_t speckv_ada_workspace_bytes(const speckv_params *p);
speckv_status speckv_select_ada(const speckv_params *p, int32_t c_floor, const float *pooled,
                                int32_t *idx, int32_t *head_off, void *workspace,
                                size_t workspace_bytes, void *stream);
speckv_status speckv_compact_ada(const speckv_params *p, const void *k, const void *v,
                                 const int32_t *idx, const int32_t *head_off, void *k_out,
                                 void *v_out, void *stream);
/* score -> shared-budget selection -> compaction in one call (see speckv_compress). */
speckv_status speckv_compress_ada(const speckv_params *p, int32_t c_floor, const void *q,
                                  const void *k, const void *v, int32_t *idx, int32_t *head_off,
                                  void *k_out, void *v_out, void *workspace,
                                  size_t workspace_bytes, void *stream);

/* Prompt-token selection from draft-model attention (Sec. 4.2 / Alg. 2, in the reduced
 * form: sum instead of max aggregation, no row weights, no skipped layers).  Needs
 * n_seqs == 1.  score[j] = attention probability summed over all layers, heads and
 * observation rows; max-pooled with pool_k over j < m; the top_k best candidates are
 * each widened to [t - n_neighbor, t + n_neighbor] (clipped to the prompt), united with
 * the window m..n_in-1 and emitted ascending without duplicates into idx_out
 * (capacity n_in), with ids_out[r] = token_ids[idx_out[r]] and *count_out (device int32)
 * the number of entries.  p->c_max, p->reduce_op and p->pool_op are ignored (the reduced form
 * is a sum with max pooling; invalid values of the two ops are still rejected). */
size_t specpc_workspace_bytes(const speckv_params *p, int32_t top_k);
speckv_status specpc_select_tokens(const speckv_params *p, int32_t top_k, int32_t n_neighbor,
                                   const void *q, const void *k, const int32_t *token_ids,
                                   int32_t *idx_out, int32_t *ids_out, int32_t *count_out,
                                   void *workspace, size_t workspace_bytes, void *stream);

/* specpc_select_tokens with per-stage timing marks (see speckv_compress_events): [0] start
 * [1] after scoring pass 1  [2] after the row-statistics merge  [3] after scoring pass 2
 * [4] after the cross-layer reduction and pooling  [5] after the top-k selection  [6] after the
 * neighbour expansion and id gather.  Same results as specpc_select_tokens (Alg. 2, reduced). */
speckv_status specpc_select_tokens_events(const speckv_params *p, int32_t top_k, int32_t n_neighbor,
                                          const void *q, const void *k, const int32_t *token_ids,
                                          int32_t *idx_out, int32_t *ids_out, int32_t *count_out,
                                          void *workspace, size_t workspace_bytes, void *stream,
                                          void **events, int32_t n_events);

/* Prompt compression as printed in Sec. 4.2 / Alg. 2.  Needs n_seqs == 1.  q holds the draft
 * model's queries of the n_window last prompt rows followed by the lookahead rows, k its prompt
 * keys, for every layer.  Layers below l_skip are ignored; window row j (1-based) is weighted
 * j / n_window; the weighted attention probabilities are max-reduced over layers, heads and
 * rows into one score per prompt token; AvgPool1D(p->pool_k) then MaxPool1D(n_neighbor) over
 * the non-window tokens (windows as for speckv_pool_op, odd or even kernels up to
 * SPECKV_MAX_POOL_K; zero padding for the mean, clipping for the max);
 * the c_max best tokens (p->c_max) and the window are emitted ascending into idx_out
 * (capacity min(c_max, m) + n_window) with ids_out[r] = token_ids[idx_out[r]] and *count_out
 * their number.  p->reduce_op / pool_op are ignored. */
size_t specpc_compress_workspace_bytes(const speckv_params *p, int32_t l_skip);
speckv_status specpc_compress_prompt(const speckv_params *p, int32_t l_skip, int32_t n_neighbor,
                                     const void *q, const void *k, const int32_t *token_ids,
                                     int32_t *idx_out, int32_t *ids_out, int32_t *count_out,
                                     void *workspace, size_t workspace_bytes, void *stream);

/* Diagnostics: what this GPU sustains for the instruction mix of the scoring sweeps (Sec. 3.1
 * Eq. 1 on MFMA score tiles) when nothing has to be fetched.  Launches one register-resident loop
 * on `stream`: kind 0 = the bf16 MFMAs of 32x32 score tiles at d = 128 alone, 1 = with the softmax
 * arithmetic of a tile (16 x (fma, exp2, add) per lane), 2 = as 1 with the B operands re-read from
 * LDS (512 bytes per MFMA).  `operands` (device, 16-byte aligned, at least 64 KiB, read only)
 * supplies the bf16 operand bits: random values and zeros draw very different power.  `out`
 * (device, 512 KiB) receives one float per thread.  *flops (HOST) gets the matrix flops the
 * launch executes; the caller times it.  Not part of the product path. */
speckv_status speckv_probe_ceiling(int32_t kind, int32_t iters, const void *operands, void *out,
                                   void *stream, int64_t *flops);

#ifdef __cplusplus
}
#endif
#endif /* SPECKV_H */
