/*
 * jq.h -- C ABI of the Judge Q KV-cache eviction hot path for AMD MI355X (gfx950).
 *
 * At the end of prefill the method (paper Section 4.3, the inference-time use of
 * the trained soft tokens) scores every prompt key by the attention it receives
 * from the appended soft-token queries (Eq. 3), keeps the key-value pairs with
 * the top-k scores and decodes on the pruned cache.  This library is that path,
 * per layer and per KV head, as HIP kernels:
 *
 *   jq_score        attention map of the soft tokens over the prompt (Eq. 3)
 *   jq_pool         1-D average pooling of the map (the pooling settings that
 *                   Section 5.1, Baselines, shares with the compared methods)
 *   jq_select_topk  top-B retention per KV head (Section 4.3)
 *   jq_compact      gather of the kept K/V rows into a dense pruned cache
 *   jq_compact_inplace  the same, written over the front of K and V themselves
 *   jq_evict        all of the above for n_layers x n_seq problems in one call
 *   jq_evict_inplace  the same, the pruned cache written over the front of K and V themselves
 *   jq_evict_stream   the same step during decoding: re-evicts a pruned cache, carries the rows' positions along
 *   jq_score_lse, jq_evict_lse    the same with caller-supplied softmax normalisers
 *   jq_score_tail, jq_evict_tail  the same with the soft tokens' own keys in the softmax
 *   jq_score_paged, jq_evict_paged  the same on a paged cache (pools + block table)
 *   jq_hit_rate     critical-KV hit rate between two kept sets (Eq. 6)
 *   jq_map_mse      forward value of the training objective (Eq. 5) from two score maps
 *   jq_map_mse_fused  the same from the two query sets, the second map never stored
 *
 * Conventions common to every entry point
 * ---------------------------------------
 * - Pointers named Q, K, V, scores, pooled, idx, K_out, V_out, ws are DEVICE
 *   pointers on the current HIP device.  `shape`, `shape->cu_seqlens`,
 *   `shape->budgets` and `bytes` are HOST pointers, read before the call
 *   returns (they may be freed afterwards).
 * - bf16 tensors are raw 16-bit patterns.  All tensors are dense, row-major:
 *     Q       [n_layers, n_seq, n_q, h_q, d]   bf16  soft-token queries
 *     K, V    [n_layers, T, h_kv, d]           bf16  prompt keys / values,
 *                                                     T = cu_seqlens[n_seq]
 *     scores  [n_layers, h_kv, T]              fp32  (unpooled or pooled)
 *     idx     [n_layers, h_kv, TB]             int32 kept positions, local to
 *                                                     their sequence, ascending
 *                                                     inside each (layer, head,
 *                                                     sequence) segment;
 *                                                     TB = sum of budgets
 *     K_out,  [n_layers, TB, h_kv, d]          bf16  pruned cache; sequence s
 *     V_out                                           owns rows cu_budgets[s]..
 * - Query head h reads KV head h / (h_q / h_kv).  The softmax runs over the L_s
 *   prompt keys of the query's own sequence only; probabilities are summed (not
 *   averaged) over the n_q soft tokens and the h_q/h_kv heads of the group, so
 *   the unpooled scores of a (layer, sequence, KV head) sum to n_q * h_q / h_kv.
 * - The caller owns every buffer.  The library allocates nothing, keeps no
 *   state between calls (apart from the knobs below, read once, and a one-time
 *   per-device raise of one kernel's LDS limit), never synchronises the stream
 *   and may be called from several host threads at once.  `stream` is a hipStream_t passed as void*
 *   (NULL = the default stream).  Work is only enqueued; results are ready when
 *   the stream reaches the end of the enqueued work.
 * - Every entry point returns a jq_status.  All argument errors are detected
 *   on the host before anything is launched; nothing is written in that case.
 *   After JQ_ERR_LAUNCH the contents of the outputs are unspecified.
 * - NaN or infinite inputs are not checked; results are then unspecified.
 */
#ifndef JQ_H_
#define JQ_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum jq_status {
    JQ_OK = 0,
    JQ_ERR_NULL = -1,        /* a required pointer is NULL                               */
    JQ_ERR_SHAPE = -2,       /* a dimension, pool_k, scale or cu_seqlens is malformed    */
    JQ_ERR_BUDGET = -3,      /* some budget is outside 1..L_s, or below keep_first+keep_last */
    JQ_ERR_UNSUPPORTED = -4, /* valid but not implemented: d != 128, more than JQ_MAX_SEQ  */
                             /* sequences, more than 65535 layers or 256 KV heads, more    */
                             /* than 2^20 query rows per KV head, a sequence (or a layer's */
                             /* page pool) with 4 GiB or more of keys, 2^31 or more kept   */
                             /* rows or workgroups in one call, a misaligned tensor        */
    JQ_ERR_WORKSPACE = -5,   /* workspace missing, misaligned (16 B) or too small        */
    JQ_ERR_ALIAS = -6,       /* an output overlaps an input or another output            */
    JQ_ERR_LAUNCH = -7       /* the HIP runtime refused a launch                         */
} jq_status;

#define JQ_MAX_SEQ 128 /* most sequences one call may carry */

/* Problem description (host memory).  One call handles n_layers * n_seq
 * independent (layer, sequence) problems that share every other dimension. */
typedef struct jq_shape {
    int32_t n_layers;          /* 1..65535                                                    */
    int32_t n_seq;             /* 1..JQ_MAX_SEQ                                               */
    int32_t n_q;               /* soft tokens per sequence (the paper's n; 32 in its runs)    */
    int32_t h_q;               /* query heads                                                 */
    int32_t h_kv;              /* KV heads; h_q % h_kv == 0; at most 256                      */
    int32_t d;                 /* head dimension; only 128 is implemented                     */
    int32_t pool_k;            /* odd >= 1; 1 = no pooling                                    */
    float scale;               /* logit scale; 0 selects 1/sqrt(d); must be finite and >= 0   */
    const int32_t* cu_seqlens; /* HOST [n_seq+1]; cu[0] = 0, strictly increasing; one sequence's  */
                               /* keys (L_s * h_kv * d * 2 bytes) must stay below 4 GiB           */
    const int32_t* budgets;    /* HOST [n_seq]; 1 <= budgets[s] <= L_s.  May be NULL for      */
                               /* jq_score and jq_pool, which do not use it.                  */
    int32_t keep_first;        /* >= 0: the first keep_first and the last keep_last positions  */
    int32_t keep_last;         /* of every sequence are kept whatever they score (the sinks    */
                               /* and the local window of the Section 5.1 baselines); they     */
                               /* count towards the budget: keep_first + keep_last <=          */
                               /* budgets[s].  Read by jq_select_topk and jq_evict* only.      */
    int32_t window;            /* 0: the queries are soft tokens appended after the prompt (the */
                               /* paper's method).  1: the queries are the prompt's OWN last    */
                               /* n_q tokens (the observation window of the window-query        */
                               /* baselines of Section 5.1): K holds their keys as the last n_q */
                               /* rows of every sequence (n_q <= L_s), query i attends to       */
                               /* positions 0 .. L_s - n_q + i only (causal), the window's own  */
                               /* positions score 0 and are always kept (keep_last counts as    */
                               /* at least n_q).  Not with jq_score_tail / jq_evict_tail.       */
    const int32_t* layer_budgets; /* NULL, or DEVICE int32 [n_layers, n_seq]: budgets that differ from */
                               /* layer to layer in one call (the depth-dependent allocation of the   */
                               /* PyramidKV baseline, Section 5.1).  `budgets` then gives each          */
                               /* sequence's LARGEST budget and with it the layout of idx / K_out /     */
                               /* V_out; layer l keeps layer_budgets[l, s] positions of sequence s and  */
                               /* writes only the first that many slots of the sequence's segment (the  */
                               /* rest is left untouched).  Read on the device only, so it cannot be    */
                               /* validated: a value outside max(1, keep_first + keep_last) ..           */
                               /* budgets[s] is clamped into that range (the always-kept positions are   */
                               /* kept in every layer; keep_last counts as at least n_q in window mode). */
                               /* Used by jq_select_topk, jq_compact, jq_compact_inplace and jq_evict*.  */
} jq_shape;

/* Bytes of device workspace that jq_score, jq_select_topk and jq_evict need for
 * this shape (one size serves all three; 256-byte granular).  With `budgets` NULL
 * the size only serves jq_score. */
int jq_workspace_bytes(const jq_shape* shape, size_t* bytes);

/* Unpooled importance scores (Eq. 3 without the 1/n):
 *   scores[l,g,t] = sum_{h in group g} sum_i softmax_j(scale * Q[l,s,i,h,:].K[l,j,g,:])[t]
 * for every token t of every sequence s.  Two passes over K (softmax statistics,
 * then normalised probabilities).  Uses `ws` as scratch. */
int jq_score(const jq_shape* shape, const void* Q, const void* K, float* scores,
             void* ws, size_t ws_bytes, void* stream);

/* The same scores as a slice of a wider softmax, in ONE pass over K.  In the model's
 * own prefill (Eq. 1: the soft tokens are concatenated after the prompt) soft token i
 * also attends to the soft tokens up to itself, so the normaliser of its attention row
 * covers more than the prompt keys; attention kernels keep it as a log-sum-exp.  Given
 *   lse[l,s,i,h] = log sum_{j in the row's key domain} exp(scale * Q[l,s,i,h,:].K_j)
 * (DEVICE, fp32, natural log, [n_layers, n_seq, n_q, h_q]) this computes
 *   scores[l,g,t] = sum_{h in group g} sum_i exp(scale * Q[l,s,i,h,:].K[l,t,g,:] - lse[l,s,i,h]).
 * With lse taken over the prompt keys alone the result equals jq_score. */
int jq_score_lse(const jq_shape* shape, const void* Q, const void* K, const float* lse,
                 float* scores, void* ws, size_t ws_bytes, void* stream);

/* The scores with the soft tokens' own keys in the softmax (Section 4.2: the soft tokens
 * are appended to the prompt, so in a causal model soft token i attends to the prompt
 * and to soft tokens 0..i, itself included).  K_tail (DEVICE, bf16,
 * [n_layers, n_seq, n_q, h_kv, d]) holds those keys:
 *   Z[l,s,i,h]    = sum_{j in sequence s} exp(scale * Q[l,s,i,h,:].K[l,j,g,:])
 *                 + sum_{i' <= i} exp(scale * Q[l,s,i,h,:].K_tail[l,s,i',g,:])
 *   scores[l,g,t] = sum_{h in group g} sum_i exp(scale * Q[l,s,i,h,:].K[l,t,g,:]) / Z[l,s,i,h].
 * Two passes over K like jq_score; the tail only enters the normalisers.  The same call
 * scores a prompt under its own last n_q tokens (the observation window of the
 * SnapKV-style baselines of Section 5.1): pass the prompt without the window as K and
 * the window's queries and keys as Q and K_tail. */
int jq_score_tail(const jq_shape* shape, const void* Q, const void* K, const void* K_tail, float* scores,
                  void* ws, size_t ws_bytes, void* stream);

/* Pooling of the attention map before the selection (Section 5.1, Baselines: the method runs with the
 * local-window and pooling settings of the compared methods; the paper gives no operator, this library reads
 * it as a 1-D average with zero padding):
 * pooled[l,g,t] = (1/pool_k) * sum_{|u| <= (pool_k-1)/2} scores[l,g,t+u], taking
 * zero for positions outside t's own sequence (divisor is always pool_k).
 * `pooled` must not overlap `scores`. */
int jq_pool(const jq_shape* shape, const float* scores, float* pooled, void* stream);

/* Top-k retention (Section 4.3: the key-value pairs with the highest scores stay, the rest is discarded).
 * For every (layer, sequence, KV head): the budgets[s] positions with the largest
 * pooled value; equal values are resolved towards the lower position; positions
 * are written in ascending order.  Exact for any finite fp32 input (-0 == +0).
 * The first keep_first and last keep_last positions of a sequence are always among
 * them (their values are ignored); the remaining places go to the largest values
 * of the other positions.  Uses `ws` as scratch. */
int jq_select_topk(const jq_shape* shape, const float* pooled, int32_t* idx,
                   void* ws, size_t ws_bytes, void* stream);

/* The pruned cache that decoding continues on (Section 4.3), as a gather of the kept rows:
 * K_out[l, cu_budgets[s]+b, g, :] = K[l, cu_seqlens[s] + idx[l,g,cu_budgets[s]+b], g, :]
 * and the same for V, as 16-bit patterns.  An index outside 0..L_s-1 is clamped
 * into that range (never dereferenced out of bounds). */
int jq_compact(const jq_shape* shape, const void* K, const void* V, const int32_t* idx,
               void* K_out, void* V_out, void* stream);

/* The pruned cache written over the front of the cache it was taken from (Section 4.3: decoding
 * continues on the pruned cache, so a server can hand the rest of the memory back): after the call
 *   K[l, cu_budgets[s]+b, g, :] = (old) K[l, cu_seqlens[s] + idx[l,g,cu_budgets[s]+b], g, :]
 * for every kept row, likewise V; rows from sum(budgets) on are left as they were.  K and V keep
 * their [n_layers, T, h_kv, d] strides.  Kept rows whose source lies inside the overwritten front are
 * first copied to `ws` (DEVICE, 16-byte aligned, at least jq_compact_inplace_workspace_bytes), then
 * every row is written, so no order between workgroups is assumed.  Indices are clamped as in
 * jq_compact; idx must not overlap K, V or ws. */
int jq_compact_inplace_workspace_bytes(const jq_shape* shape, size_t* bytes);
int jq_compact_inplace(const jq_shape* shape, void* K, void* V, const int32_t* idx,
                       void* ws, size_t ws_bytes, void* stream);

/* Critical-KV hit rate (Eq. 6): for every (layer, sequence, KV head)
 *   rate[l,s,g] = |I_cur & I_ref| / |I_ref|
 * where I_cur = idx_cur[l, g, cu_budgets[s] .. cu_budgets[s+1]) holds shape->budgets[s]
 * positions and I_ref = idx_ref[l, g, ...] holds ref_budgets[s] positions (HOST array of
 * n_seq entries, each 1..L_s; NULL means the same budgets as `shape`).  Both lists must be
 * ascending, as jq_select_topk / jq_evict write them; idx_cur is [n_layers, h_kv, sum budgets],
 * idx_ref [n_layers, h_kv, sum ref_budgets], rate [n_layers, n_seq, h_kv] fp32 (DEVICE). */
int jq_hit_rate(const jq_shape* shape, const int32_t* idx_cur, const int32_t* idx_ref,
                const int32_t* ref_budgets, float* rate, void* stream);

/* Forward value of the training objective (Section 4.2, Eq. 3-5).  scores_a and scores_b are
 * jq_score outputs for the same prompt under two sets of query tokens (soft tokens and response
 * tokens); rows_a, rows_b are their numbers of summed probability rows per KV head
 * (tokens * h_q / h_kv), so that scores / rows is the attention map averaged over the tokens:
 *   mse[l,s,g] = (1 / L_s) * sum_t ( scores_a[l,g,t] / rows_a - scores_b[l,g,t] / rows_b )^2
 * over the tokens t of sequence s.  mse is [n_layers, n_seq, h_kv] fp32 (DEVICE).  Only
 * n_layers, n_seq, h_kv and cu_seqlens of `shape` matter here. */
int jq_map_mse(const jq_shape* shape, const float* scores_a, float rows_a, const float* scores_b, float rows_b,
               float* mse, void* stream);

/* The same value (Section 4.2: the maps of Eq. 3 and Eq. 4, the loss of Eq. 5) straight from the two query sets,
 * without handing the maps to the caller: Q_a [n_layers, n_seq, shape->n_q, h_q, d] are the soft tokens' queries,
 * Q_b [n_layers, n_seq, n_q_b, h_q, d] the response tokens' (any n_q_b >= 1; rows beyond 128 per KV head take
 * further passes over K), K the prompt's keys as in jq_score.  The soft tokens' map is computed first; the
 * launch that completes the response's map does not store it but accumulates
 *   ( map_a[t] / (n_q * G) - map_b[t] / (n_q_b * G) )^2,  G = h_q / h_kv,
 * per workgroup in fp64, and a last small launch adds the workgroups' sums in a fixed order:
 *   mse[l,s,g] as in jq_map_mse, [n_layers, n_seq, h_kv] fp32 (DEVICE).
 * Dense caches, prompt-only softmax (shape->window must be 0).  `ws` (DEVICE, 16-byte aligned) must hold
 * jq_map_mse_fused_workspace_bytes; nothing may overlap anything else. */
int jq_map_mse_fused_workspace_bytes(const jq_shape* shape, int32_t n_q_b, size_t* bytes);
int jq_map_mse_fused(const jq_shape* shape, const void* Q_a, const void* Q_b, int32_t n_q_b, const void* K, float* mse,
                     void* ws, size_t ws_bytes, void* stream);

/* The whole eviction step of Section 4.3 at the end of prefill (Eq. 3 scores -> pooling -> top-k retention ->
 * pruned cache) for n_layers x n_seq problems: score -> pool -> select -> compact in one call.  `idx_out` (kept positions) and
 * `scores_out` (POOLED scores) may each be NULL when the caller does not want
 * them; the workspace then holds them. */
int jq_evict(const jq_shape* shape, const void* Q, const void* K, const void* V,
             void* K_out, void* V_out, int32_t* idx_out, float* scores_out,
             void* ws, size_t ws_bytes, void* stream);

/* jq_evict for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same inputs, outputs and results as jq_evict, but no workspace argument: the
 * kernels' scratch memory is a fixed array of JQ_STATIC_WS_BYTES inside the library's device image (every GPU the
 * library runs on holds its own copy until the process ends).  The call allocates and frees nothing.  A shape
 * whose jq_workspace_bytes exceeds JQ_STATIC_WS_BYTES is rejected with JQ_ERR_WORKSPACE before any launch (the
 * 128K-token layer with 8 KV heads needs 16.6 MiB).  All calls on one GPU share that GPU's array, which keeps
 * the previous call's contents (the kernels clear what they need cleared): calls that overlap in time on one GPU
 * -- two streams, two host threads -- race on it and must be serialised by the caller. */
#define JQ_STATIC_WS_BYTES (32u << 20)
int jq_evict_static(const jq_shape* shape, const void* Q, const void* K, const void* V,
                    void* K_out, void* V_out, int32_t* idx_out, float* scores_out, void* stream);

/* The eviction step of Section 4.3 when no second cache may exist (decoding continues on the pruned cache, so a
 * server wants the rest of the memory back at once): after the call
 *   K[l, cu_budgets[s]+b, g, :] = (old) K[l, cu_seqlens[s] + idx[l,g,cu_budgets[s]+b], g, :]
 * for every kept row, likewise V -- the pruned cache lies at the front of every layer of K and V themselves,
 * rows from sum(budgets) on are left as they were, and K and V keep their [n_layers, T, h_kv, d] strides.
 * `lse` NULL: two passes over K as jq_evict; otherwise one pass with the supplied normalisers as jq_evict_lse.
 * The kernel that selects the kept positions also copies the kept rows that are about to be overwritten to the
 * workspace, and one more launch writes every kept row; no order between workgroups is assumed.  `ws` (DEVICE, 16-byte
 * aligned) must hold jq_evict_inplace_workspace_bytes (the scratch of jq_evict plus room for the pruned cache).
 * idx_out (kept positions) and scores_out (pooled scores) may be NULL; nothing may overlap K or V. */
int jq_evict_inplace_workspace_bytes(const jq_shape* shape, size_t* bytes);
int jq_evict_inplace(const jq_shape* shape, const void* Q, void* K, void* V, const float* lse,
                     int32_t* idx_out, float* scores_out, void* ws, size_t ws_bytes, void* stream);

/* One step of eviction DURING DECODING (the paper's closing paragraph names streaming eviction in the decoding
 * phase as future work and defines nothing; this is the Section 4.3 step applied to the cache as it stands).
 * Between two steps a layer's cache holds, per KV head, the rows the last step kept plus the rows of the tokens
 * decoded since; row b of head g is that head's own b-th row (heads keep different tokens), and
 *   pos[l, g, cu_seqlens[s] + b]     (DEVICE int32 [n_layers, h_kv, T])
 * says which token of the conversation it came from.  The soft tokens are appended after the generated text and run
 * through the model as at the end of prefill; their queries Q score the cached rows -- softmax over the cached
 * rows alone (lse NULL, two passes), or with the normalisers the attention kernel produced for those soft tokens
 * (lse as in jq_score_lse, one pass) -- then pooling along the cache rows (pool_k = 1 is the natural choice once
 * neighbouring rows are no longer neighbouring tokens), top-budgets[s] per head and the gather, exactly as
 * jq_evict; keep_first / keep_last protect the first rows (sinks) and the newest rows (e.g. the tokens decoded
 * since the last step).  Besides K_out, V_out and idx_out (ROW numbers in the cache that was passed in) the call
 * writes
 *   pos_out[l, g, cu_budgets[s] + b] = pos[l, g, cu_seqlens[s] + idx_out[l, g, cu_budgets[s] + b]]
 * (DEVICE int32 [n_layers, h_kv, sum budgets]), so that positions survive any number of steps. */
int jq_evict_stream(const jq_shape* shape, const void* Q, const void* K, const void* V, const int32_t* pos,
                    const float* lse, void* K_out, void* V_out, int32_t* pos_out,
                    int32_t* idx_out, float* scores_out, void* ws, size_t ws_bytes, void* stream);

/* jq_evict with caller-supplied normalisers (see jq_score_lse): one pass over K. */
int jq_evict_lse(const jq_shape* shape, const void* Q, const void* K, const void* V, const float* lse,
                 void* K_out, void* V_out, int32_t* idx_out, float* scores_out,
                 void* ws, size_t ws_bytes, void* stream);

/* jq_evict with the soft tokens' own keys in the softmax (see jq_score_tail). */
int jq_evict_tail(const jq_shape* shape, const void* Q, const void* K, const void* V, const void* K_tail,
                  void* K_out, void* V_out, int32_t* idx_out, float* scores_out,
                  void* ws, size_t ws_bytes, void* stream);

/* The same eviction (Section 4.3) on a PAGED key-value cache, the layout serving engines keep:
 * each layer's keys live in a pool of fixed-size pages, and a per-sequence block table says which
 * page holds which stretch of the sequence.
 *   K_pool, V_pool  DEVICE bf16 [n_layers, n_pages, page_size, h_kv, d]
 *   token t of sequence s is row (t % page_size) of page block_table[s, t / page_size]
 * Everything else -- Q, scores, idx (sequence-local LOGICAL positions), the dense K_out / V_out
 * [n_layers, sum budgets, h_kv, d], cu_seqlens, budgets, keep_first / keep_last -- is as in jq_evict.
 * Rows of a page beyond the sequence's end are never read.  A block-table entry outside
 * 0..n_pages-1 is clamped into that range (never dereferenced out of bounds); the table is read
 * on the device only, so its entries cannot be validated here. */
typedef struct jq_pages {
    int32_t page_size;          /* tokens per page: a power of two, 32..65536                       */
    int32_t n_pages;            /* pages in each layer's pool; n_pages * page_size * h_kv * d * 2   */
                                /* bytes must stay below 4 GiB                                      */
    int32_t max_pages_per_seq;  /* row length of block_table; >= ceil(L_s / page_size) for every s  */
    const int32_t* block_table; /* DEVICE int32 [n_seq, max_pages_per_seq]                          */
} jq_pages;

/* jq_score / jq_score_lse on a paged cache: `lse` NULL selects the two-pass softmax over the
 * prompt keys, otherwise the supplied normalisers are used and K is read once. */
int jq_score_paged(const jq_shape* shape, const jq_pages* pages, const void* Q, const void* K_pool,
                   const float* lse, float* scores, void* ws, size_t ws_bytes, void* stream);

/* jq_evict / jq_evict_lse on a paged cache (`lse` as above).  With `out_pages` NULL the kept rows are
 * gathered out of the pools into the dense K_out / V_out [n_layers, sum budgets, h_kv, d].  Otherwise
 * K_out / V_out are pools of their own, [n_layers, out_pages->n_pages, out_pages->page_size, h_kv, d],
 * and kept row b of sequence s (0 <= b < budgets[s]) goes to row (b % page_size) of page
 * out_pages->block_table[s, b / page_size]: the pruned cache is paged again and can be handed to the
 * attention kernels as it is.  For the output the page size may be any power of two (1..65536), the pool may
 * exceed 4 GiB, and max_pages_per_seq must cover ceil(budgets[s] / page_size); the output pools must not
 * overlap the input pools (jq_evict_paged_inplace writes into the input's own pools). */
int jq_evict_paged(const jq_shape* shape, const jq_pages* pages, const jq_pages* out_pages, const void* Q,
                   const void* K_pool, const void* V_pool, const float* lse, void* K_out, void* V_out,
                   int32_t* idx_out, float* scores_out, void* ws, size_t ws_bytes, void* stream);

/* The paged eviction without a second cache: the kept rows are written into pages of the very pools they are
 * taken from.  `out_pages` describes where (same page_size and n_pages as `pages`, its own block table
 * [n_seq, max_pages_per_seq]): kept row b of sequence s goes to row (b % page_size) of page
 * out_pages->block_table[s, b / page_size] -- any pages of the pool, in particular pages the sequences occupy now, so
 * that everything else can be handed back to the allocator.  A kept row that lives on a page which receives rows is
 * copied to the workspace before anything is written (a one-bit-per-page map of those pages is built first), then one
 * more launch writes every kept row; no order between workgroups is assumed.  Pages named by out_pages must not be
 * shared between sequences; rows of those pages beyond the kept rows keep their old contents.  `lse` as in
 * jq_evict_paged.  `ws` must hold jq_evict_paged_inplace_workspace_bytes. */
int jq_evict_paged_inplace_workspace_bytes(const jq_shape* shape, const jq_pages* pages, size_t* bytes);
int jq_evict_paged_inplace(const jq_shape* shape, const jq_pages* pages, const jq_pages* out_pages, const void* Q,
                           void* K_pool, void* V_pool, const float* lse, int32_t* idx_out, float* scores_out,
                           void* ws, size_t ws_bytes, void* stream);

/* jq_evict with kernel timing (the measurement hook of the benchmark): `marks` is a
 * HOST array of JQ_TRACE_MARKS hipEvent_t (passed as void*), created by the caller.
 * Kernel i of the sequence below is launched with marks[2i] / marks[2i+1] as its
 * start / stop events, so that hipEventElapsedTime(marks[2i], marks[2i+1]) is the
 * duration of that dispatch alone:
 *   0 statistics pass over K   1 score pass over K (merges the statistics first)
 *   2 pooling (+ histogram and sorted segments)    3 selection + gather
 * (when a stage needs several launches the last one is reported; sequences too long
 * for the selection's fast path take a streaming selection, reported in slot 3, and an
 * untimed separate gather; sequences long enough to leave hundreds of partial
 * statistics get an untimed merge launch between slots 0 and 1).  Results are those of
 * jq_evict. */
#define JQ_TRACE_MARKS 8
int jq_evict_traced(const jq_shape* shape, const void* Q, const void* K, const void* V,
                    void* K_out, void* V_out, int32_t* idx_out, float* scores_out,
                    void* ws, size_t ws_bytes, void* stream, void* const* marks, int n_marks);

/* Measurement aid, not part of the method: a plain device-to-device copy kernel of
 * `bytes` bytes (a multiple of 16; 16-byte aligned, non-overlapping DEVICE buffers).
 * Profilers read its known traffic to calibrate their HBM byte counters. */
int jq_copy_probe(const void* src, void* dst, size_t bytes, void* stream);

/* Ablation and diagnosis knobs.  The library reads a few environment variables ONCE per process, at its first
 * call (never on the path of a later call): JQ_CHUNK_KEYS / JQ_CHUNK_KEYS_2 (keys per wave in the first / second
 * pass over K, multiples of 32 up to 8192), JQ_DEPTH_1 / JQ_DEPTH_2 (key tiles a wave keeps in flight, 1 or 2),
 * JQ_LOG (print the HIP error string when a launch is refused).  Results do not depend on them beyond rounding
 * order.  jq_reload_knobs reads the environment again; it must not run concurrently with other calls (tests use
 * it to force rarely taken code paths at small sizes).  Always returns JQ_OK. */
int jq_reload_knobs(void);

/* Static, never-NULL description of a status code. */
const char* jq_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* JQ_H_ */
