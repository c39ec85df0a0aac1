/*
 * asyncspade.h -- C ABI of the MI355X (gfx950) KV-selection hot path of AsyncSpade.
 *
 * One decode step of token-level, query-aware KV-cache selection:
 *   predict  the next-step query from a sliding window of recent queries
 *            (Sec. 4.2: Eq. 2-3 ridge regression + softmax, Eq. 4 single-token shift,
 *            Eq. 5 mean over window sizes; Appendix C Alg. 1 steps 1-6),
 *   score    every cached key against the predicted query (Alg. 1 step 7; shapes of
 *            Sec. 4.3 "Batched Matmul"), aggregated over each GQA group,
 *   top-k    keep a per-KV-head budget of the highest-scoring tokens (Sec. 4.3,
 *            cache-rank item (2)),
 *   attend   decode attention with the REAL query over only the selected tokens
 *            (Sec. 4.1; Appendix B counts 4*q*h*C flops for exactly this).
 *
 * Conventions
 *   - Every pointer except as_ctx* / as_params* / as_kv_view* is a DEVICE pointer owned
 *     by the caller.  The library allocates device memory only in as_create (the ctx
 *     workspace), frees it in as_destroy, and never synchronises the host: all work is
 *     enqueued on the hipStream_t passed (as void*; NULL = the default stream).
 *   - One ctx per concurrently used stream (the workspace is per ctx).
 *   - bf16 = raw 16-bit brain-float bit patterns.  head_dim must be 128 and page_size 16.
 *   - KV layout: token n of sequence b lives in page block_table[b][n / 16], slot n % 16;
 *     element offset ((page * n_kv_heads + j) * 16 + slot) * 128 in the pool (64-bit).
 *   - Query head h belongs to KV head h / G with G = n_q_heads / n_kv_heads (1 <= G <= 64: multi-head,
 *     grouped-query and multi-query layouts).
 *   - Return codes only; nothing throws or aborts across this boundary.  Arguments are
 *     validated on the host before any launch: AS_ERR_INVALID_ARG for null pointers,
 *     non-positive sizes, n_q_heads % n_kv_heads != 0, ridge_eps <= 0;
 *     AS_ERR_UNSUPPORTED for head_dim != 128, page_size != 16, window > 64, group > 64,
 *     budget > 65536, batch or n_kv_heads > 65535, batch * n_kv_heads > 2^31 - 1,
 *     n_kv_heads * ceil(group / 16) > 65535, a block table of more than 2^25 tokens per sequence, and for as_select_step_pack and the softmax-normalised aggregation when
 *     budget > 4096 is combined with a block table of more than 8 million tokens per sequence
 *     (as_score_topk and as_select_step then run the stand-alone stages);
 *     AS_ERR_WORKSPACE if the ctx workspace is too small for the call.
 *     Contents of device arrays (page ids in range, indices unique and in range) are
 *     the caller's contract; as a guard against faults, page ids are clamped into
 *     [0, num_pages) and token indices into [0, ctx_lens[b]) before they are used, so a
 *     corrupt table gives unspecified results for its rows but no out-of-pool access.
 *     num_pages must be >= 1.
 */
#ifndef ASYNCSPADE_H
#define ASYNCSPADE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The library is built with hidden visibility; only the entry points declared here (and in
 * asyncspade_debug.h) are exported. */
#if defined(AS_BUILDING_LIBRARY)
#define AS_API __attribute__((visibility("default")))
#else
#define AS_API
#endif

typedef struct as_ctx as_ctx; /* opaque: device id + scratch workspace */

typedef enum {
  AS_OK = 0,
  AS_ERR_INVALID_ARG = 1,
  AS_ERR_UNSUPPORTED = 2,
  AS_ERR_WORKSPACE = 3,
  AS_ERR_HIP = 4,
  AS_ERR_STATIC_SCRATCH = 5 /* as_select_step_static: the parameters need more scratch than the static array holds */
} as_status;

/* How the per-query-head logits of a GQA group become one score per KV head (the paper leaves it open):
 *   AS_AGG_MAX          max over the group of the raw logits (default)
 *   AS_AGG_SUM          sum over the group of the raw logits (= the logit of the summed query)
 *   AS_AGG_SOFTMAX_SUM  sum over the group of each head's softmax probability,
 *                       s[n] = sum_g exp(sm_scale * l[g][n] - LSE_g): scale-free across heads; costs a second
 *                       pass over K; only the fused calls (as_score_topk, as_select_step, as_select_step_pack)
 *                       offer it, as_score_keys returns AS_ERR_UNSUPPORTED */
typedef enum { AS_AGG_MAX = 0, AS_AGG_SUM = 1, AS_AGG_SOFTMAX_SUM = 2 } as_agg;

/* How the weights of window size k are obtained (Sec. 4.2 vs Appendix C):
 *   AS_PRED_PER_WINDOW    one ridge problem per window size, over its k newest predecessors (Sec. 4.2,
 *                         "Assembled Regression": the default and the reading the parity tests pin);
 *   AS_PRED_SINGLE_SOLVE  one ridge solve over all W predecessors, the weights of window size k are the
 *                         softmax of the solution truncated to its k newest entries (Alg. 1 steps 3-5). */
typedef enum { AS_PRED_PER_WINDOW = 0, AS_PRED_SINGLE_SOLVE = 1 } as_predictor;

typedef struct {
  int32_t batch, n_q_heads, n_kv_heads, head_dim; /* head_dim must be 128                          */
  int32_t page_size;                              /* must be 16                                    */
  int32_t window;                                 /* W >= 1 predecessors in q_win (<= 64)          */
  int32_t budget;                                 /* C >= 1 tokens kept per (sequence, kv head)    */
  int32_t max_pages_per_seq;                      /* row stride of block_table; bounds every ctx   */
  float ridge_eps;                                /* eps > 0 added to the Gram diagonal (absolute) */
  float softmax_beta;                             /* weights = softmax(beta * omega); +1 default,  */
                                                  /* -1 is the sign printed in Alg. 1 step 3       */
  float sm_scale;                                 /* attention logit scale, e.g. 1/sqrt(128)       */
  int32_t agg;                                    /* as_agg: group aggregation of the scores       */
  int32_t predictor;                              /* as_predictor                                  */
} as_params;

typedef struct {            /* caller-owned device memory, never freed by the library */
  const void* k_pool;       /* bf16 [num_pages][n_kv_heads][16][128]                  */
  const void* v_pool;       /* same shape (may be NULL for calls that only score)     */
  const int32_t* block_table; /* [batch][max_pages_per_seq] physical page ids         */
  const int32_t* ctx_lens;  /* [batch] tokens currently cached, <= 16*max_pages_per_seq */
  int64_t num_pages;
} as_kv_view;

/* Bytes of ctx workspace that every call with these parameters fits in (the attention split
 * partials, then as_select_step's q_hat, score rows and per-share candidates).  The longest
 * context is bounded by p->max_pages_per_seq, so no separate context length is passed.
 * as_workspace_bytes_attn is the leading part of that layout that as_sparse_decode_attn and
 * as_dense_decode_attn need: a ctx that only ever attends can be created with just that.
 * Both return 0 for parameters the library rejects. */
AS_API size_t as_workspace_bytes(const as_params* p);
AS_API size_t as_workspace_bytes_attn(const as_params* p);

/* Creates a ctx on `device` with a workspace of `workspace_bytes` (hipMalloc).  as_destroy frees it
 * (hipFree): like any allocation call, neither belongs inside an open stream capture, and work that
 * still uses the workspace must have finished.  Every other call only enqueues kernels. */
AS_API as_status as_create(as_ctx** out, int device, size_t workspace_bytes);
AS_API as_status as_destroy(as_ctx* ctx);
AS_API const char* as_status_str(as_status s);

/*
 * Query predictor (Sec. 4.2, Eq. 2-5).  For every (b, h): for each window size k = 1..W
 * solve (R_k R_k^T + eps I) omega = R_k Q_t over the k newest predecessors, take
 * w = softmax(beta * omega), apply w to the window shifted by one token (Q_t, Q_{t-1}, ...),
 * and average the W candidates.  fp64 inside, fp32 out.
 *   q_win  bf16 [B][Hq][W][128], oldest first (Q_{t-W} .. Q_{t-1})
 *   q_cur  bf16 [B][Hq][128]     (Q_t: regression target and newest shifted element)
 *   q_hat  fp32 [B][Hq][128]     out
 */
AS_API as_status as_predict_query(as_ctx* ctx, const as_params* p, const void* q_win, const void* q_cur,
                           float* q_hat, void* stream);

/*
 * Criticality scores (Alg. 1 step 7 with the (bs, N_kv, N_q/N_kv, D_h) x (bs, N_kv, N_t, D_h)
 * shapes of Sec. 4.3):  scores[b][j][n] = agg_g <q_hat[b][j*G+g], K[b][j][n]> for n < ctx_lens[b],
 * fp32, with -0 written as +0.  Entries n >= ctx_lens[b] are left untouched.
 *   scores fp32 [B][Hkv][score_stride], score_stride >= 16 * max_pages_per_seq
 */
AS_API as_status as_score_keys(as_ctx* ctx, const as_params* p, const as_kv_view* kv, const float* q_hat,
                        float* scores, int64_t score_stride, void* stream);

/*
 * Top-k (Sec. 4.3 item (2)).  Per (b, j): the min(C, ctx_lens[b]) tokens with the largest
 * score; equal scores resolve to the lowest index; NaN ranks below -inf; -0 == +0.
 *   sel_idx int32 [B][Hkv][C]  ascending token indices, padded with -1
 *   sel_cnt int32 [B][Hkv]
 */
AS_API as_status as_topk_select(as_ctx* ctx, const as_params* p, const float* scores, int64_t score_stride,
                         const int32_t* ctx_lens, int32_t* sel_idx, int32_t* sel_cnt, void* stream);

/*
 * Sparse decode attention (Sec. 4.1).  For query head h (KV head j = h / G), over
 * S = sel_idx[b][j][0 .. sel_cnt) plus the dense tail [sel_ctx_lens[b], ctx_lens[b]):
 *   out = sum_{n in S} softmax_n(sm_scale * <q, K_n>) V_n      (fp32 inside, bf16 out)
 *   lse = log sum_{n in S} exp(sm_scale * <q, K_n>)            (natural log)
 * The tail lets a step attend to tokens appended after its selection was made
 * (selection for step t+1 happens at step t); pass NULL for no tail.
 * Empty S gives out = 0, lse = -inf.
 *   q    bf16 [B][Hq][128];  out bf16 [B][Hq][128];  lse nullable fp32 [B][Hq]
 */
AS_API as_status as_sparse_decode_attn(as_ctx* ctx, const as_params* p, const as_kv_view* kv, const void* q,
                                const int32_t* sel_idx, const int32_t* sel_cnt,
                                const int32_t* sel_ctx_lens, void* out, float* lse, void* stream);

/*
 * Dense decode attention over the whole cache, tokens [0, ctx_lens[b]): the full-attention
 * baseline the method is measured against (Appendix B: 4*q*h*T per layer instead of 4*q*h*C),
 * and the call that reads a compact pool written by as_gather_kv.  Same kernels, layouts and
 * precision as as_sparse_decode_attn; the work is split over the longest context the block
 * table allows (16 * max_pages_per_seq).
 */
AS_API as_status as_dense_decode_attn(as_ctx* ctx, const as_params* p, const as_kv_view* kv, const void* q, void* out,
                               float* lse, void* stream);

/*
 * Scoring and top-k in one pass (Alg. 1 step 7 + Sec. 4.3 item (2)): same result as
 * as_score_keys followed by as_topk_select, but the per-token scores never leave the chip
 * (rows are scored in slices whose keys stay in LDS; only per-slice candidates, 8 B each,
 * go through the ctx workspace).  This is the kernel pair as_select_step runs.  One exception,
 * chosen on the host from the shapes: when the rows are so few that they are cut into slices
 * no longer than the budget (batch 1, short context), no slice could discard anything, and on
 * small shapes in general (at most 128 rows and 2^20 tokens in all) pruning saves less than it
 * costs: the call then scores into score rows in the ctx workspace and selects from them, in
 * one launch where the rows fit the register top-k (32768 tokens, groups of up to 16 heads),
 * else with the two stand-alone kernels; the result is the same.
 */
AS_API as_status as_score_topk(as_ctx* ctx, const as_params* p, const as_kv_view* kv, const float* q_hat,
                        int32_t* sel_idx, int32_t* sel_cnt, void* stream);

/*
 * Fused selection for one layer-step: as_predict_query then as_score_topk enqueued back to
 * back on `stream`, with q_hat and the candidates kept in the ctx workspace.  This is the work
 * the paper's Cache Rank does per layer (Sec. 4.1, Sec. 4.3); run it on its own stream
 * to overlap it with another layer's attention.
 */
AS_API as_status as_select_step(as_ctx* ctx, const as_params* p, const as_kv_view* kv, const void* q_win,
                         const void* q_cur, int32_t* sel_idx, int32_t* sel_cnt, void* stream);

/*
 * as_select_step for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  It needs no ctx.  The same kernels run with q_hat, the score rows and
 * the per-share candidates in a static device array of AS_STATIC_SCRATCH_BYTES that is part of the library
 * image (every GPU the library runs on holds that much until the process ends); the call makes no
 * allocation and frees nothing.  Results are identical, bit for bit, to as_select_step.
 *   - runs on the CURRENT device; inputs and outputs are the caller's, as in as_select_step
 *   - scratch need: q_hat (batch * n_q_heads * 512 B) plus the one region the shape's route uses, the
 *     per-share candidates (rows cut into several shares: 8 B per candidate) or the score rows (few-row shapes
 *     that run the stand-alone stages: 4 B per token); as_workspace_bytes(p) - as_workspace_bytes_attn(p) is
 *     an upper bound.  Parameters that need more than AS_STATIC_SCRATCH_BYTES are refused with
 *     AS_ERR_STATIC_SCRATCH before anything is launched
 *   - the array's device address is looked up once per device, on the first call there or in any earlier
 *     as_create on that device: make one of the two happen before a stream capture begins
 *   - all calls on one GPU share the one array.  Nothing in it needs clearing between calls: apart from the
 *     arrival counters at its head, every word a kernel reads was written earlier in the same call, and the
 *     counters (zero when the library is loaded) are put back to zero by the kernel that used them.  Calls that
 *     overlap in time on one GPU, on whatever streams, race and give unspecified results
 */
#define AS_STATIC_SCRATCH_BYTES (48u << 20)
AS_API as_status as_select_step_static(const as_params* p, const as_kv_view* kv, const void* q_win, const void* q_cur,
                                       int32_t* sel_idx, int32_t* sel_cnt, void* stream);

/*
 * Depth-wise packed selection (Sec. 4.3, the paragraph on depth-wise parallelism of the cache
 * rank: the selections of several consecutive layers are made together, as one unit of work).
 * One call = as_select_step for n_layers layers, run as ONE predictor launch and ONE
 * scoring/top-k launch (plus one merge launch when rows are cut into more shares than the
 * kernel merges itself) whose grids cover every layer of the pack.  Each layer brings its own cache view, query
 * window and output arrays; all layers share the shapes in `p`.  Results are identical, bit
 * for bit, to n_layers separate as_select_step calls.
 *   layers    HOST array of n_layers entries (read during the call, not kept);
 *             1 <= n_layers <= AS_MAX_PACK, else AS_ERR_UNSUPPORTED
 *   the ctx workspace must hold as_workspace_bytes_pack(p, n_layers), else AS_ERR_WORKSPACE
 */
#define AS_MAX_PACK 16
typedef struct {
  as_kv_view kv;       /* this layer's cache; block_table / ctx_lens may be shared by the layers */
  const void* q_win;   /* bf16 [B][Hq][W][128] oldest first */
  const void* q_cur;   /* bf16 [B][Hq][128]                 */
  int32_t* sel_idx;    /* int32 [B][Hkv][C] out             */
  int32_t* sel_cnt;    /* int32 [B][Hkv]    out             */
} as_layer_io;
AS_API size_t as_workspace_bytes_pack(const as_params* p, int32_t n_layers);
AS_API as_status as_select_step_pack(as_ctx* ctx, const as_params* p, const as_layer_io* layers, int32_t n_layers,
                              void* stream);

/*
 * Cache-side state update of one decode step (Sec. 4.1, workflow: the cache rank appends the
 * step's key / value states to the KV cache and enqueues its query state to the sliding window).
 *
 * as_kv_append: for every sequence b with room (ctx_lens[b] < 16 * max_pages_per_seq) the rows
 * k_new[b][j], v_new[b][j] are stored at token position n = ctx_lens[b] (page
 * block_table[b][n / 16], which the caller's allocator must have mapped) and ctx_lens[b]
 * becomes n + 1.  A sequence without room is left unchanged.  The pools and ctx_lens are
 * written: calls that read them on other streams must be ordered after this one by the caller.
 *   k_pool, v_pool bf16 [num_pages][Hkv][16][128] (in place); ctx_lens int32 [B] (in place)
 *   k_new, v_new   bf16 [B][Hkv][128]
 *
 * as_window_push: q_win loses its oldest entry, the previous q_cur becomes its newest entry and
 * q_new becomes q_cur (all in place; q_new may not alias q_cur).
 */
AS_API as_status as_kv_append(as_ctx* ctx, const as_params* p, void* k_pool, void* v_pool, const int32_t* block_table,
                       int32_t* ctx_lens, int64_t num_pages, const void* k_new, const void* v_new, void* stream);
AS_API as_status as_window_push(as_ctx* ctx, const as_params* p, void* q_win, void* q_cur, const void* q_new,
                         void* stream);

/*
 * KV re-organisation for the filtered tokens (Sec. 4.3, cache-rank item (3)): copies the
 * selected K and V rows, in selection order, into a compact paged pool that any paged decode
 * kernel can read contiguously.  With Cp = ceil(budget / 16) pages per sequence, token i of
 * (b, j) goes to page b * Cp + i / 16, slot i % 16; slots at and beyond sel_cnt[b][j] are left
 * untouched.  out_table / out_lens describe the compact pool as a cache view of its own
 * (out_table[b][i] = b * Cp + i, out_lens[b] = sel_cnt[b][0]): as_dense_decode_attn over that
 * view, with max_pages_per_seq = Cp, is attention over exactly the selected tokens.
 *   k_out, v_out bf16 [B * Cp][Hkv][16][128];  out_table int32 [B][Cp];  out_lens int32 [B]
 */
AS_API as_status as_gather_kv(as_ctx* ctx, const as_params* p, const as_kv_view* kv, const int32_t* sel_idx,
                       const int32_t* sel_cnt, void* k_out, void* v_out, int32_t* out_table, int32_t* out_lens,
                       void* stream);

/*
 * Overlap ratio of two selections (Sec. 3, Eq. 1): per (b, j), inter = |S_a intersect S_b| and
 * ratio = inter / |S|, |S| being the common set size (the larger of the two counts if they
 * differ; 0 / 0 gives 0).  Both index lists must be ascending, as the selection calls emit them.
 *   idx_a, idx_b int32 [B][Hkv][C]; cnt_a, cnt_b int32 [B][Hkv]
 *   inter int32 [B][Hkv] out; ratio nullable fp32 [B][Hkv] out
 */
AS_API as_status as_overlap_ratio(as_ctx* ctx, const as_params* p, const int32_t* idx_a, const int32_t* cnt_a,
                           const int32_t* idx_b, const int32_t* cnt_b, int32_t* inter, float* ratio,
                           void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ASYNCSPADE_H */
