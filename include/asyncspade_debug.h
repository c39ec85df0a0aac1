/*
 * asyncspade_debug.h -- development and measurement entry points of libasyncspade.so.
 *
 * Nothing here is part of the method: these calls expose host-side planning decisions, check the
 * ctx workspace for overruns, override two launch heuristics of ONE ctx (never process-wide), and
 * run the memory-bandwidth calibration kernels that the benchmark and the profiler runs use.
 * Same conventions as asyncspade.h (device pointers owned by the caller, status codes, the
 * stream passed as void*).
 */
#ifndef ASYNCSPADE_DEBUG_H
#define ASYNCSPADE_DEBUG_H

#include "asyncspade.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Share plan of the fused selection for a pack of n_layers layers:
 * out[0..2] = {share length in tokens, shares per row, candidates kept per share}. */
AS_API as_status as_debug_select_plan(const as_params* p, int32_t n_layers, int32_t* out);

/* The one-launch selection over score rows (few rows) for a pack of n_layers layers:
 * out[0..3] = {the form serves the shape (0/1), the library prefers it to the fused kernels for the shape (0/1),
 * pages of a row one workgroup scores, workgroups per row}.  out[2] and out[3] are 0 when out[0] is. */
AS_API as_status as_debug_rows_plan(const as_params* p, int32_t n_layers, int32_t* out);

/* Checks the 256-byte gaps that separate the regions of the ctx workspace (layout of (p, n_layers)); a kernel
 * that wrote beyond its region has overwritten the pattern as_create left there.  Synchronises the device.
 * *first_bad = -1 if every gap is intact, else the index of the first damaged one (0 attention partials,
 * 1 q_hat, 2 score rows, 3 candidates).  Only meaningful for a ctx used with this one layout since as_create. */
AS_API as_status as_debug_workspace_gaps(as_ctx* ctx, const as_params* p, int32_t n_layers, int32_t* first_bad);

/* Route of single-layer selections of THIS ctx: 0 = chosen from the share plan (default), 1 = always the
 * stand-alone scoring and top-k kernels through score rows in the workspace (two launches), 2 = always the fused
 * kernels (where a share plan exists), 3 = always through score rows, scoring and top-k in one launch where the
 * shape allows it (what mode 0 does for few-row shapes). */
AS_API as_status as_debug_set_select_mode(as_ctx* ctx, int32_t mode);

/* How rows that the fused selection cuts into several shares are merged for THIS ctx: 0 = inside the selection kernel
 * by the last workgroup of the row to finish, wherever the row's candidates fit that kernel's LDS buffer (the
 * default), 1 = always by a second launch.  Results are identical, bit for bit. */
AS_API as_status as_debug_set_merge_mode(as_ctx* ctx, int32_t mode);

/* Where the predictor of as_select_step / as_select_step_pack runs for THIS ctx: 0 = as a launch of its own (the
 * default: measured faster on every benchmark workload), 1 = in the prologue of the fused selection kernel wherever
 * that kernel can (windows of up to 16 queries, groups of up to 16 heads, max or sum aggregation, fused route):
 * up to eight wavefronts of each workgroup predict one head each before the workgroup starts to stream.  Results
 * are identical, bit for bit. */
AS_API as_status as_debug_set_predict_mode(as_ctx* ctx, int32_t mode);

/* Forces the number of attention splits per (sequence, KV head) for THIS ctx (0 = the library's rule).  A forced
 * count that needs more partial buffers than the ctx workspace holds makes the attention calls return
 * AS_ERR_WORKSPACE; as_debug_attn_workspace_bytes gives the bytes the attention region needs under a forced count. */
AS_API as_status as_debug_set_attn_splits(as_ctx* ctx, int32_t splits);
AS_API size_t as_debug_attn_workspace_bytes(const as_params* p, int32_t splits);

/* Workgroup timeline of THIS ctx: while buf is set, every workgroup w (linear index, x fastest) of the fused
 * selection kernel and of the attention kernel writes the device's 100 MHz wall clock at its entry to buf[2 * w]
 * and at its exit to buf[2 * w + 1] (workgroups at and beyond `capacity` write nothing).  The buffer is device
 * memory of the caller's, 2 * capacity int64; each launch overwrites the last one's marks.  capacity = 0 switches
 * the marks off (the default). */
AS_API as_status as_debug_set_timeline(as_ctx* ctx, int64_t* buf, int32_t capacity);

/* Calibration kernels.  as_debug_stream_read_paged walks the K pages of every (sequence, KV head) exactly like
 * the scoring kernels (block table, coalesced non-temporal 128-bit loads) and does no arithmetic beyond an XOR
 * fold; words_per_token != 0 writes one 4-byte word per token into sink[b][j][n] (known read and write sizes,
 * for scaling profiler byte counters), 0 writes one word per wavefront.
 *   sink fp32 [B][Hkv][stride], stride >= 16 * max_pages_per_seq
 * as_debug_stream_read_flat reads nbytes (a multiple of 16) starting at buf front to back with coalesced
 * non-temporal 128-bit loads, no page table, and writes one word per workgroup: the plain streaming-read rate
 * of the chip.
 *   sink uint32 [as_debug_stream_read_flat_sink_words()] */
AS_API as_status as_debug_stream_read_paged(as_ctx* ctx, const as_params* p, const as_kv_view* kv, float* sink,
                                            int64_t stride, int32_t words_per_token, void* stream);
AS_API as_status as_debug_stream_read_flat(as_ctx* ctx, const void* buf, size_t nbytes, uint32_t* sink,
                                           void* stream);
AS_API size_t as_debug_stream_read_flat_sink_words(void);

#ifdef __cplusplus
}
#endif
#endif /* ASYNCSPADE_DEBUG_H */
