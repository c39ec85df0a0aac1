// C ABI of the KV-selection hot path: argument validation, workspace carving, launches.
// No device allocation outside as_create / as_destroy and no host synchronisation.
#include <mutex>
#include <new>

#include "common.hpp"

// Scratch of as_select_step_static: device memory that belongs to the library image, not to a ctx.  Every GPU the
// library is loaded on holds its own copy at its own address.  In host code this name is only a handle for
// hipGetSymbolAddress (see static_scratch below); it is never passed to a kernel, a copy or a fill.
static __device__ __align__(256) unsigned char scratch[AS_STATIC_SCRATCH_BYTES];

namespace {

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

constexpr size_t WS_GAP = 256;          // never written by a kernel: separates the regions of the workspace
constexpr unsigned char WS_FILL = 0xA5;  // what as_create fills the workspace with
// The workspace begins with the arrival counters of the selection kernel (rows cut into shares: the last workgroup
// of a row merges it): zero when as_create returns and zero again after every launch that used them, whatever the
// parameters of the call were.
constexpr size_t WS_COUNTER_BYTES = AS_SEL_COUNTERS * sizeof(int32_t);

struct ws_layout {
  size_t counters, attn, q_hat, q_hat_layer, scores, cand, total;
  size_t attn_end;   // what the attention calls need: the attention region and the gap behind it
  size_t gap[4];     // offsets of the gaps behind the attention partials, q_hat, the score rows, the candidates
  int64_t score_stride;
};

// The attention partials come first, so that a ctx that only attends needs nothing else.  n_layers > 1: the
// layout of a packed selection (one q_hat block per layer, candidates of the whole pack); the single-layer
// layout also holds the score rows of the unfused path.  attn_splits: the forced split count of the ctx (0 = rule).
// a pack whose shape the one-launch form over score rows serves and wins on (select_rows.hip)
bool pack_rows_shape(const as_params* p, int n_layers) {
  return p->agg != AS_AGG_SOFTMAX_SUM && asx::select_rows_ok(p, n_layers) && asx::select_rows_preferred(p, n_layers);
}

ws_layout layout_of(const as_params* p, int n_layers = 1, int attn_splits = 0) {
  ws_layout l;
  l.score_stride = (int64_t)p->max_pages_per_seq * AS_PAGE;
  l.counters = 0;                                            // same place and size under every layout
  l.attn = WS_COUNTER_BYTES + WS_GAP;
  l.gap[0] = l.attn + align_up(asx::attn_workspace_bytes(p, attn_splits));
  l.attn_end = l.gap[0] + WS_GAP;
  l.q_hat = l.attn_end;
  l.q_hat_layer = align_up((size_t)p->batch * p->n_q_heads * AS_HEAD_DIM * sizeof(float));
  l.gap[1] = l.q_hat + l.q_hat_layer * n_layers;
  l.scores = l.gap[1] + WS_GAP;
  // score rows: of the single layer (stand-alone stages, one-launch form); of a pack only where the pack's shape
  // can take the one-launch form
  size_t sc = 0;
  if (n_layers == 1) sc = align_up((size_t)p->batch * p->n_kv_heads * (size_t)l.score_stride * sizeof(float));
  else if (pack_rows_shape(p, n_layers)) sc = align_up(asx::select_rows_score_bytes(p, n_layers));
  l.gap[2] = l.scores + sc;
  l.cand = l.gap[2] + WS_GAP;
  l.gap[3] = l.cand + align_up(asx::select_workspace_bytes(p, n_layers));
  l.total = l.gap[3] + WS_GAP;
  return l;
}

as_status check_params(const as_params* p) {
  if (!p) return AS_ERR_INVALID_ARG;
  if (p->batch < 0 || p->n_q_heads <= 0 || p->n_kv_heads <= 0 || p->head_dim <= 0 || p->page_size <= 0 ||
      p->window < 1 || p->budget < 1 || p->max_pages_per_seq < 0)
    return AS_ERR_INVALID_ARG;
  if (p->n_q_heads % p->n_kv_heads != 0) return AS_ERR_INVALID_ARG;
  if (!(p->ridge_eps > 0.f)) return AS_ERR_INVALID_ARG;
  if (p->agg != AS_AGG_MAX && p->agg != AS_AGG_SUM && p->agg != AS_AGG_SOFTMAX_SUM) return AS_ERR_INVALID_ARG;
  if (p->predictor != AS_PRED_PER_WINDOW && p->predictor != AS_PRED_SINGLE_SOLVE) return AS_ERR_INVALID_ARG;
  if (p->head_dim != AS_HEAD_DIM || p->page_size != AS_PAGE) return AS_ERR_UNSUPPORTED;
  if (p->window > AS_MAX_WINDOW || p->budget > AS_MAX_BUDGET) return AS_ERR_UNSUPPORTED;
  if (p->n_q_heads / p->n_kv_heads > AS_MAX_GROUP) return AS_ERR_UNSUPPORTED;
  if (p->batch > 65535 || p->n_kv_heads > 65535) return AS_ERR_UNSUPPORTED;                 // grid dimensions
  if ((int64_t)p->batch * p->n_kv_heads > 0x7fffffffLL) return AS_ERR_UNSUPPORTED;          // rows are grid.x of the top-k
  if ((int64_t)p->n_kv_heads * ((p->n_q_heads / p->n_kv_heads + 15) / 16) > 65535) return AS_ERR_UNSUPPORTED;  // grid.y of attention
  if ((int64_t)p->max_pages_per_seq * AS_PAGE > (int64_t)1 << 25) return AS_ERR_UNSUPPORTED;
  return AS_OK;
}

as_status check_kv(const as_kv_view* kv, bool need_v) {
  if (!kv || !kv->k_pool || !kv->block_table || !kv->ctx_lens) return AS_ERR_INVALID_ARG;
  if (need_v && !kv->v_pool) return AS_ERR_INVALID_ARG;
  if (kv->num_pages < 1) return AS_ERR_INVALID_ARG;
  if (kv->num_pages > 0x7fffffffLL) return AS_ERR_UNSUPPORTED;   // page ids are int32
  return AS_OK;
}

inline as_status hip_status(hipError_t e) { return e == hipSuccess ? AS_OK : AS_ERR_HIP; }

// Whether a single-layer selection runs as the two stand-alone stages (scores through the workspace) instead of
// the fused kernels: when the fused kernels have no share plan for the shape, when the plan could not prune
// anything, when the one-launch form over score rows is faster for the shape, or when the development knob says so.
// The softmax-normalised aggregation exists only in the fused kernels.
bool use_stages(int select_mode, bool one_launch, const as_params* p) {
  if (p->agg == AS_AGG_SOFTMAX_SUM) return false;
  if (!asx::select_plan_ok(p, 1)) return true;      // more shares per row than the merge kernel indexes
  if (select_mode == 2) return false;
  if (select_mode == 1 || select_mode == 3 || asx::select_prefers_stages(p)) return true;
  // mid-size shapes where scoring and top-k in one launch beat the fused kernels (only if that form will run)
  return one_launch && asx::select_rows_ok(p, 1) && asx::select_rows_preferred(p, 1);
}

// arrivals != nullptr and a shape the one-launch form serves: scoring and the per-row top-k share a grid
// (select_rows.hip); otherwise the two stand-alone kernels, one after the other.  Same scores, same selection.
hipError_t score_then_topk(const as_params* p, const as_kv_view* kv, const float* q_hat, float* scores, int64_t stride,
                           int32_t* arrivals, int32_t* sel_idx, int32_t* sel_cnt, hipStream_t s) {
  if (arrivals && asx::select_rows_ok(p, 1)) {
    asx::sel_tab tab = {};                       // a pack of one layer
    tab.k_pool[0] = static_cast<const uint16_t*>(kv->k_pool);
    tab.block_table[0] = kv->block_table;
    tab.ctx_lens[0] = kv->ctx_lens;
    tab.q_hat[0] = q_hat;
    tab.sel_idx[0] = sel_idx;
    tab.sel_cnt[0] = sel_cnt;
    tab.last_page[0] = (int32_t)(kv->num_pages - 1);
    return asx::launch_select_rows(p, 1, tab, scores, stride, arrivals, s);
  }
  const hipError_t e = asx::launch_score(p, kv, q_hat, scores, stride, s);
  if (e != hipSuccess) return e;
  return asx::launch_topk(p, scores, stride, kv->ctx_lens, sel_idx, sel_cnt, s);
}


as_status check_select_step(const as_params* p, const as_kv_view* kv, const void* q_win, const void* q_cur,
                            const int32_t* sel_idx, const int32_t* sel_cnt) {
  as_status st = check_params(p);
  if (st != AS_OK) return st;
  if ((st = check_kv(kv, false)) != AS_OK) return st;
  if (!q_win || !q_cur || !sel_idx || !sel_cnt) return AS_ERR_INVALID_ARG;
  if (p->agg == AS_AGG_SOFTMAX_SUM && !asx::select_plan_ok(p, 1)) return AS_ERR_UNSUPPORTED;
  return AS_OK;
}

// One layer-step of selection with its scratch regions given explicitly (parts of the ctx workspace, or of the
// static scratch array): q_hat, then the score rows (stand-alone stages) or the candidate region (fused
// kernels), whichever the route needs.  The predictor is a launch of its own (measured faster in every workload);
// with predict_mode 1 and a shape whose fused selection kernel can run the predictor in its own prologue, no
// separate predictor launch is made and q_hat is not used at all.
as_status select_step_on(int32_t* arrivals, float* q_hat, float* scores, int64_t score_stride, char* cand, bool stages, int predict_mode,
                         const as_params* p, const as_kv_view* kv, const void* q_win, const void* q_cur,
                         int32_t* sel_idx, int32_t* sel_cnt, asx::wg_timeline tl, hipStream_t s) {
  const uint16_t* qw = static_cast<const uint16_t*>(q_win);
  const uint16_t* qc = static_cast<const uint16_t*>(q_cur);
  if (!stages && predict_mode == 1 && asx::select_can_predict(p))
    return hip_status(asx::launch_select_fused(p, kv, nullptr, qw, qc, cand, arrivals, sel_idx, sel_cnt, tl, s));
  hipError_t e = asx::launch_predict(p, qw, qc, q_hat, s);
  if (e != hipSuccess) return AS_ERR_HIP;
  if (!stages)
    return hip_status(asx::launch_select_fused(p, kv, q_hat, nullptr, nullptr, cand, arrivals, sel_idx, sel_cnt, tl, s));
  return hip_status(score_then_topk(p, kv, q_hat, scores, score_stride, arrivals, sel_idx, sel_cnt, s));
}

// The device address of `scratch` that kernels, copies and fills may use: resolved once per device, with that
// device current, and kept here.
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
char* g_scratch_ptr[MAX_DEVICES] = {};

// `device` must be the current device.  nullptr if the address cannot be resolved.
char* static_scratch(int device) {
  if (device < 0 || device >= MAX_DEVICES) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
    g_scratch_ptr[device] = static_cast<char*>(ptr);
  }
  return g_scratch_ptr[device];
}

}  // namespace

extern "C" {

size_t as_workspace_bytes(const as_params* p) {
  if (check_params(p) != AS_OK) return 0;
  return layout_of(p).total;
}

size_t as_workspace_bytes_attn(const as_params* p) {
  if (check_params(p) != AS_OK) return 0;
  return layout_of(p).attn_end;
}

as_status as_create(as_ctx** out, int device, size_t workspace_bytes) {
  if (!out) return AS_ERR_INVALID_ARG;
  *out = nullptr;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) return AS_ERR_HIP;
  if (hipSetDevice(device) != hipSuccess) return AS_ERR_HIP;
  (void)static_scratch(device);   // set-up of as_select_step_static on this device (its own call repeats it if needed)
  as_ctx* c = new (std::nothrow) as_ctx();
  if (!c) return AS_ERR_HIP;
  c->device = device;
  c->ws = nullptr;
  c->ws_bytes = workspace_bytes;
  c->select_mode = 0;
  c->attn_splits = 0;
  c->predict_mode = 0;
  c->merge_mode = 0;
  c->timeline = nullptr;
  c->timeline_cap = 0;
  if (workspace_bytes > 0) {
    if (hipMalloc(&c->ws, workspace_bytes) != hipSuccess) {
      delete c;
      return AS_ERR_HIP;
    }
    if (hipMemset(c->ws, WS_FILL, workspace_bytes) != hipSuccess ||   // the gaps between regions keep this pattern
        hipMemset(c->ws, 0, workspace_bytes < WS_COUNTER_BYTES ? workspace_bytes : WS_COUNTER_BYTES) != hipSuccess) {
      (void)hipFree(c->ws);
      delete c;
      return AS_ERR_HIP;
    }
  }
  *out = c;
  return AS_OK;
}

as_status as_destroy(as_ctx* ctx) {
  if (!ctx) return AS_ERR_INVALID_ARG;
  hipError_t e = hipSuccess;
  if (ctx->ws) e = hipFree(ctx->ws);
  delete ctx;
  return hip_status(e);
}

const char* as_status_str(as_status s) {
  switch (s) {
    case AS_OK: return "ok";
    case AS_ERR_INVALID_ARG: return "invalid argument";
    case AS_ERR_UNSUPPORTED: return "unsupported configuration";
    case AS_ERR_WORKSPACE: return "ctx workspace too small";
    case AS_ERR_HIP: return "HIP runtime error";
    case AS_ERR_STATIC_SCRATCH: return "parameters need more than the static scratch array holds";
  }
  return "unknown status";
}

as_status as_predict_query(as_ctx* ctx, const as_params* p, const void* q_win, const void* q_cur, float* q_hat,
                           void* stream) {
  as_status st = check_params(p);
  if (st != AS_OK) return st;
  if (!ctx || !q_win || !q_cur || !q_hat) return AS_ERR_INVALID_ARG;
  return hip_status(asx::launch_predict(p, static_cast<const uint16_t*>(q_win), static_cast<const uint16_t*>(q_cur),
                                        q_hat, static_cast<hipStream_t>(stream)));
}

as_status as_score_keys(as_ctx* ctx, const as_params* p, const as_kv_view* kv, const float* q_hat, float* scores,
                        int64_t score_stride, void* stream) {
  as_status st = check_params(p);
  if (st != AS_OK) return st;
  if ((st = check_kv(kv, false)) != AS_OK) return st;
  if (!ctx || !q_hat || !scores) return AS_ERR_INVALID_ARG;
  if (p->agg == AS_AGG_SOFTMAX_SUM) return AS_ERR_UNSUPPORTED;   // needs the row-wide normalisers: fused calls only
  if (score_stride < (int64_t)p->max_pages_per_seq * AS_PAGE) return AS_ERR_INVALID_ARG;
  return hip_status(asx::launch_score(p, kv, q_hat, scores, score_stride, static_cast<hipStream_t>(stream)));
}

as_status as_topk_select(as_ctx* ctx, const as_params* p, const float* scores, int64_t score_stride,
                         const int32_t* ctx_lens, int32_t* sel_idx, int32_t* sel_cnt, void* stream) {
  as_status st = check_params(p);
  if (st != AS_OK) return st;
  if (!ctx || !scores || !ctx_lens || !sel_idx || !sel_cnt) return AS_ERR_INVALID_ARG;
  if (score_stride < (int64_t)p->max_pages_per_seq * AS_PAGE) return AS_ERR_INVALID_ARG;
  return hip_status(asx::launch_topk(p, scores, score_stride, ctx_lens, sel_idx, sel_cnt,
                                     static_cast<hipStream_t>(stream)));
}

as_status as_sparse_decode_attn(as_ctx* ctx, const as_params* p, const as_kv_view* kv, const void* q,
                                const int32_t* sel_idx, const int32_t* sel_cnt, const int32_t* sel_ctx_lens,
                                void* out, float* lse, void* stream) {
  as_status st = check_params(p);
  if (st != AS_OK) return st;
  if ((st = check_kv(kv, true)) != AS_OK) return st;
  if (!ctx || !q || !sel_idx || !sel_cnt || !out) return AS_ERR_INVALID_ARG;
  const ws_layout l = layout_of(p, 1, ctx->attn_splits);
  if (!ctx->ws || ctx->ws_bytes < l.attn_end) return AS_ERR_WORKSPACE;   // the attention region leads the layout
  return hip_status(asx::launch_attn(p, kv, static_cast<const uint16_t*>(q), sel_idx, sel_cnt, sel_ctx_lens,
                                     static_cast<uint16_t*>(out), lse, static_cast<char*>(ctx->ws) + l.attn,
                                     ctx->attn_splits, asx::wg_timeline{ctx->timeline, ctx->timeline_cap},
                                     static_cast<hipStream_t>(stream)));
}

as_status as_dense_decode_attn(as_ctx* ctx, const as_params* p, const as_kv_view* kv, const void* q, void* out,
                               float* lse, void* stream) {
  as_status st = check_params(p);
  if (st != AS_OK) return st;
  if ((st = check_kv(kv, true)) != AS_OK) return st;
  if (!ctx || !q || !out) return AS_ERR_INVALID_ARG;
  const ws_layout l = layout_of(p, 1, ctx->attn_splits);
  if (!ctx->ws || ctx->ws_bytes < l.attn_end) return AS_ERR_WORKSPACE;
  return hip_status(asx::launch_attn(p, kv, static_cast<const uint16_t*>(q), nullptr, nullptr, nullptr,
                                     static_cast<uint16_t*>(out), lse, static_cast<char*>(ctx->ws) + l.attn,
                                     ctx->attn_splits, asx::wg_timeline{ctx->timeline, ctx->timeline_cap},
                                     static_cast<hipStream_t>(stream)));
}

as_status as_score_topk(as_ctx* ctx, const as_params* p, const as_kv_view* kv, const float* q_hat, int32_t* sel_idx,
                        int32_t* sel_cnt, void* stream) {
  as_status st = check_params(p);
  if (st != AS_OK) return st;
  if ((st = check_kv(kv, false)) != AS_OK) return st;
  if (!ctx || !q_hat || !sel_idx || !sel_cnt) return AS_ERR_INVALID_ARG;
  if (p->agg == AS_AGG_SOFTMAX_SUM && !asx::select_plan_ok(p, 1)) return AS_ERR_UNSUPPORTED;
  const bool one_launch = ctx->merge_mode == 0 && ctx->select_mode != 1;
  const bool stages = use_stages(ctx->select_mode, one_launch, p);
  const ws_layout l = layout_of(p, 1, ctx->attn_splits);
  if (!ctx->ws || ctx->ws_bytes < l.total) return AS_ERR_WORKSPACE;
  char* ws = static_cast<char*>(ctx->ws);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (!stages)
    return hip_status(asx::launch_select_fused(p, kv, q_hat, nullptr, nullptr, ws + l.cand,
                                               ctx->merge_mode == 0 ? reinterpret_cast<int32_t*>(ws + l.counters) : nullptr,
                                               sel_idx, sel_cnt, asx::wg_timeline{ctx->timeline, ctx->timeline_cap}, s));
  return hip_status(score_then_topk(p, kv, q_hat, reinterpret_cast<float*>(ws + l.scores), l.score_stride,
                                    one_launch ? reinterpret_cast<int32_t*>(ws + l.counters) : nullptr,
                                    sel_idx, sel_cnt, s));
}

as_status as_select_step(as_ctx* ctx, const as_params* p, const as_kv_view* kv, const void* q_win, const void* q_cur,
                         int32_t* sel_idx, int32_t* sel_cnt, void* stream) {
  as_status st = check_select_step(p, kv, q_win, q_cur, sel_idx, sel_cnt);
  if (st != AS_OK) return st;
  if (!ctx) return AS_ERR_INVALID_ARG;
  const ws_layout l = layout_of(p, 1, ctx->attn_splits);
  if (!ctx->ws || ctx->ws_bytes < l.total) return AS_ERR_WORKSPACE;
  char* ws = static_cast<char*>(ctx->ws);
  const bool stages = use_stages(ctx->select_mode, ctx->merge_mode == 0 && ctx->select_mode != 1, p);
  // the arrival counters serve the merge inside the fused kernel and the one-launch form over score rows alike
  const bool counters = ctx->merge_mode == 0 && !(stages && ctx->select_mode == 1);
  return select_step_on(counters ? reinterpret_cast<int32_t*>(ws + l.counters) : nullptr,
                        reinterpret_cast<float*>(ws + l.q_hat), reinterpret_cast<float*>(ws + l.scores), l.score_stride,
                        ws + l.cand, stages, ctx->predict_mode, p, kv, q_win, q_cur, sel_idx,
                        sel_cnt, asx::wg_timeline{ctx->timeline, ctx->timeline_cap}, static_cast<hipStream_t>(stream));
}

as_status as_select_step_static(const as_params* p, const as_kv_view* kv, const void* q_win, const void* q_cur,
                                int32_t* sel_idx, int32_t* sel_cnt, void* stream) {
  as_status st = check_select_step(p, kv, q_win, q_cur, sel_idx, sel_cnt);
  if (st != AS_OK) return st;
  // q_hat, a gap, then the one region the route of this shape uses: score rows or candidates
  const bool stages = use_stages(0, true, p);
  const int64_t score_stride = (int64_t)p->max_pages_per_seq * AS_PAGE;
  const size_t q_bytes = align_up((size_t)p->batch * p->n_q_heads * AS_HEAD_DIM * sizeof(float));
  const size_t region = stages ? (size_t)p->batch * p->n_kv_heads * (size_t)score_stride * sizeof(float)
                               : asx::select_workspace_bytes(p, 1);
  // the array starts with the arrival counters (zero at load time like the whole array, zero again after every call)
  const size_t q_off = WS_COUNTER_BYTES + WS_GAP;
  const size_t region_off = q_off + q_bytes + WS_GAP;
  if (region_off + region > (size_t)AS_STATIC_SCRATCH_BYTES) return AS_ERR_STATIC_SCRATCH;
  int device = 0;
  if (hipGetDevice(&device) != hipSuccess) return AS_ERR_HIP;
  char* base = static_scratch(device);    // this GPU's copy of the array (its address is resolved once per device)
  if (!base) return AS_ERR_HIP;
  return select_step_on(reinterpret_cast<int32_t*>(base), reinterpret_cast<float*>(base + q_off),
                        reinterpret_cast<float*>(base + region_off), score_stride,
                        base + region_off, stages, 0, p, kv, q_win, q_cur, sel_idx, sel_cnt,
                        asx::wg_timeline{nullptr, 0}, static_cast<hipStream_t>(stream));
}

size_t as_workspace_bytes_pack(const as_params* p, int32_t n_layers) {
  if (check_params(p) != AS_OK || n_layers < 1 || n_layers > AS_MAX_PACK) return 0;
  return layout_of(p, n_layers).total;
}

as_status as_select_step_pack(as_ctx* ctx, const as_params* p, const as_layer_io* layers, int32_t n_layers,
                              void* stream) {
  as_status st = check_params(p);
  if (st != AS_OK) return st;
  if (!ctx || !layers || n_layers < 1) return AS_ERR_INVALID_ARG;
  if (n_layers > AS_MAX_PACK || (int64_t)p->batch * n_layers > 65535) return AS_ERR_UNSUPPORTED;
  for (int l = 0; l < n_layers; ++l) {
    if ((st = check_kv(&layers[l].kv, false)) != AS_OK) return st;
    if (!layers[l].q_win || !layers[l].q_cur || !layers[l].sel_idx || !layers[l].sel_cnt) return AS_ERR_INVALID_ARG;
  }
  if (!asx::select_plan_ok(p, n_layers)) return AS_ERR_UNSUPPORTED;
  const ws_layout lay = layout_of(p, n_layers, ctx->attn_splits);
  if (!ctx->ws || ctx->ws_bytes < lay.total) return AS_ERR_WORKSPACE;
  char* ws = static_cast<char*>(ctx->ws);
  asx::pred_tab pt = {};
  asx::sel_tab stab = {};
  stab.timeline = asx::wg_timeline{ctx->timeline, ctx->timeline_cap};
  for (int l = 0; l < n_layers; ++l) {
    float* q_hat = reinterpret_cast<float*>(ws + lay.q_hat + lay.q_hat_layer * l);
    pt.q_win[l] = static_cast<const uint16_t*>(layers[l].q_win);
    pt.q_cur[l] = static_cast<const uint16_t*>(layers[l].q_cur);
    pt.q_hat[l] = q_hat;
    stab.k_pool[l] = static_cast<const uint16_t*>(layers[l].kv.k_pool);
    stab.block_table[l] = layers[l].kv.block_table;
    stab.ctx_lens[l] = layers[l].kv.ctx_lens;
    stab.q_hat[l] = q_hat;
    stab.sel_idx[l] = layers[l].sel_idx;
    stab.sel_cnt[l] = layers[l].sel_cnt;
    stab.last_page[l] = (int32_t)(layers[l].kv.num_pages - 1);
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  // few rows in the whole pack: scoring and top-k over score rows in one grid (the workspace holds score rows for a
  // pack only where pack_rows_shape says so); development routes 1 and 2 keep the fused kernels
  const bool rows_route = n_layers > 1 && ctx->merge_mode == 0 && (ctx->select_mode == 0 || ctx->select_mode == 3) &&
                          pack_rows_shape(p, n_layers);
  const bool fuse = !rows_route && ctx->predict_mode == 1 && asx::select_can_predict(p);   // predictor in the selection kernel's prologue
  if (fuse) {
    for (int l = 0; l < n_layers; ++l) {
      stab.q_win[l] = pt.q_win[l];
      stab.q_cur[l] = pt.q_cur[l];
    }
  } else {
    hipError_t e = asx::launch_predict_pack(p, n_layers, pt, s);
    if (e != hipSuccess) return AS_ERR_HIP;
  }
  if (rows_route)
    return hip_status(asx::launch_select_rows(p, n_layers, stab, reinterpret_cast<float*>(ws + lay.scores),
                                              lay.score_stride, reinterpret_cast<int32_t*>(ws + lay.counters), s));
  return hip_status(asx::launch_select_pack(p, n_layers, stab, ws + lay.cand,
                                            ctx->merge_mode == 0 ? reinterpret_cast<int32_t*>(ws + lay.counters) : nullptr,
                                            fuse, s));
}

as_status as_kv_append(as_ctx* ctx, const as_params* p, void* k_pool, void* v_pool, const int32_t* block_table,
                       int32_t* ctx_lens, int64_t num_pages, const void* k_new, const void* v_new, void* stream) {
  as_status st = check_params(p);
  if (st != AS_OK) return st;
  if (!ctx || !k_pool || !v_pool || !block_table || !ctx_lens || !k_new || !v_new || num_pages < 1)
    return AS_ERR_INVALID_ARG;
  if (num_pages > 0x7fffffffLL) return AS_ERR_UNSUPPORTED;
  return hip_status(asx::launch_kv_append(p, static_cast<uint16_t*>(k_pool), static_cast<uint16_t*>(v_pool),
                                          block_table, ctx_lens, num_pages, static_cast<const uint16_t*>(k_new),
                                          static_cast<const uint16_t*>(v_new), static_cast<hipStream_t>(stream)));
}

as_status as_window_push(as_ctx* ctx, const as_params* p, void* q_win, void* q_cur, const void* q_new,
                         void* stream) {
  as_status st = check_params(p);
  if (st != AS_OK) return st;
  if (!ctx || !q_win || !q_cur || !q_new || q_new == q_cur) return AS_ERR_INVALID_ARG;
  return hip_status(asx::launch_window_push(p, static_cast<uint16_t*>(q_win), static_cast<uint16_t*>(q_cur),
                                            static_cast<const uint16_t*>(q_new), static_cast<hipStream_t>(stream)));
}

as_status as_gather_kv(as_ctx* ctx, const as_params* p, const as_kv_view* kv, const int32_t* sel_idx,
                       const int32_t* sel_cnt, void* k_out, void* v_out, int32_t* out_table, int32_t* out_lens,
                       void* stream) {
  as_status st = check_params(p);
  if (st != AS_OK) return st;
  if ((st = check_kv(kv, true)) != AS_OK) return st;
  if (!ctx || !sel_idx || !sel_cnt || !k_out || !v_out || !out_table || !out_lens) return AS_ERR_INVALID_ARG;
  if (k_out == kv->k_pool || v_out == kv->v_pool) return AS_ERR_INVALID_ARG;
  return hip_status(asx::launch_gather_kv(p, kv, sel_idx, sel_cnt, static_cast<uint16_t*>(k_out),
                                          static_cast<uint16_t*>(v_out), out_table, out_lens,
                                          static_cast<hipStream_t>(stream)));
}

as_status as_overlap_ratio(as_ctx* ctx, const as_params* p, const int32_t* idx_a, const int32_t* cnt_a,
                           const int32_t* idx_b, const int32_t* cnt_b, int32_t* inter, float* ratio, void* stream) {
  as_status st = check_params(p);
  if (st != AS_OK) return st;
  if (!ctx || !idx_a || !cnt_a || !idx_b || !cnt_b || !inter) return AS_ERR_INVALID_ARG;
  return hip_status(asx::launch_overlap(p, idx_a, cnt_a, idx_b, cnt_b, inter, ratio,
                                        static_cast<hipStream_t>(stream)));
}

// ---- development and measurement entry points (asyncspade_debug.h) ----

as_status as_debug_select_plan(const as_params* p, int32_t n_layers, int32_t* out) {
  if (check_params(p) != AS_OK || !out || n_layers < 1) return AS_ERR_INVALID_ARG;
  const asx::select_plan pl = asx::plan_select(p, n_layers);
  out[0] = pl.slice_len;
  out[1] = pl.nslices;
  out[2] = pl.ccap;
  return AS_OK;
}

as_status as_debug_rows_plan(const as_params* p, int32_t n_layers, int32_t* out) {
  if (check_params(p) != AS_OK || !out || n_layers < 1 || n_layers > AS_MAX_PACK) return AS_ERR_INVALID_ARG;
  out[0] = asx::select_rows_ok(p, n_layers) ? 1 : 0;
  out[1] = out[0] && (n_layers == 1 ? use_stages(0, true, p) : pack_rows_shape(p, n_layers)) ? 1 : 0;
  out[2] = out[0] ? asx::select_rows_share_pages(p, n_layers) : 0;
  out[3] = out[0] ? (p->max_pages_per_seq > 0 ? (p->max_pages_per_seq + out[2] - 1) / out[2] : 1) : 0;
  return AS_OK;
}

as_status as_debug_workspace_gaps(as_ctx* ctx, const as_params* p, int32_t n_layers, int32_t* first_bad) {
  if (!ctx || !first_bad || check_params(p) != AS_OK || n_layers < 1 || n_layers > AS_MAX_PACK)
    return AS_ERR_INVALID_ARG;
  const ws_layout l = layout_of(p, n_layers, ctx->attn_splits);
  if (!ctx->ws || ctx->ws_bytes < l.total) return AS_ERR_WORKSPACE;
  if (hipDeviceSynchronize() != hipSuccess) return AS_ERR_HIP;
  *first_bad = -1;
  for (int g = 0; g < 4; ++g) {
    unsigned char host[WS_GAP];
    if (hipMemcpy(host, static_cast<char*>(ctx->ws) + l.gap[g], WS_GAP, hipMemcpyDeviceToHost) != hipSuccess)
      return AS_ERR_HIP;
    for (size_t i = 0; i < WS_GAP; ++i)
      if (host[i] != WS_FILL) {
        *first_bad = g;
        return AS_OK;
      }
  }
  return AS_OK;
}

as_status as_debug_set_select_mode(as_ctx* ctx, int32_t mode) {
  if (!ctx || mode < 0 || mode > 3) return AS_ERR_INVALID_ARG;
  ctx->select_mode = mode;
  return AS_OK;
}

as_status as_debug_set_merge_mode(as_ctx* ctx, int32_t mode) {
  if (!ctx || mode < 0 || mode > 1) return AS_ERR_INVALID_ARG;
  ctx->merge_mode = mode;
  return AS_OK;
}

as_status as_debug_set_predict_mode(as_ctx* ctx, int32_t mode) {
  if (!ctx || mode < 0 || mode > 1) return AS_ERR_INVALID_ARG;
  ctx->predict_mode = mode;
  return AS_OK;
}

as_status as_debug_set_timeline(as_ctx* ctx, int64_t* buf, int32_t capacity) {
  if (!ctx || capacity < 0 || (capacity > 0 && !buf)) return AS_ERR_INVALID_ARG;
  ctx->timeline = capacity > 0 ? reinterpret_cast<long long*>(buf) : nullptr;
  ctx->timeline_cap = capacity;
  return AS_OK;
}

as_status as_debug_set_attn_splits(as_ctx* ctx, int32_t splits) {
  if (!ctx || splits < 0) return AS_ERR_INVALID_ARG;
  ctx->attn_splits = splits;
  return AS_OK;
}

size_t as_debug_attn_workspace_bytes(const as_params* p, int32_t splits) {
  if (check_params(p) != AS_OK || splits < 0) return 0;
  return layout_of(p, 1, splits).attn_end;
}

as_status as_debug_stream_read_paged(as_ctx* ctx, const as_params* p, const as_kv_view* kv, float* sink,
                                     int64_t stride, int32_t words_per_token, void* stream) {
  as_status st = check_params(p);
  if (st != AS_OK) return st;
  if ((st = check_kv(kv, false)) != AS_OK) return st;
  if (!ctx || !sink) return AS_ERR_INVALID_ARG;
  if (stride < (int64_t)p->max_pages_per_seq * AS_PAGE) return AS_ERR_INVALID_ARG;
  return hip_status(asx::launch_stream_read_paged(p, kv, sink, stride, words_per_token != 0,
                                                  static_cast<hipStream_t>(stream)));
}

as_status as_debug_stream_read_flat(as_ctx* ctx, const void* buf, size_t nbytes, uint32_t* sink, void* stream) {
  if (!ctx || !buf || !sink || nbytes % 16 != 0) return AS_ERR_INVALID_ARG;
  return hip_status(asx::launch_stream_read_flat(buf, nbytes, sink, static_cast<hipStream_t>(stream)));
}

size_t as_debug_stream_read_flat_sink_words(void) { return asx::stream_read_flat_sink_words(); }

}  // extern "C"
