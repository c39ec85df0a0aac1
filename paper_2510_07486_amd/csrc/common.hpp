// Internal declarations shared by the gfx950 kernels of the KV-selection hot path.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "asyncspade.h"
#include "asyncspade_debug.h"
#include "guards.hpp"

#define AS_HEAD_DIM 128
#define AS_PAGE 16
#define AS_MAX_WINDOW 64
#define AS_MAX_GROUP 64
#define AS_MAX_BUDGET 65536
#define AS_ATTN_CHUNK 128 /* tokens per attention split */
#define AS_PACK_MAX AS_MAX_PACK /* layers one packed selection launch can cover */
#define AS_SEL_COUNTERS 16384 /* arrival counters of the selection kernel (one per row of a launch), at the head of the scratch */

struct as_ctx {
  int device;
  void* ws;
  size_t ws_bytes;
  int select_mode;   /* 0: fused score+top-k unless the share plan keeps every token (see select_prefers_stages),
                        1: always the separate kernels via HBM scores, 2: always fused, 3: always via HBM scores, in one
                        launch where the shape allows */
  int attn_splits;   /* > 0: forced number of attention splits per (sequence, KV head) */
  int merge_mode;    /* 0: rows cut into shares are merged inside the selection kernel where its LDS holds the row's
                        candidates, 1: always by a second launch */
  int predict_mode;  /* 0: the predictor is a launch of its own, 1: it runs in the prologue of the fused selection
                        kernel where that kernel can */
  long long* timeline;   /* development: device buffer that receives wall_clock64 at entry and exit of every */
  int timeline_cap;      /* workgroup of the selection and attention kernels (pairs), and its capacity in pairs */
};

namespace asx {

// development hook: where workgroups leave their entry / exit clock (buf == nullptr: nowhere)
struct wg_timeline {
  long long* buf;
  int cap;
};
// The entry clock is only read (it stays in scalar registers); both marks are stored at the exit.  A store at the
// very start of a kernel was measured to cost the selection kernel a quarter more vector registers.
__device__ __forceinline__ long long timeline_begin(const wg_timeline& tl) { return tl.buf ? wall_clock64() : 0; }
__device__ __forceinline__ void timeline_end(const wg_timeline& tl, long long t_in) {
  if (tl.buf && threadIdx.x == 0) {
    const int wg = (blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;
    if (wg < tl.cap) {
      tl.buf[2 * wg] = t_in;
      tl.buf[2 * wg + 1] = wall_clock64();
    }
  }
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t lo16) { return __uint_as_float(lo16 << 16); }
// low / high bf16 of a packed dword -> fp32
__device__ __forceinline__ float bf16lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
// fp32 -> bf16 bits, round to nearest even (finite inputs; NaN kept quiet)
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

// element offset of token `slot` of (page, kv head j) in a [pages][Hkv][16][128] pool
__device__ __forceinline__ int64_t chunk_offset(int32_t page, int Hkv, int j) {
  return ((int64_t)page * Hkv + j) * (int64_t)(AS_PAGE * AS_HEAD_DIM);
}

// Per-layer pointers of a packed launch (several decoder layers in one grid).  Passed to the
// kernels by value: the layer index is uniform per workgroup, so a kernel reads its entry with
// scalar loads from the kernel-argument segment and no pointer table has to be staged in HBM.
struct pred_tab {
  const uint16_t* q_win[AS_PACK_MAX];
  const uint16_t* q_cur[AS_PACK_MAX];
  float* q_hat[AS_PACK_MAX];
};
struct sel_tab {
  const uint16_t* k_pool[AS_PACK_MAX];
  const int32_t* block_table[AS_PACK_MAX];
  const int32_t* ctx_lens[AS_PACK_MAX];
  const float* q_hat[AS_PACK_MAX];
  int32_t* sel_idx[AS_PACK_MAX];
  int32_t* sel_cnt[AS_PACK_MAX];
  int32_t last_page[AS_PACK_MAX];   // num_pages - 1 of the layer's pool (page ids are clamped to it)
  wg_timeline timeline;             // development hook of the slice kernel
  // predictor in the kernel's prologue (q_hat[] is then unused): the query window and the predictor's parameters
  const uint16_t* q_win[AS_PACK_MAX];
  const uint16_t* q_cur[AS_PACK_MAX];
  double pred_eps, pred_beta;
  int32_t pred_window, pred_single;
};

// ---- launchers (host) -------------------------------------------------------------
// predictor over n_layers * batch * n_q_heads heads; single-layer form below
hipError_t launch_predict_pack(const as_params* p, int n_layers, const pred_tab& tab, hipStream_t s);
hipError_t launch_predict(const as_params* p, const uint16_t* q_win, const uint16_t* q_cur, float* q_hat,
                          hipStream_t s);
hipError_t launch_score(const as_params* p, const as_kv_view* kv, const float* q_hat, float* scores, int64_t stride,
                        hipStream_t s);
// calibration kernels (score.hip): the paged walk of the scoring kernels, and a plain front-to-back read
hipError_t launch_stream_read_paged(const as_params* p, const as_kv_view* kv, float* sink, int64_t stride,
                                    bool words_per_token, hipStream_t s);
hipError_t launch_stream_read_flat(const void* buf, size_t nbytes, uint32_t* sink, hipStream_t s);
size_t stream_read_flat_sink_words();
// few-row shapes: scoring and the per-row top-k in one grid (select_rows.hip), over the rows of n_layers layers
bool select_rows_ok(const as_params* p, int n_layers);
bool select_rows_preferred(const as_params* p, int n_layers);
int select_rows_share_pages(const as_params* p, int n_layers);   // pages of a row per workgroup; 0: the form does not serve the shape
size_t select_rows_score_bytes(const as_params* p, int n_layers);
hipError_t launch_select_rows(const as_params* p, int n_layers, const sel_tab& tab, float* scores, int64_t stride,
                              int32_t* arrivals, hipStream_t s);
hipError_t launch_topk(const as_params* p, const float* scores, int64_t stride, const int32_t* ctx_lens,
                       int32_t* sel_idx, int32_t* sel_cnt, hipStream_t s);
// fused scoring + top-k (select_fused.hip): rows are cut into slices of `slice_len` tokens
struct select_plan { int slice_len, nslices, ccap; };
select_plan plan_select(const as_params* p, int n_layers);
bool select_plan_ok(const as_params* p, int n_layers);
bool select_prefers_stages(const as_params* p);
size_t select_workspace_bytes(const as_params* p, int n_layers);
// whether the slice kernel of this shape can run the predictor in its prologue (windows of up to 16 queries,
// groups of up to 16 heads, max / sum aggregation)
bool select_can_predict(const as_params* p);
// fuse_predict: tab carries q_win / q_cur instead of q_hat (only where select_can_predict)
// arrivals: AS_SEL_COUNTERS counters that are zero before the launch (and zero again after it), or nullptr
hipError_t launch_select_pack(const as_params* p, int n_layers, const sel_tab& tab, void* ws, int32_t* arrivals,
                              bool fuse_predict, hipStream_t s);
// q_win != nullptr: the predictor runs in the kernel's prologue and q_hat is not read
hipError_t launch_select_fused(const as_params* p, const as_kv_view* kv, const float* q_hat, const uint16_t* q_win,
                               const uint16_t* q_cur, void* ws, int32_t* arrivals, int32_t* sel_idx, int32_t* sel_cnt,
                               wg_timeline tl, hipStream_t s);
// partial buffers live in the ctx workspace
// forced_splits > 0 overrides the split rule (development knob of a ctx)
size_t attn_workspace_bytes(const as_params* p, int forced_splits);
hipError_t launch_attn(const as_params* p, const as_kv_view* kv, const uint16_t* q, const int32_t* sel_idx,
                       const int32_t* sel_cnt, const int32_t* sel_ctx_lens, uint16_t* out, float* lse, void* ws,
                       int forced_splits, wg_timeline tl, hipStream_t s);

// cache-side bookkeeping (cache_ops.hip)
hipError_t launch_kv_append(const as_params* p, uint16_t* k_pool, uint16_t* v_pool, const int32_t* block_table,
                            int32_t* ctx_lens, int64_t num_pages, const uint16_t* k_new, const uint16_t* v_new,
                            hipStream_t s);
hipError_t launch_window_push(const as_params* p, uint16_t* q_win, uint16_t* q_cur, const uint16_t* q_new,
                              hipStream_t s);
hipError_t launch_gather_kv(const as_params* p, const as_kv_view* kv, const int32_t* sel_idx, const int32_t* sel_cnt,
                            uint16_t* k_out, uint16_t* v_out, int32_t* out_table, int32_t* out_lens, hipStream_t s);
hipError_t launch_overlap(const as_params* p, const int32_t* idx_a, const int32_t* cnt_a, const int32_t* idx_b,
                          const int32_t* cnt_b, int32_t* inter, float* ratio, hipStream_t s);

}  // namespace asx
