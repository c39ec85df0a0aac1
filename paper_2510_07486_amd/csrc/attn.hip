// Host side of sparse / dense decode attention (Sec. 4.1; the 4*q*h*C term of Appendix B): the split
// geometry, the partial buffers in the ctx workspace, and the kernel that merges the split partials.  The
// attention kernel itself (both contractions on the matrix cores) is in attn_mfma.hip.
#include "common.hpp"

namespace asx {

static constexpr int AT_SPLIT = AS_ATTN_CHUNK;  // smallest workgroup split, tokens (bounds the number of partials)

// Split geometry for a logical token list of at most `list_len` tokens per (sequence, KV head): how many
// workgroups share a row and how many wavefronts (4 or 8) a workgroup has.  Measured (32/8 and 64/8 heads,
// budgets 1024-4096): what counts is that all wavefronts are resident at once, about eight per compute unit
// (2048 in all; a second, partly filled round costs 5-10 %), and that every wavefront gets the same number of
// 32-token steps.  Rows that one workgroup can take whole are not split at all: the kernel then finishes them
// itself and neither partials nor the merge launch exist.  So: eight-wavefront workgroups when a whole number of
// them per row gives one workgroup per compute unit or fewer, else four-wavefront ones; the split count is the
// largest that keeps the grid within one round, preferably one that divides the list into equal whole steps per
// wavefront; never below AT_SPLIT tokens per split.
struct attn_geom { int nsplit, waves; };
static attn_geom attn_geometry(const as_params* p, int64_t list_len, int forced) {
  const int G = p->n_q_heads / p->n_kv_heads;
  if (list_len < 1) list_len = 1;
  int64_t pairs = (int64_t)p->batch * p->n_kv_heads * ((G + 15) / 16);
  if (pairs < 1) pairs = 1;
  const int64_t max_sel = (list_len + AT_SPLIT - 1) / AT_SPLIT;
  attn_geom g;
  // eight wavefronts per workgroup, one workgroup per compute unit: rows x splits <= 256 with >= 256 tokens per wavefront-set
  for (int waves : {8, 4}) {
    const int64_t slots = waves == 8 ? 256 : 768;            // workgroups resident at once
    const int64_t step_unit = 32 * waves;                    // tokens of one step of every wavefront
    int64_t nsel = slots / pairs;
    if (nsel > max_sel) nsel = max_sel;
    if (nsel < 1) nsel = 1;
    const int64_t units = list_len / step_unit;
    bool even = false;
    for (int64_t d = nsel; d >= 1 && d * pairs >= slots / 2; --d)
      if (units > 0 && units % d == 0 && list_len % step_unit == 0) {
        nsel = d;
        even = true;
        break;
      }
    g.nsplit = (int)nsel;
    g.waves = waves;
    // the eight-wavefront shape is taken when it fills at least seven eighths of the compute units evenly
    if (waves == 8 && even && nsel * pairs >= 224 && pairs <= 256) break;
  }
  if (forced > 0) {
    g.nsplit = (int)(forced < max_sel ? forced : max_sel);
    g.waves = 4;
  }
  return g;
}
static int attn_splits_for(const as_params* p, int64_t list_len, int forced) {
  return attn_geometry(p, list_len, forced).nsplit;
}

// partial outputs and partial (m, l) pairs, for the sparse call (list = budget) and the dense one
// (list = longest context the block table allows)
size_t attn_workspace_bytes(const as_params* p, int forced_splits) {
  const size_t heads = (size_t)p->batch * p->n_q_heads;
  const int ns = attn_splits_for(p, (int64_t)p->budget, forced_splits);
  const int nd = attn_splits_for(p, (int64_t)p->max_pages_per_seq * AS_PAGE, forced_splits);
  return heads * (size_t)(ns > nd ? ns : nd) * (AS_HEAD_DIM + 2) * sizeof(float);
}

// merges the split partials of one (sequence, query head).  A separate launch on purpose.  "Last workgroup of a
// row merges" was built twice and measured: with device-scope fences it is several times slower (they write back
// and invalidate the whole per-XCD L2); without fences (write-through stores, a completion wait, a barrier, one
// device-scope atomic, device-scope loads) it is correct but its serial chain of round trips at the end of the
// kernel costs what this launch costs (batch 16, 64/8 heads, budget 4096: 52.8 against 52.6 us).
__global__ __launch_bounds__(AS_HEAD_DIM) void attn_combine_kernel(const float* __restrict__ part_o,
                                                                   const float* __restrict__ part_ml,
                                                                   uint16_t* __restrict__ out,
                                                                   float* __restrict__ lse, int nsplit) {
  const int64_t bh = blockIdx.x;
  const int d = threadIdx.x;
  const float2* ml = reinterpret_cast<const float2*>(part_ml) + bh * nsplit;
  const float* po = part_o + bh * nsplit * AS_HEAD_DIM + d;
  // Partials are loaded in batches whose loads are all issued before the first is used (slots beyond nsplit re-read
  // the last partial and are masked afterwards: a guarded load would wait for its own round trip).  The first
  // sixteen (m, l) pairs and output values are fetched once, together, and serve both the maximum and the sum.
  constexpr int HELD = 16;
  const int last = nsplit - 1;
  float2 v0[HELD];
  float x0[HELD];
#pragma unroll
  for (int e = 0; e < HELD; ++e) {
    const int si = e < nsplit ? e : last;
    v0[e] = ml[si];
    x0[e] = po[(int64_t)si * AS_HEAD_DIM];
  }
  float M = -INFINITY;
#pragma unroll
  for (int e = 0; e < HELD; ++e)
    if (e < nsplit && v0[e].y > 0.f) M = fmaxf(M, v0[e].x);
  for (int s0 = HELD; s0 < nsplit; s0 += 8) {
    float2 v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = ml[s0 + e < nsplit ? s0 + e : last];
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (s0 + e < nsplit && v[e].y > 0.f) M = fmaxf(M, v[e].x);
  }
  float Lsum = 0.f, o = 0.f;
#pragma unroll
  for (int e = 0; e < HELD; ++e)
    if (e < nsplit && v0[e].y > 0.f) {
      const float wgt = expf(v0[e].x - M);
      Lsum += v0[e].y * wgt;
      o += wgt * x0[e];
    }
  for (int s0 = HELD; s0 < nsplit; s0 += 8) {
    float2 v[8];
    float x[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int si = s0 + e < nsplit ? s0 + e : last;
      v[e] = ml[si];
      x[e] = po[(int64_t)si * AS_HEAD_DIM];
    }
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (s0 + e < nsplit && v[e].y > 0.f) {
        const float wgt = expf(v[e].x - M);
        Lsum += v[e].y * wgt;
        o += wgt * x[e];
      }
  }
  const float r = (Lsum > 0.f) ? o / Lsum : 0.f;
  out[bh * AS_HEAD_DIM + d] = (uint16_t)f32_to_bf16_rne(r);
  if (lse && d == 0) lse[bh] = (Lsum > 0.f) ? M + logf(Lsum) : -INFINITY;
}

hipError_t launch_attn_mfma(const as_params* p, const as_kv_view* kv, const uint16_t* q, const int32_t* sel_idx,
                            const int32_t* sel_cnt, const int32_t* sel_ctx_lens, float* part_o, float* part_ml,
                            uint16_t* out, float* lse, int nsplit, int waves, int list_len, wg_timeline tl,
                            hipStream_t s);

// sel_idx == nullptr: dense attention over [0, ctx_lens[b]) (the token list is only the "tail", from 0)
hipError_t launch_attn(const as_params* p, const as_kv_view* kv, const uint16_t* q, const int32_t* sel_idx,
                       const int32_t* sel_cnt, const int32_t* sel_ctx_lens, uint16_t* out, float* lse, void* ws,
                       int forced_splits, wg_timeline tl, hipStream_t s) {
  const int64_t heads = (int64_t)p->batch * p->n_q_heads;
  if (heads == 0) return hipSuccess;
  const bool dense = sel_idx == nullptr;
  const int64_t list_len = dense ? (int64_t)p->max_pages_per_seq * AS_PAGE : (int64_t)p->budget;
  const attn_geom gm = attn_geometry(p, list_len, forced_splits);
  const int nsplit = gm.nsplit;
  float* part_o = reinterpret_cast<float*>(ws);
  float* part_ml = part_o + heads * nsplit * AS_HEAD_DIM;
  hipError_t e = launch_attn_mfma(p, kv, q, sel_idx, sel_cnt, sel_ctx_lens, part_o, part_ml, out, lse, nsplit,
                                  gm.waves, (int)list_len, tl, s);
  if (e != hipSuccess || nsplit == 1) return e;      // unsplit rows are finished by the attention kernel itself
  hipLaunchKernelGGL(attn_combine_kernel, dim3((unsigned)heads), dim3(AS_HEAD_DIM), 0, s, part_o, part_ml, out, lse,
                     nsplit);
  return hipGetLastError();
}

}  // namespace asx
