// Sparse decode attention with the real query over the selected tokens (Sec. 4.1; the
// 4*q*h*C term of Appendix B), plus an optional dense tail of tokens appended after the
// selection was made.
//
// HBM-bound on the index-gathered K and V rows (2 x 256 B per selected token and KV head).
// Split-C: a 256-thread workgroup owns one 128-token chunk of the logical token list of one
// (sequence, KV head) and up to 8 of the group's query heads, so every gathered row is read
// once for the whole group.  A 16-lane segment reads one 256-byte row with 128-bit loads
// (4 rows per wavefront load).  Per chunk: logits -> LDS, chunk max, p = exp(l - m), then
// P*V with no rescaling inside the chunk.  Partials (m, l, o) go to the workspace and a
// small second kernel merges them and writes bf16.
#include "common.hpp"

namespace asx {

static constexpr int AT_CHUNK = AS_ATTN_CHUNK;  // 128 tokens: 4 waves x 8 loads x 4 rows

__host__ __device__ inline int attn_nsplit(int C) { return (C + AT_CHUNK - 1) / AT_CHUNK + 1; }
static inline int attn_gh(int G) { return (G % 8 == 0) ? 8 : (G % 4 == 0) ? 4 : (G % 2 == 0) ? 2 : 1; }

size_t attn_workspace_bytes(const as_params* p) {
  size_t heads = (size_t)p->batch * p->n_q_heads;
  size_t ns = (size_t)attn_nsplit(p->budget);
  return heads * ns * (AS_HEAD_DIM + 2) * sizeof(float);
}

__device__ __forceinline__ float seg16_sum(float v) {
  v += __shfl_xor(v, 1);
  v += __shfl_xor(v, 2);
  v += __shfl_xor(v, 4);
  v += __shfl_xor(v, 8);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
  for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

template <int GH>
__global__ __launch_bounds__(256) void attn_split_kernel(
    const uint16_t* __restrict__ k_pool, const uint16_t* __restrict__ v_pool, const int32_t* __restrict__ block_table,
    const int32_t* __restrict__ ctx_lens, const uint16_t* __restrict__ q, const int32_t* __restrict__ sel_idx,
    const int32_t* __restrict__ sel_cnt, const int32_t* __restrict__ sel_ctx_lens, float* __restrict__ part_o,
    float* __restrict__ part_ml, int Hq, int Hkv, int G, int C, int max_pages, float sm_scale, int nsplit) {
  __shared__ float lg[GH][AT_CHUNK];        // logits, then probabilities
  __shared__ float sc_sh[GH];               // rescale factor of the running accumulator
  __shared__ float red[4][GH][AS_HEAD_DIM]; // per-wave partial outputs

  const int b = blockIdx.z;
  const int hblocks = G / GH;
  const int j = blockIdx.y / hblocks, hb = blockIdx.y % hblocks;
  const int h0 = j * G + hb * GH;
  const int split = blockIdx.x;
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int slot = lane >> 4, c = lane & 15;

  const int N = ctx_lens[b];
  int cnt = sel_cnt[b * Hkv + j];
  cnt = cnt < 0 ? 0 : (cnt > C ? C : cnt);
  int tail0 = sel_ctx_lens ? sel_ctx_lens[b] : N;
  tail0 = tail0 < 0 ? 0 : (tail0 > N ? N : tail0);
  const int L = cnt + (N - tail0);
  const int nchunks = (L + AT_CHUNK - 1) / AT_CHUNK;
  const int ck_begin = split;
  const int ck_end = (split == nsplit - 1) ? nchunks : (split + 1 < nchunks ? split + 1 : nchunks);

  const int64_t pbase = ((int64_t)b * Hq + h0) * nsplit + split;  // + g * nsplit per head
  if (ck_begin >= ck_end) {                                       // nothing here: mark empty
    if (tid < GH) {
      part_ml[(pbase + (int64_t)tid * nsplit) * 2 + 0] = -INFINITY;
      part_ml[(pbase + (int64_t)tid * nsplit) * 2 + 1] = 0.f;
    }
    return;
  }

  // the block's query heads, dims 8c..8c+7, as fp32
  float qf[GH][8];
#pragma unroll
  for (int g = 0; g < GH; ++g) {
    const uint4 u = *reinterpret_cast<const uint4*>(q + ((int64_t)b * Hq + h0 + g) * AS_HEAD_DIM + c * 8);
    qf[g][0] = bf16lo(u.x); qf[g][1] = bf16hi(u.x); qf[g][2] = bf16lo(u.y); qf[g][3] = bf16hi(u.y);
    qf[g][4] = bf16lo(u.z); qf[g][5] = bf16hi(u.z); qf[g][6] = bf16lo(u.w); qf[g][7] = bf16hi(u.w);
  }
  float acc[GH][8];
#pragma unroll
  for (int g = 0; g < GH; ++g)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
  // running softmax stats of head g live in wave (g & 3), slot g >> 2 (all lanes alike)
  float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};

  const int32_t* idx_row = sel_idx + ((int64_t)b * Hkv + j) * C;
  const int32_t* bt_row = block_table + (int64_t)b * max_pages;

#pragma unroll 1
  for (int ck = ck_begin; ck < ck_end; ++ck) {
    const int ti0 = ck * AT_CHUNK + w * 32 + slot;
    uint4 vreg[8];
    // ---- phase 1: logits of this wave's 32 tokens (8 loads x 4 rows) ----
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int ti = ti0 + it * 4;
      const bool valid = ti < L;
      int n = 0;
      if (valid) n = (ti < cnt) ? idx_row[ti] : tail0 + (ti - cnt);
      n = n < 0 ? 0 : (n >= N ? N - 1 : n);  // keeps a bad index inside the sequence's pages
      const int32_t page = bt_row[n >> 4];
      const int64_t off = chunk_offset(page, Hkv, j) + (int64_t)(n & 15) * AS_HEAD_DIM + c * 8;
      const uint4 ku = *reinterpret_cast<const uint4*>(k_pool + off);
      vreg[it] = *reinterpret_cast<const uint4*>(v_pool + off);
      float kf[8] = {bf16lo(ku.x), bf16hi(ku.x), bf16lo(ku.y), bf16hi(ku.y),
                     bf16lo(ku.z), bf16hi(ku.z), bf16lo(ku.w), bf16hi(ku.w)};
      float mine = 0.f;
#pragma unroll
      for (int g = 0; g < GH; ++g) {
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) s = fmaf(qf[g][e], kf[e], s);
        s = seg16_sum(s);
        if (c == g) mine = s;
      }
      if (c < GH) lg[c][w * 32 + it * 4 + slot] = valid ? mine * sm_scale : -INFINITY;
    }
    __syncthreads();
    // ---- phase 1b: chunk max, probabilities, running stats (wave w owns heads w, w+4) ----
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const int g = w + 4 * k;
      if (g < GH) {
        const float x0 = lg[g][lane], x1 = lg[g][lane + 64];
        const float mx = wave_max(fmaxf(x0, x1));
        const float m_new = fmaxf(m_run[k], mx);      // finite: the chunk holds >= 1 valid token
        const float scl = (m_run[k] == -INFINITY) ? 0.f : expf(m_run[k] - m_new);
        const float p0 = expf(x0 - m_new), p1 = expf(x1 - m_new);
        lg[g][lane] = p0;
        lg[g][lane + 64] = p1;
        const float ps = wave_sum(p0 + p1);
        l_run[k] = l_run[k] * scl + ps;
        m_run[k] = m_new;
        if (lane == 0) sc_sh[g] = scl;
      }
    }
    __syncthreads();
    // ---- phase 2: acc = acc * scale + sum_t p_t V_t ----
#pragma unroll
    for (int g = 0; g < GH; ++g) {
      const float scl = sc_sh[g];
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[g][e] *= scl;
    }
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const uint4 vu = vreg[it];
      float vf[8] = {bf16lo(vu.x), bf16hi(vu.x), bf16lo(vu.y), bf16hi(vu.y),
                     bf16lo(vu.z), bf16hi(vu.z), bf16lo(vu.w), bf16hi(vu.w)};
#pragma unroll
      for (int g = 0; g < GH; ++g) {
        const float pr = lg[g][w * 32 + it * 4 + slot];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] = fmaf(pr, vf[e], acc[g][e]);
      }
    }
    __syncthreads();
  }

  // ---- reduce the 4 slots of a wave, then the 4 waves ----
#pragma unroll
  for (int g = 0; g < GH; ++g)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float v = acc[g][e];
      v += __shfl_xor(v, 16);
      v += __shfl_xor(v, 32);
      if (slot == 0) red[w][g][c * 8 + e] = v;
    }
  __syncthreads();
  for (int i = tid; i < GH * AS_HEAD_DIM; i += 256) {
    const int g = i / AS_HEAD_DIM, d = i % AS_HEAD_DIM;
    const float v = red[0][g][d] + red[1][g][d] + red[2][g][d] + red[3][g][d];
    part_o[(pbase + (int64_t)g * nsplit) * AS_HEAD_DIM + d] = v;
  }
  if (lane == 0) {
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const int g = w + 4 * k;
      if (g < GH) {
        part_ml[(pbase + (int64_t)g * nsplit) * 2 + 0] = m_run[k];
        part_ml[(pbase + (int64_t)g * nsplit) * 2 + 1] = l_run[k];
      }
    }
  }
}

// merges the split partials of one (sequence, query head)
__global__ __launch_bounds__(AS_HEAD_DIM) void attn_combine_kernel(const float* __restrict__ part_o,
                                                                   const float* __restrict__ part_ml,
                                                                   uint16_t* __restrict__ out,
                                                                   float* __restrict__ lse, int nsplit) {
  const int64_t bh = blockIdx.x;
  const int d = threadIdx.x;
  const float* ml = part_ml + bh * nsplit * 2;
  float M = -INFINITY;
  for (int s = 0; s < nsplit; ++s)
    if (ml[2 * s + 1] > 0.f) M = fmaxf(M, ml[2 * s]);
  float Lsum = 0.f, o = 0.f;
  for (int s = 0; s < nsplit; ++s) {
    const float l = ml[2 * s + 1];
    if (l > 0.f) {
      const float wgt = expf(ml[2 * s] - M);
      Lsum += l * wgt;
      o += wgt * part_o[(bh * nsplit + s) * AS_HEAD_DIM + d];
    }
  }
  const float r = (Lsum > 0.f) ? o / Lsum : 0.f;
  out[bh * AS_HEAD_DIM + d] = (uint16_t)f32_to_bf16_rne(r);
  if (lse && d == 0) lse[bh] = (Lsum > 0.f) ? M + logf(Lsum) : -INFINITY;
}

template <int GH>
static hipError_t launch_attn_gh(const as_params* p, const as_kv_view* kv, const uint16_t* q, const int32_t* sel_idx,
                                 const int32_t* sel_cnt, const int32_t* sel_ctx_lens, float* part_o, float* part_ml,
                                 int nsplit, hipStream_t s) {
  const int G = p->n_q_heads / p->n_kv_heads;
  dim3 grid(nsplit, p->n_kv_heads * (G / GH), p->batch);
  hipLaunchKernelGGL(attn_split_kernel<GH>, grid, dim3(256), 0, s, reinterpret_cast<const uint16_t*>(kv->k_pool),
                     reinterpret_cast<const uint16_t*>(kv->v_pool), kv->block_table, kv->ctx_lens, q, sel_idx, sel_cnt,
                     sel_ctx_lens, part_o, part_ml, p->n_q_heads, p->n_kv_heads, G, p->budget, p->max_pages_per_seq,
                     p->sm_scale, nsplit);
  return hipGetLastError();
}

hipError_t launch_attn(const as_params* p, const as_kv_view* kv, const uint16_t* q, const int32_t* sel_idx,
                       const int32_t* sel_cnt, const int32_t* sel_ctx_lens, uint16_t* out, float* lse, void* ws,
                       hipStream_t s) {
  const int64_t heads = (int64_t)p->batch * p->n_q_heads;
  if (heads == 0) return hipSuccess;
  const int nsplit = attn_nsplit(p->budget);
  float* part_o = reinterpret_cast<float*>(ws);
  float* part_ml = part_o + heads * nsplit * AS_HEAD_DIM;
  const int G = p->n_q_heads / p->n_kv_heads;
  hipError_t e;
  switch (attn_gh(G)) {
    case 8: e = launch_attn_gh<8>(p, kv, q, sel_idx, sel_cnt, sel_ctx_lens, part_o, part_ml, nsplit, s); break;
    case 4: e = launch_attn_gh<4>(p, kv, q, sel_idx, sel_cnt, sel_ctx_lens, part_o, part_ml, nsplit, s); break;
    case 2: e = launch_attn_gh<2>(p, kv, q, sel_idx, sel_cnt, sel_ctx_lens, part_o, part_ml, nsplit, s); break;
    default: e = launch_attn_gh<1>(p, kv, q, sel_idx, sel_cnt, sel_ctx_lens, part_o, part_ml, nsplit, s); break;
  }
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(attn_combine_kernel, dim3((unsigned)heads), dim3(AS_HEAD_DIM), 0, s, part_o, part_ml, out, lse,
                     nsplit);
  return hipGetLastError();
}

}  // namespace asx
