// Sparse decode attention with the real query over the selected tokens (Sec. 4.1; the
// 4*q*h*C term of Appendix B), plus an optional dense tail of tokens appended after the
// selection was made.
//
// HBM-bound on the index-gathered K and V rows (2 x 256 B per selected token and KV head).
// Split-C: a 256-thread workgroup owns a split (a few hundred tokens, chosen so that about six
// workgroups per compute unit exist) of the logical token list of one (sequence, KV head) and up
// to 8 of the group's query heads, so every gathered row is read once for the whole group; it
// walks the split in 64-token inner chunks with an online softmax across chunks.  The dependent
// chain index -> page id -> row address is resolved for four chunks at a time with one lane per
// token, speculatively and one step ahead, so it is off the critical path; a 16-lane row of the
// wavefront reads one 256-byte K / V row with non-temporal 128-bit loads.  Q.K uses
// v_dot2c_f32_bf16 and a DPP rotate all-reduce inside the row; logits go to LDS, the chunk max and
// p = exp(l - m) follow, then P.V with no rescaling inside the chunk.  Each workgroup writes its
// partial (m, l, o); a small second kernel merges them and writes bf16.  (Measured and rejected: a
// barrier-free variant with one online softmax per 16-lane row, 40 % slower from register
// pressure; a "last workgroup merges" variant, 8x slower from device-scope fences.)
#include "common.hpp"

namespace asx {

static constexpr int AT_SPLIT = AS_ATTN_CHUNK;  // smallest workgroup split, tokens (sizes the workspace)
static constexpr int AT_IT = 4;                 // row loads per lane and inner chunk (K and V each)
static constexpr int AT_CHUNK = 4 * AT_IT * 4;  // inner chunk: 4 waves x AT_IT loads x 4 rows = 64 tokens

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__host__ __device__ inline int attn_nsplit(int C) { return (C + AT_SPLIT - 1) / AT_SPLIT + 1; }
static inline int attn_gh(int G) { return (G % 8 == 0) ? 8 : (G % 4 == 0) ? 4 : (G % 2 == 0) ? 2 : 1; }

static int g_attn_impl = 0;  // 0: matrix-core kernel (attn_mfma.hip), 1: vector-ALU kernel below
static int g_attn_splits = 0; // development knob: > 0 forces the number of splits per (sequence, KV head)

// Split geometry for a logical token list of at most `list_len` tokens per (sequence, KV head).  Measured on the
// matrix-core kernel (32/8 and 64/8 heads, budgets 1024-4096): what counts is that all workgroups are resident at
// once (three fit a compute unit: at most 768; a second, partly filled round costs 5-10 %) and that the four
// wavefronts of a workgroup get the same number of 32-token steps; 512 workgroups of 1024 tokens beat 1536 of 256-341
// by 6-9 %.  So: the largest split count that keeps the grid within one round, preferably one that divides the
// list into multiples of 128 tokens; never below AT_SPLIT tokens per split.  One extra split at the end takes
// whatever lies beyond list_len (the dense tail of a sparse call under the vector-ALU kernel).
struct attn_geom { int nsplit, split_tokens, nsel; };
static attn_geom attn_geometry(const as_params* p, int64_t list_len, int impl) {
  const int G = p->n_q_heads / p->n_kv_heads;
  if (list_len < 1) list_len = 1;
  int64_t pairs = (int64_t)p->batch * p->n_kv_heads * (impl == 0 ? (G + 15) / 16 : G / attn_gh(G));
  if (pairs < 1) pairs = 1;
  int64_t nsel = 768 / pairs;
  const int64_t max_sel = (list_len + AT_SPLIT - 1) / AT_SPLIT;
  if (nsel > max_sel) nsel = max_sel;
  if (nsel < 1) nsel = 1;
  const int64_t units = list_len / 128;           // a split of whole units gives every wavefront the same steps
  for (int64_t d = nsel; d >= 1 && d * pairs >= 384; --d)
    if (units > 0 && units % d == 0 && list_len % 128 == 0) {
      nsel = d;
      break;
    }
  if (g_attn_splits > 0) nsel = g_attn_splits < max_sel ? g_attn_splits : max_sel;
  int64_t split_tokens = (list_len + nsel - 1) / nsel;
  split_tokens = (split_tokens + AT_CHUNK - 1) / AT_CHUNK * AT_CHUNK;
  if (split_tokens < AT_SPLIT) split_tokens = AT_SPLIT;
  attn_geom g;
  g.split_tokens = (int)split_tokens;
  g.nsplit = (int)((list_len + split_tokens - 1) / split_tokens) + 1;
  g.nsel = (int)nsel;
  return g;
}

// partial outputs and partial (m, l) pairs, for the sparse call (list = budget) and the dense one
// (list = longest context the block table allows), under either kernel
size_t attn_workspace_bytes(const as_params* p) {
  const size_t heads = (size_t)p->batch * p->n_q_heads;
  size_t ns = (size_t)attn_nsplit(p->budget);
  for (int impl = 0; impl < 2; ++impl) {   // the matrix-core kernel runs nsel splits, the vector-ALU one nsplit
    const attn_geom gd = attn_geometry(p, (int64_t)p->max_pages_per_seq * AS_PAGE, impl);
    const size_t nd = (size_t)(gd.nsplit > gd.nsel ? gd.nsplit : gd.nsel);
    if (nd > ns) ns = nd;
  }
  return heads * ns * (AS_HEAD_DIM + 2) * sizeof(float);
}

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), c, false);
}
// sum over the 16 lanes of a DPP row, result in every lane (rotations by 8, 4, 2, 1)
__device__ __forceinline__ float row16_allsum(float x) {
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x128, 0xf, 0xf, false));
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x124, 0xf, 0xf, false));
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x122, 0xf, 0xf, false));
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x121, 0xf, 0xf, false));
  return x;
}
__device__ __forceinline__ float wave_max(float v) {
  for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
__device__ __forceinline__ uint4 ld16_nt(const void* p) {
  const u32x4_t r = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(r.x, r.y, r.z, r.w);
}

template <int GH>
__global__ __launch_bounds__(256) void attn_split_kernel(
    const uint16_t* __restrict__ k_pool, const uint16_t* __restrict__ v_pool, const int32_t* __restrict__ block_table,
    const int32_t* __restrict__ ctx_lens, const uint16_t* __restrict__ q, const int32_t* __restrict__ sel_idx,
    const int32_t* __restrict__ sel_cnt, const int32_t* __restrict__ sel_ctx_lens, float* __restrict__ part_o,
    float* __restrict__ part_ml, int Hq, int Hkv, int G, int C, int max_pages, float sm_scale, int nsplit,
    int cps /* inner chunks per split */, int32_t last_page) {
  __shared__ float lg[GH][AT_CHUNK];         // logits, then probabilities
  __shared__ float sc_sh[GH];                // rescale factor of the running accumulator
  __shared__ float red[4][GH][AS_HEAD_DIM];  // per-wave partial outputs

  const int b = blockIdx.z;
  const int hblocks = G / GH;
  const int j = blockIdx.y / hblocks, hb = blockIdx.y % hblocks;
  const int h0 = j * G + hb * GH;
  const int split = blockIdx.x;
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int slot = lane >> 4, c = lane & 15;

  const int32_t* idx_row = sel_idx + ((int64_t)b * Hkv + j) * C;
  // lane l resolves token (l & 15) of this wave's share of inner chunk (first + (l >> 4)): four chunks at once
  auto fetch_index = [&](int ck_first) -> int {
    const int ti = (ck_first + (lane >> 4)) * AT_CHUNK + w * (AT_IT * 4) + (lane & 15);
    return (ti < C) ? idx_row[ti] : 0;
  };
  const int raw_first = fetch_index(split * cps);  // speculative: validated once the lengths are known

  const int N = clamp_ctx(ctx_lens[b], max_pages);
  int cnt = sel_cnt ? sel_cnt[b * Hkv + j] : 0;   // no selection arrays: dense attention over [0, N)
  cnt = (cnt < 0 || N == 0) ? 0 : (cnt > C ? C : cnt);   // an empty sequence has nothing to select from
  int tail0 = sel_idx ? (sel_ctx_lens ? sel_ctx_lens[b] : N) : 0;
  tail0 = tail0 < 0 ? 0 : (tail0 > N ? N : tail0);
  const int L = cnt + (N - tail0);
  const int nchunks = (L + AT_CHUNK - 1) / AT_CHUNK;
  const int ck_begin = split * cps;
  const int ck_end = (split == nsplit - 1) ? nchunks : ((split + 1) * cps < nchunks ? (split + 1) * cps : nchunks);

  const int64_t pbase = ((int64_t)b * Hq + h0) * nsplit + split;  // + g * nsplit per head
  if (ck_begin >= ck_end) {                                       // nothing here: mark empty
    if (tid < GH) {
      part_ml[(pbase + (int64_t)tid * nsplit) * 2 + 0] = -INFINITY;
      part_ml[(pbase + (int64_t)tid * nsplit) * 2 + 1] = 0.f;
    }
  } else {
    // the block's query heads, dims 8c..8c+7, as packed bf16 pairs
    uint32_t qp[GH][4];
#pragma unroll
    for (int g = 0; g < GH; ++g) {
      const uint4 u = *reinterpret_cast<const uint4*>(q + ((int64_t)b * Hq + h0 + g) * AS_HEAD_DIM + c * 8);
      qp[g][0] = u.x; qp[g][1] = u.y; qp[g][2] = u.z; qp[g][3] = u.w;
    }
    float acc[GH][8];
#pragma unroll
    for (int g = 0; g < GH; ++g)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
    // running softmax stats of head g live in wave (g & 3), slot g >> 2 (all lanes alike)
    float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};

    const int32_t* bt_row = block_table + (int64_t)b * max_pages;

    // Addresses of four inner chunks are resolved together, one lane per token.  The index load does
    // not wait for the lengths (any slot below C is readable; it is validated afterwards) and the
    // next four chunks are resolved while the current ones are processed, so after the first chunk
    // the chain index -> page id -> row address is off the critical path.
    auto page_of = [&](int ck_first, int raw) -> uint32_t {
      const int ti = (ck_first + (lane >> 4)) * AT_CHUNK + w * (AT_IT * 4) + (lane & 15);
      int n = 0;
      if (ti < L) n = (ti < cnt) ? raw : tail0 + (ti - cnt);
      n = n < 0 ? 0 : (n >= N ? N - 1 : n);  // keeps a bad index inside the sequence's pages
      int32_t pg = bt_row[n >> 4];
      pg = pg < 0 ? 0 : (pg > last_page ? last_page : pg);           // a corrupt table must not leave the pool
      return ((uint32_t)pg << 4) | (uint32_t)(n & 15);              // page id << 4 | slot in page
    };
    uint32_t my_pk = page_of(ck_begin, raw_first);
#pragma unroll 1
    for (int ck0 = ck_begin; ck0 < ck_end; ck0 += 4) {
      const bool more = ck0 + 4 < ck_end;
      int raw_next = 0;
      if (more) raw_next = fetch_index(ck0 + 4);
      uint32_t pk_next = 0;
#pragma unroll 1
      for (int cc = 0; cc < 4; ++cc) {
      const int ck = ck0 + cc;
      if (ck >= ck_end) break;
      if (cc == 1 && more) pk_next = page_of(ck0 + 4, raw_next);
      const int tw0 = ck * AT_CHUNK + w * (AT_IT * 4);
      // ---- all row loads of this lane (AT_IT K, AT_IT V) ----
      uint4 kreg[AT_IT], vreg[AT_IT];
#pragma unroll
      for (int it = 0; it < AT_IT; ++it) {
        const uint32_t pk = __shfl(my_pk, cc * 16 + it * 4 + slot);
        const int64_t off = chunk_offset((int32_t)(pk >> 4), Hkv, j) + (int64_t)(pk & 15) * AS_HEAD_DIM + c * 8;
        kreg[it] = ld16_nt(k_pool + off);
        vreg[it] = ld16_nt(v_pool + off);
      }
      // ---- phase 1: logits ----
#pragma unroll
      for (int it = 0; it < AT_IT; ++it) {
        const bool valid = tw0 + it * 4 + slot < L;
        float mine = 0.f;
#pragma unroll
        for (int g = 0; g < GH; ++g) {
          float s = dot2_bf16(qp[g][0], kreg[it].x, 0.f);
          s = dot2_bf16(qp[g][1], kreg[it].y, s);
          s = dot2_bf16(qp[g][2], kreg[it].z, s);
          s = dot2_bf16(qp[g][3], kreg[it].w, s);
          s = row16_allsum(s);
          if (c == g) mine = s;
        }
        if (c < GH) lg[c][w * (AT_IT * 4) + it * 4 + slot] = valid ? mine * sm_scale : -INFINITY;
      }
      __syncthreads();
      // ---- phase 1b: chunk max, probabilities, running stats (wave w owns heads w, w+4) ----
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        const int g = w + 4 * k;
        if (g < GH) {
          const float x0 = lg[g][lane];
          const float mx = wave_max(x0);
          const float m_new = fmaxf(m_run[k], mx);  // finite: the chunk holds >= 1 valid token
          const float scl = (m_run[k] == -INFINITY) ? 0.f : expf(m_run[k] - m_new);
          const float p0 = expf(x0 - m_new);
          lg[g][lane] = p0;
          const float ps = wave_sum(p0);
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
      for (int it = 0; it < AT_IT; ++it) {
        const uint4 vu = vreg[it];
        float vf[8] = {bf16lo(vu.x), bf16hi(vu.x), bf16lo(vu.y), bf16hi(vu.y),
                       bf16lo(vu.z), bf16hi(vu.z), bf16lo(vu.w), bf16hi(vu.w)};
#pragma unroll
        for (int g = 0; g < GH; ++g) {
          const float pr = lg[g][w * (AT_IT * 4) + it * 4 + slot];
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[g][e] = fmaf(pr, vf[e], acc[g][e]);
        }
      }
      __syncthreads();
      }
      my_pk = pk_next;
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

}

// merges the split partials of one (sequence, query head).  A separate launch on purpose: a
// "last workgroup merges" scheme needs device-scope fences, which write back and invalidate
// the whole per-XCD L2 on this chip and cost several times the kernel itself.
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

template <int GH>
static hipError_t launch_attn_gh(const as_params* p, const as_kv_view* kv, const uint16_t* q, const int32_t* sel_idx,
                                 const int32_t* sel_cnt, const int32_t* sel_ctx_lens, float* part_o, float* part_ml,
                                 int nsplit, int cps, hipStream_t s) {
  const int G = p->n_q_heads / p->n_kv_heads;
  dim3 grid(nsplit, p->n_kv_heads * (G / GH), p->batch);
  hipLaunchKernelGGL(attn_split_kernel<GH>, grid, dim3(256), 0, s, reinterpret_cast<const uint16_t*>(kv->k_pool),
                     reinterpret_cast<const uint16_t*>(kv->v_pool), kv->block_table, kv->ctx_lens, q, sel_idx, sel_cnt,
                     sel_ctx_lens, part_o, part_ml, p->n_q_heads, p->n_kv_heads, G, sel_idx ? p->budget : 0,
                     p->max_pages_per_seq,
                     p->sm_scale, nsplit, cps, (int32_t)(kv->num_pages > 0 ? kv->num_pages - 1 : 0));
  return hipGetLastError();
}

hipError_t launch_attn_mfma(const as_params* p, const as_kv_view* kv, const uint16_t* q, const int32_t* sel_idx,
                            const int32_t* sel_cnt, const int32_t* sel_ctx_lens, float* part_o, float* part_ml,
                            int nsplit, int list_len, hipStream_t s);

extern "C" void as_debug_set_attn_impl(int v) { g_attn_impl = v; }   // development knob
// development knob for split-count sweeps; set it before the context is created (the workspace is sized from it)
extern "C" void as_debug_set_attn_splits(int n) { g_attn_splits = n > 0 ? n : 0; }

// sel_idx == nullptr: dense attention over [0, ctx_lens[b]) (the token list is only the "tail", from 0)
hipError_t launch_attn(const as_params* p, const as_kv_view* kv, const uint16_t* q, const int32_t* sel_idx,
                       const int32_t* sel_cnt, const int32_t* sel_ctx_lens, uint16_t* out, float* lse, void* ws,
                       hipStream_t s) {
  const int64_t heads = (int64_t)p->batch * p->n_q_heads;
  if (heads == 0) return hipSuccess;
  const int G = p->n_q_heads / p->n_kv_heads;
  const bool dense = sel_idx == nullptr;
  const int64_t list_len = dense ? (int64_t)p->max_pages_per_seq * AS_PAGE : (int64_t)p->budget;
  const int impl = g_attn_impl;
  const attn_geom gm = attn_geometry(p, list_len, impl);
  // The matrix-core kernel cuts the list into equal splits (no separate tail split); the vector-ALU
  // kernel walks whole 64-token chunks and keeps one extra split for the tail.
  const int nsplit = impl == 0 ? gm.nsel : gm.nsplit;
  const int split_tokens = gm.split_tokens;
  const int cps = split_tokens / AT_CHUNK;
  float* part_o = reinterpret_cast<float*>(ws);
  float* part_ml = part_o + heads * nsplit * AS_HEAD_DIM;
  hipError_t e;
  if (impl == 0) {
    e = launch_attn_mfma(p, kv, q, sel_idx, sel_cnt, sel_ctx_lens, part_o, part_ml, nsplit, (int)list_len, s);
  } else {
    switch (attn_gh(G)) {
      case 8: e = launch_attn_gh<8>(p, kv, q, sel_idx, sel_cnt, sel_ctx_lens, part_o, part_ml, nsplit, cps, s); break;
      case 4: e = launch_attn_gh<4>(p, kv, q, sel_idx, sel_cnt, sel_ctx_lens, part_o, part_ml, nsplit, cps, s); break;
      case 2: e = launch_attn_gh<2>(p, kv, q, sel_idx, sel_cnt, sel_ctx_lens, part_o, part_ml, nsplit, cps, s); break;
      default: e = launch_attn_gh<1>(p, kv, q, sel_idx, sel_cnt, sel_ctx_lens, part_o, part_ml, nsplit, cps, s); break;
    }
  }
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(attn_combine_kernel, dim3((unsigned)heads), dim3(AS_HEAD_DIM), 0, s, part_o, part_ml, out, lse,
                     nsplit);
  return hipGetLastError();
}

}  // namespace asx
