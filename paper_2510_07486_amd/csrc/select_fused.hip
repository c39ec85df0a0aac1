// Fused key scoring + top-k for one layer-step (Alg. 1 step 7 followed by the cache rank's
// top-k, Sec. 4.3 items (1)-(2)), without ever writing the per-token scores to HBM.
//
// Each (sequence, KV head) row is cut into slices of at most 8192 tokens.  One 512-thread
// workgroup streams the slice's K pages (coalesced non-temporal 128-bit loads, transposed
// through a per-wave 4 KB LDS image into the MFMA operand layout, see score_common.hpp),
// keeps the 32-bit order-preserving keys of its scores in LDS (32 KB) and accumulates the first
// radix histogram while it streams.  It then radix-selects its local top-min(C, slice) in LDS
// and emits them in ascending token order: straight into sel_idx when the row has a single
// slice, otherwise as (key, index) candidates that a small merge kernel reduces to the row's
// top-C.  72 KB of LDS per workgroup lets two share a compute unit, so one workgroup's
// latency-bound phases (table and query fetch, radix select) hide behind the other's streaming.
// The global top-C is contained in the union of the per-slice top-C, and both levels
// resolve equal keys to the lowest index, so the result equals a full sort of the row.
// HBM traffic: one read of K, 8 B per candidate instead of 4 B per token.
#include "common.hpp"
#include "score_common.hpp"
#include "topk_common.hpp"

namespace asx {

// Two shapes of the slice workgroup: 512 threads / 8192 tokens / 72 KB LDS (two per compute
// unit) and 1024 threads / 16384 tokens / 144 KB (one per compute unit, half the candidates).
template <int THREADS> struct fs_shape {
  static constexpr int WAVES = THREADS / 64;
  static constexpr int SMAX = THREADS * 16;               // tokens per slice (keys: 4 B each)
  static constexpr int B0 = THREADS == 1024 ? 12 : 11;    // bits of the histogram built while streaming
  static constexpr int BINS = 1 << B0;
};
static constexpr int FS_MAX_SLICES = 8192;
static int g_fs_threads = 512;   // development knob
extern "C" void as_debug_set_slice_threads(int t) { g_fs_threads = (t == 1024) ? 1024 : 512; }

select_plan plan_select(const as_params* p) {
  select_plan pl;
  const int64_t rows = (int64_t)p->batch * p->n_kv_heads;
  const int64_t max_ctx = (int64_t)p->max_pages_per_seq * AS_PAGE;
  const int smax = g_fs_threads * 16;
  const int target_wgs = g_fs_threads == 1024 ? 512 : 1024;   // two rounds per compute unit
  int64_t st = rows > 0 ? (target_wgs + rows - 1) / rows : 1;
  if (st < 1) st = 1;
  int64_t sl = (max_ctx + st - 1) / st;
  sl = (sl + 63) / 64 * 64;
  if (sl < 256) sl = 256;
  if (sl > smax) sl = smax;
  pl.slice_len = (int)sl;
  pl.nslices = (int)((max_ctx + sl - 1) / sl);
  if (pl.nslices < 1) pl.nslices = 1;
  pl.ccap = p->budget < pl.slice_len ? p->budget : pl.slice_len;
  return pl;
}

size_t select_workspace_bytes(const as_params* p) {
  const select_plan pl = plan_select(p);
  if (pl.nslices == 1) return 0;
  const size_t rows = (size_t)p->batch * p->n_kv_heads;
  return rows * pl.nslices * ((size_t)pl.ccap * 8 + 4);
}

template <int NSET, int FS_THREADS>
__global__ __launch_bounds__(FS_THREADS) void select_slice_kernel(
    const uint16_t* __restrict__ k_pool, const int32_t* __restrict__ block_table,
    const int32_t* __restrict__ ctx_lens, const float* __restrict__ q_hat, int Hq, int Hkv, int G, int agg,
    int max_pages, int slice_len, int nslices, int C, int ccap, uint32_t* __restrict__ cand_key,
    int32_t* __restrict__ cand_idx, int32_t* __restrict__ cand_cnt, int32_t* __restrict__ sel_idx,
    int32_t* __restrict__ sel_cnt) {
  constexpr int FS_WAVES = fs_shape<FS_THREADS>::WAVES, FS_SMAX = fs_shape<FS_THREADS>::SMAX;
  constexpr int FS_B0 = fs_shape<FS_THREADS>::B0, FS_BINS = fs_shape<FS_THREADS>::BINS;
  __shared__ __attribute__((aligned(16))) uint32_t keys[FS_SMAX];
  __shared__ uint4 stage[FS_WAVES][256];  // per-wave page images; output staging after streaming
  __shared__ uint32_t hist[FS_BINS];
  __shared__ __attribute__((aligned(16))) uint32_t xch[TK_XCH];

  const int b = blockIdx.z, j = blockIdx.y, sl = blockIdx.x;
  const int64_t row = (int64_t)b * Hkv + j;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int t = lane & 15, grp = lane >> 4;
  const int N = ctx_lens[b];
  const int tok0 = sl * slice_len;
  int n_loc = N - tok0;
  n_loc = n_loc < 0 ? 0 : (n_loc > slice_len ? slice_len : n_loc);
  const bool final_out = (nslices == 1);
  if (n_loc == 0) {
    if (final_out) {
      for (int i = tid; i < C; i += FS_THREADS) sel_idx[row * C + i] = -1;
      if (tid == 0) sel_cnt[row] = 0;
    } else if (tid == 0) {
      cand_cnt[row * nslices + sl] = 0;
    }
    return;
  }
  for (int i = tid; i < FS_BINS; i += FS_THREADS) hist[i] = 0;

  // ---- stream the slice: wave w owns page quads w, w+8, ...; lane l keeps the page id of
  //      (iteration l>>2, page l&3), one table load per wave for the whole slice ----
  const int npages_loc = (n_loc + AS_PAGE - 1) / AS_PAGE;
  const int page0 = tok0 / AS_PAGE;
  int32_t my_page = 0;
  {
    const int lp = ((lane >> 2) * FS_WAVES + wave) * 4 + (lane & 3);
    if (lp < npages_loc) my_page = block_table[(int64_t)b * max_pages + page0 + lp];
  }
  bf16x8 aq[NSET][4];
  build_q_operand<NSET>(q_hat, b, j, Hq, G, agg, lane, aq);
  __syncthreads();

  uint4* st = stage[wave];
  const int nquads = (npages_loc + 3) / 4;
#pragma unroll 1
  for (int it = 0; wave + FS_WAVES * it < nquads; ++it) {
    const int q = wave + FS_WAVES * it;
    uint4 kb[4][4];
#pragma unroll
    for (int pg = 0; pg < 4; ++pg) {
      const int32_t page = __shfl(my_page, it * 4 + pg);
      const uint4* base = reinterpret_cast<const uint4*>(k_pool + chunk_offset(page, Hkv, j));
#pragma unroll
      for (int i = 0; i < 4; ++i) kb[pg][i] = ld16<true>(base + i * 64 + lane);
    }
    float res[4];
#pragma unroll
    for (int pg = 0; pg < 4; ++pg) {
#pragma unroll
      for (int i = 0; i < 4; ++i) st[lds_slot(4 * i + grp, t)] = kb[pg][i];
      __builtin_amdgcn_wave_barrier();
      uint4 kk[4];
#pragma unroll
      for (int m = 0; m < 4; ++m) kk[m] = st[lds_slot(t, cmap(grp, m))];
      __builtin_amdgcn_wave_barrier();
      float v = -INFINITY;
#pragma unroll
      for (int s = 0; s < NSET; ++s) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int m = 0; m < 4; ++m)
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aq[s][m], __builtin_bit_cast(bf16x8, kk[m]), acc, 0, 0, 0);
        v = fmaxf(v, fold_rows(acc));
      }
      res[pg] = group_max(v);
    }
    const float outv = grp == 0 ? res[0] : grp == 1 ? res[1] : grp == 2 ? res[2] : res[3];
    const int tl = (q * 4 + grp) * AS_PAGE + t;  // token within the slice
    if (tl < n_loc) {
      const uint32_t key = score_key(outv + 0.0f);
      keys[tl] = key;
      atomicAdd(&hist[key >> (32 - FS_B0)], 1u);
    }
  }
  __syncthreads();

  // ---- local top-min(C, n_loc), ascending token order; results are staged in LDS (the page
  //      images are dead by now) and written out with coalesced stores ----
  const int keep = n_loc < C ? n_loc : C;
  const int64_t cbase = (row * nslices + sl) * (int64_t)ccap;
  uint32_t* o_key = reinterpret_cast<uint32_t*>(&stage[0][0]);          // [FS_SMAX / 2]
  int32_t* o_idx = reinterpret_cast<int32_t*>(o_key + FS_SMAX / 2);      // [FS_SMAX / 2]
  const bool staged = final_out || keep <= FS_SMAX / 2;
  auto key4_of = [&](int i4, uint32_t (&k)[4], bool (&v)[4]) {
    const uint4 u = (i4 < n_loc) ? *reinterpret_cast<const uint4*>(&keys[i4]) : make_uint4(0, 0, 0, 0);
    k[0] = u.x; k[1] = u.y; k[2] = u.z; k[3] = u.w;
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = i4 + e < n_loc;
  };
  auto emit = [&](uint32_t pos, int i, uint32_t key) {
    if (final_out) {
      reinterpret_cast<int32_t*>(o_key)[pos] = tok0 + i;           // up to FS_SMAX indices
    } else if (staged) {
      o_key[pos] = key;
      o_idx[pos] = tok0 + i;
    } else {
      cand_key[cbase + pos] = key;
      cand_idx[cbase + pos] = tok0 + i;
    }
  };
  block_select<FS_THREADS, FS_B0>(n_loc, n_loc, keep, true, key4_of, emit, hist, xch);
  __syncthreads();
  if (final_out) {
    const int32_t* src = reinterpret_cast<const int32_t*>(o_key);
    for (int i = tid; i < C; i += FS_THREADS) sel_idx[row * C + i] = i < keep ? src[i] : -1;
    if (tid == 0) sel_cnt[row] = keep;
  } else {
    if (staged)
      for (int i = tid; i < keep; i += FS_THREADS) {
        cand_key[cbase + i] = o_key[i];
        cand_idx[cbase + i] = o_idx[i];
      }
    if (tid == 0) cand_cnt[row * nslices + sl] = keep;
  }
}

// Reduces a row's per-slice candidates (ascending token order within and across slices) to
// its top-C, again ascending and with ties to the lowest index.
__global__ __launch_bounds__(TK_THREADS) void select_merge_kernel(const uint32_t* __restrict__ cand_key,
                                                                  const int32_t* __restrict__ cand_idx,
                                                                  const int32_t* __restrict__ cand_cnt, int nslices,
                                                                  int ccap, int C, int32_t* __restrict__ sel_idx,
                                                                  int32_t* __restrict__ sel_cnt) {
  __shared__ int32_t cnt_sh[FS_MAX_SLICES];
  __shared__ uint32_t hist[TK_BINS];
  __shared__ __attribute__((aligned(16))) uint32_t xch[TK_XCH];
  __shared__ int total_sh;
  const int64_t row = blockIdx.x;
  const int tid = threadIdx.x;
  if (tid == 0) total_sh = 0;
  __syncthreads();
  int mine = 0;
  for (int s = tid; s < nslices; s += TK_THREADS) {
    const int c = cand_cnt[row * nslices + s];
    cnt_sh[s] = c;
    mine += c;
  }
  for (int o = 32; o >= 1; o >>= 1) mine += __shfl_xor(mine, o);
  if ((tid & 63) == 0 && mine) atomicAdd(&total_sh, mine);
  __syncthreads();
  const int total = total_sh;
  const int keep = total < C ? total : C;
  const int64_t cbase = row * nslices * (int64_t)ccap;
  auto key_of = [&](int v, bool& valid) -> uint32_t {
    valid = (v % ccap) < cnt_sh[v / ccap];
    return valid ? cand_key[cbase + v] : 0u;
  };
  auto emit = [&](uint32_t pos, int v, uint32_t) { sel_idx[row * C + pos] = cand_idx[cbase + v]; };
  if (keep > 0)
    block_select<TK_THREADS, 12>(nslices * ccap, total, keep, false, key4_from_scalar(nslices * ccap, key_of), emit, hist,
                                 xch);
  for (int i = keep + tid; i < C; i += TK_THREADS) sel_idx[row * C + i] = -1;
  if (tid == 0) sel_cnt[row] = keep;
}

hipError_t launch_select_fused(const as_params* p, const as_kv_view* kv, const float* q_hat, void* ws,
                               int32_t* sel_idx, int32_t* sel_cnt, hipStream_t s) {
  const int64_t rows = (int64_t)p->batch * p->n_kv_heads;
  if (rows == 0) return hipSuccess;
  const select_plan pl = plan_select(p);
  const int G = p->n_q_heads / p->n_kv_heads;
  uint32_t* cand_key = nullptr;
  int32_t *cand_idx = nullptr, *cand_cnt = nullptr;
  if (pl.nslices > 1) {
    const size_t n = (size_t)rows * pl.nslices * pl.ccap;
    cand_key = reinterpret_cast<uint32_t*>(ws);
    cand_idx = reinterpret_cast<int32_t*>(cand_key + n);
    cand_cnt = cand_idx + n;
  }
  dim3 grid(pl.nslices, p->n_kv_heads, p->batch);
  const bool two = (p->agg != AS_AGG_SUM) && G > 8;
  const uint16_t* kp = reinterpret_cast<const uint16_t*>(kv->k_pool);
#define AS_SLICE_LAUNCH(NSET_, THR_)                                                                            \
  hipLaunchKernelGGL((select_slice_kernel<NSET_, THR_>), grid, dim3(THR_), 0, s, kp, kv->block_table, kv->ctx_lens, \
                     q_hat, p->n_q_heads, p->n_kv_heads, G, p->agg, p->max_pages_per_seq, pl.slice_len, pl.nslices, \
                     p->budget, pl.ccap, cand_key, cand_idx, cand_cnt, sel_idx, sel_cnt)
  if (g_fs_threads == 1024) {
    if (two) AS_SLICE_LAUNCH(2, 1024); else AS_SLICE_LAUNCH(1, 1024);
  } else {
    if (two) AS_SLICE_LAUNCH(2, 512); else AS_SLICE_LAUNCH(1, 512);
  }
#undef AS_SLICE_LAUNCH
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || pl.nslices == 1) return e;
  hipLaunchKernelGGL(select_merge_kernel, dim3((unsigned)rows), dim3(TK_THREADS), 0, s, cand_key, cand_idx, cand_cnt,
                     pl.nslices, pl.ccap, p->budget, sel_idx, sel_cnt);
  return hipGetLastError();
}

}  // namespace asx
