// Cache-side bookkeeping around the selection kernels: the per-step state update of the cache
// rank (Sec. 4.1 workflow: append the step's K/V to the cache, enqueue its query to the sliding
// window), the KV re-organisation of the filtered tokens (Sec. 4.3, cache-rank item (3)) and the
// overlap ratio of two selections (Sec. 3, Eq. 1).  All of it is data movement or integer set
// arithmetic: 128-bit coalesced copies, one 16-lane row per 256-byte K or V row.
#include "common.hpp"

namespace asx {

typedef uint32_t u32x4_c __attribute__((ext_vector_type(4)));

// ---- KV append -----------------------------------------------------------------------------
// One workgroup per sequence; 16 lanes copy one 256-byte row, so 256 threads move the K and V
// rows of 8 KV heads per pass.  The length is read once, before any thread of the workgroup can
// have bumped it.
__global__ __launch_bounds__(256) void kv_append_kernel(uint16_t* __restrict__ k_pool, uint16_t* __restrict__ v_pool,
                                                        const int32_t* __restrict__ block_table,
                                                        int32_t* __restrict__ ctx_lens,
                                                        const uint16_t* __restrict__ k_new,
                                                        const uint16_t* __restrict__ v_new, int Hkv, int max_pages,
                                                        int32_t last_page) {
  const int b = blockIdx.x, tid = threadIdx.x;
  const int n = ctx_lens[b];
  __syncthreads();
  if (n < 0 || n >= max_pages * AS_PAGE) return;      // no room (or a corrupt length): leave the sequence alone
  int32_t pg = block_table[(int64_t)b * max_pages + (n >> 4)];
  pg = clamp_page(pg, last_page);
  const int c = tid & 15;
  for (int r = tid >> 4; r < 2 * Hkv; r += 16) {      // rows: K of head r / 2 when r is even, V when odd
    const int j = r >> 1;
    const uint16_t* src = ((r & 1) ? v_new : k_new) + ((int64_t)b * Hkv + j) * AS_HEAD_DIM + c * 8;
    uint16_t* dst = ((r & 1) ? v_pool : k_pool) + chunk_offset(pg, Hkv, j) + (int64_t)(n & 15) * AS_HEAD_DIM + c * 8;
    *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
  }
  if (tid == 0) ctx_lens[b] = n + 1;
}

// ---- window push ---------------------------------------------------------------------------
// One wavefront per (sequence, query head); a lane owns the same two dims of every row, so the
// in-place shift has no cross-lane hazard: rows are read eight at a time, then written one slot
// down.
__global__ __launch_bounds__(64) void window_push_kernel(uint16_t* __restrict__ q_win, uint16_t* __restrict__ q_cur,
                                                         const uint16_t* __restrict__ q_new, int W) {
  const int64_t bh = blockIdx.x;
  const int lane = threadIdx.x;
  uint32_t* win = reinterpret_cast<uint32_t*>(q_win + bh * (int64_t)W * AS_HEAD_DIM) + lane;
  uint32_t* cur = reinterpret_cast<uint32_t*>(q_cur + bh * (int64_t)AS_HEAD_DIM) + lane;
  const uint32_t* nw = reinterpret_cast<const uint32_t*>(q_new + bh * (int64_t)AS_HEAD_DIM) + lane;
  constexpr int RW = AS_HEAD_DIM / 2;   // dwords per row
  for (int i0 = 0; i0 + 1 < W; i0 += 8) {
    uint32_t r[8];
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (i0 + e + 1 < W) r[e] = win[(int64_t)(i0 + e + 1) * RW];
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (i0 + e + 1 < W) win[(int64_t)(i0 + e) * RW] = r[e];
  }
  const uint32_t c = *cur, n = *nw;
  win[(int64_t)(W - 1) * RW] = c;
  *cur = n;
}

// ---- KV re-organisation of the filtered tokens ---------------------------------------------
// Grid (token chunk of 64, KV head, sequence).  16 lanes copy one K row and one V row (random
// 256-byte gathers, non-temporal) into the compact paged pool: token i of (b, j) goes to page
// b * Cp + i / 16, slot i % 16, so 16 consecutive tokens fill one contiguous 4 KB chunk.
__global__ __launch_bounds__(256) void gather_kv_kernel(
    const uint16_t* __restrict__ k_pool, const uint16_t* __restrict__ v_pool, const int32_t* __restrict__ block_table,
    const int32_t* __restrict__ ctx_lens, const int32_t* __restrict__ sel_idx, const int32_t* __restrict__ sel_cnt,
    uint16_t* __restrict__ k_out, uint16_t* __restrict__ v_out, int32_t* __restrict__ out_table,
    int32_t* __restrict__ out_lens, int Hkv, int C, int Cp, int max_pages, int32_t last_page) {
  const int b = blockIdx.z, j = blockIdx.y, tid = threadIdx.x;
  const int64_t row = (int64_t)b * Hkv + j;
  const int N = clamp_ctx(ctx_lens[b], max_pages);
  int cnt = sel_cnt[row];
  cnt = clamp_count(cnt, C, N);   // an empty sequence has nothing to select from
  if (blockIdx.x == 0 && j == 0) {
    for (int i = tid; i < Cp; i += 256) out_table[(int64_t)b * Cp + i] = b * Cp + i;
    if (tid == 0) out_lens[b] = cnt;
  }
  if (blockIdx.x * 64 >= cnt) return;    // nothing selected in this workgroup's range (cnt > 0 below, hence N > 0)
  const int c = tid & 15;
  const int i0 = blockIdx.x * 64 + (tid >> 4);
  // Three dependent rounds (index, page id, row), each with all of its loads in flight together: slots beyond the
  // count re-read the row's first index instead of sitting in a branch with a wait of its own, and are masked
  // at the store.
  int n[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int i = i0 + 16 * e;
    const int v = sel_idx[row * C + (i < cnt ? i : 0)];
    n[e] = clamp_token(v, N);      // a bad index stays inside the sequence
  }
  int32_t pg[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) pg[e] = block_table[(int64_t)b * max_pages + (n[e] >> 4)];
  uint4 kr[4], vr[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int32_t p = clamp_page(pg[e], last_page);
    const int64_t off = chunk_offset(p, Hkv, j) + (int64_t)(n[e] & 15) * AS_HEAD_DIM + c * 8;
    const u32x4_c a = __builtin_nontemporal_load(reinterpret_cast<const u32x4_c*>(k_pool + off));
    const u32x4_c d = __builtin_nontemporal_load(reinterpret_cast<const u32x4_c*>(v_pool + off));
    kr[e] = make_uint4(a.x, a.y, a.z, a.w);
    vr[e] = make_uint4(d.x, d.y, d.z, d.w);
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int i = i0 + 16 * e;
    if (i < cnt) {
      const int64_t off = chunk_offset(b * Cp + (i >> 4), Hkv, j) + (int64_t)(i & 15) * AS_HEAD_DIM + c * 8;
      *reinterpret_cast<uint4*>(k_out + off) = kr[e];
      *reinterpret_cast<uint4*>(v_out + off) = vr[e];
    }
  }
}

// ---- overlap ratio -------------------------------------------------------------------------
// One workgroup per (sequence, KV head).  Both lists are ascending (the selection kernels emit
// them so): every element of A is looked up in B by binary search, hits are counted with a
// wavefront ballot and one LDS atomic per wave.
__global__ __launch_bounds__(256) void overlap_kernel(const int32_t* __restrict__ idx_a,
                                                      const int32_t* __restrict__ cnt_a,
                                                      const int32_t* __restrict__ idx_b,
                                                      const int32_t* __restrict__ cnt_b, int C,
                                                      int32_t* __restrict__ inter, float* __restrict__ ratio) {
  __shared__ int total;
  const int64_t row = blockIdx.x;
  const int tid = threadIdx.x;
  if (tid == 0) total = 0;
  __syncthreads();
  int na = cnt_a[row], nb = cnt_b[row];
  na = na < 0 ? 0 : (na > C ? C : na);
  nb = nb < 0 ? 0 : (nb > C ? C : nb);
  const int32_t* a = idx_a + row * C;
  const int32_t* bb = idx_b + row * C;
  int mine = 0;
  for (int i = tid; i < na; i += 256) {
    const int32_t key = a[i];
    int lo = 0, hi = nb;          // first position with bb[pos] >= key
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (bb[mid] < key) lo = mid + 1; else hi = mid;
    }
    mine += (lo < nb && bb[lo] == key) ? 1 : 0;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mine += __shfl_xor(mine, o);
  if ((tid & 63) == 0 && mine) atomicAdd(&total, mine);
  __syncthreads();
  if (tid == 0) {
    const int den = na > nb ? na : nb;
    inter[row] = total;
    if (ratio) ratio[row] = den > 0 ? (float)total / (float)den : 0.f;
  }
}

// ---- launchers -----------------------------------------------------------------------------
hipError_t launch_kv_append(const as_params* p, uint16_t* k_pool, uint16_t* v_pool, const int32_t* block_table,
                            int32_t* ctx_lens, int64_t num_pages, const uint16_t* k_new, const uint16_t* v_new,
                            hipStream_t s) {
  if (p->batch == 0) return hipSuccess;
  hipLaunchKernelGGL(kv_append_kernel, dim3(p->batch), dim3(256), 0, s, k_pool, v_pool, block_table, ctx_lens, k_new,
                     v_new, p->n_kv_heads, p->max_pages_per_seq, (int32_t)(num_pages - 1));
  return hipGetLastError();
}

hipError_t launch_window_push(const as_params* p, uint16_t* q_win, uint16_t* q_cur, const uint16_t* q_new,
                              hipStream_t s) {
  const int64_t heads = (int64_t)p->batch * p->n_q_heads;
  if (heads == 0) return hipSuccess;
  hipLaunchKernelGGL(window_push_kernel, dim3((unsigned)heads), dim3(64), 0, s, q_win, q_cur, q_new, p->window);
  return hipGetLastError();
}

hipError_t launch_gather_kv(const as_params* p, const as_kv_view* kv, const int32_t* sel_idx, const int32_t* sel_cnt,
                            uint16_t* k_out, uint16_t* v_out, int32_t* out_table, int32_t* out_lens, hipStream_t s) {
  if (p->batch == 0) return hipSuccess;
  const int Cp = (p->budget + AS_PAGE - 1) / AS_PAGE;
  dim3 grid((p->budget + 63) / 64, p->n_kv_heads, p->batch);
  hipLaunchKernelGGL(gather_kv_kernel, grid, dim3(256), 0, s, reinterpret_cast<const uint16_t*>(kv->k_pool),
                     reinterpret_cast<const uint16_t*>(kv->v_pool), kv->block_table, kv->ctx_lens, sel_idx, sel_cnt,
                     k_out, v_out, out_table, out_lens, p->n_kv_heads, p->budget, Cp, p->max_pages_per_seq,
                     (int32_t)(kv->num_pages - 1));
  return hipGetLastError();
}

hipError_t launch_overlap(const as_params* p, const int32_t* idx_a, const int32_t* cnt_a, const int32_t* idx_b,
                          const int32_t* cnt_b, int32_t* inter, float* ratio, hipStream_t s) {
  const int64_t rows = (int64_t)p->batch * p->n_kv_heads;
  if (rows == 0) return hipSuccess;
  hipLaunchKernelGGL(overlap_kernel, dim3((unsigned)rows), dim3(256), 0, s, idx_a, cnt_a, idx_b, cnt_b, p->budget,
                     inter, ratio);
  return hipGetLastError();
}

}  // namespace asx
