// Key scoring (Alg. 1 step 7; batched-matmul shapes of Sec. 4.3):
//   scores[b][j][n] = agg_g <q_hat[b][j*G+g], K[b][j][n]>,  n < ctx_lens[b].
//
// HBM-bound: one full read of the K cache (256 B per token and KV head), 4 B written.
// The contraction runs on the matrix cores so the vector ALUs stay idle whatever the
// group size: per 16-token page, D[16 x 16] = Q[16 x 128] * K_page^T[128 x 16] as four
// v_mfma_f32_16x16x32_bf16.  The 16 rows of Q are the group's predicted queries split
// into bf16 hi + lo parts (q = hi + lo to 2^-17 relative, products exact, fp32
// accumulate), laid out so that a lane's four accumulators are (hi, hi', lo, lo') of two
// heads: head sums and the group max then need two adds, one max and two cross-lane maxes.
// Unused rows repeat heads (harmless under max); AS_AGG_SUM scores the summed query.
#include "common.hpp"
#include "score_common.hpp"

namespace asx {

// Variant 0: K is read from global memory directly in the MFMA B layout (lane = token,
// 64 contiguous bytes per lane across the four steps).
template <int NSET, bool NT>
__global__ __launch_bounds__(256) void score_mfma_direct(const uint16_t* __restrict__ k_pool,
                                                         const int32_t* __restrict__ block_table,
                                                         const int32_t* __restrict__ ctx_lens,
                                                         const float* __restrict__ q_hat, float* __restrict__ scores,
                                                         int64_t stride, int Hq, int Hkv, int G, int agg,
                                                         int max_pages, int32_t last_page, int ppw) {
  const int b = blockIdx.z, j = blockIdx.y;
  const int N = clamp_ctx(ctx_lens[b], max_pages);
  const int npages = (N + AS_PAGE - 1) / AS_PAGE;
  const int p0 = blockIdx.x * (4 * ppw);
  if (p0 >= npages) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int t = lane & 15, grp = lane >> 4;
  const int pw = p0 + wave * ppw;  // first page of this wave
  if (pw >= npages) return;

  int32_t my_page = 0;
  if (lane < ppw && pw + lane < npages) my_page = block_table[(int64_t)b * max_pages + pw + lane];
  my_page = my_page < 0 ? 0 : (my_page > last_page ? last_page : my_page);  // a corrupt table must not leave the pool

  bf16x8 aq[NSET][4];
  build_q_operand<NSET>(q_hat, b, j, Hq, G, agg, lane, aq);

  float* srow = scores + ((int64_t)b * Hkv + j) * stride;
#pragma unroll 1
  for (int qd = 0; qd < ppw / 4; ++qd) {
    if (pw + qd * 4 >= npages) break;
    uint4 kb[4][4];
#pragma unroll
    for (int pg = 0; pg < 4; ++pg) {
      const int32_t page = __shfl(my_page, qd * 4 + pg);
      const uint16_t* base = k_pool + chunk_offset(page, Hkv, j) + t * AS_HEAD_DIM;
#pragma unroll
      for (int m = 0; m < 4; ++m) kb[pg][m] = ld16<NT>(base + cmap(grp, m) * 8);
    }
    float res[4];
#pragma unroll
    for (int pg = 0; pg < 4; ++pg) {
      float v = -INFINITY;
#pragma unroll
      for (int s = 0; s < NSET; ++s) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int m = 0; m < 4; ++m)
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aq[s][m], __builtin_bit_cast(bf16x8, kb[pg][m]), acc, 0, 0, 0);
        v = fmaxf(v, fold_rows(acc));
      }
      res[pg] = group_max(v);
    }
    // lane (t, grp) stores token t of page qd*4 + grp: 256 contiguous bytes per wave
    float outv = grp == 0 ? res[0] : grp == 1 ? res[1] : grp == 2 ? res[2] : res[3];
    const int n = (pw + qd * 4 + grp) * AS_PAGE + t;
    if (n < N) srow[n] = outv + 0.0f;
  }
}


// Variants 1 and 2: K is read from global memory fully coalesced (a wavefront load covers
// 1 KB = 4 whole token rows), staged through LDS, and read back in the MFMA B layout.
//   DMA = false: global -> registers -> ds_write_b128 (swizzled)
//   DMA = true : global_load_lds_dwordx4 straight into LDS; the swizzle is applied on the
//                global side (lane l fetches the chunk whose slot it fills).
template <int NSET, bool DMA, bool NT>
__global__ __launch_bounds__(256) void score_mfma_lds(const uint16_t* __restrict__ k_pool,
                                                      const int32_t* __restrict__ block_table,
                                                      const int32_t* __restrict__ ctx_lens,
                                                      const float* __restrict__ q_hat, float* __restrict__ scores,
                                                      int64_t stride, int Hq, int Hkv, int G, int agg,
                                                      int max_pages, int32_t last_page, int ppw) {
  __shared__ uint4 stage[4][4 * 256];  // per wave: 4 page images of 4 KB
  const int b = blockIdx.z, j = blockIdx.y;
  const int N = clamp_ctx(ctx_lens[b], max_pages);
  const int npages = (N + AS_PAGE - 1) / AS_PAGE;
  const int p0 = blockIdx.x * (4 * ppw);
  if (p0 >= npages) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int t = lane & 15, grp = lane >> 4;
  const int pw = p0 + wave * ppw;
  if (pw >= npages) return;

  int32_t my_page = 0;
  if (lane < ppw && pw + lane < npages) my_page = block_table[(int64_t)b * max_pages + pw + lane];
  my_page = my_page < 0 ? 0 : (my_page > last_page ? last_page : my_page);  // a corrupt table must not leave the pool

  bf16x8 aq[NSET][4];
  build_q_operand<NSET>(q_hat, b, j, Hq, G, agg, lane, aq);

  uint4* st = stage[wave];
  float* srow = scores + ((int64_t)b * Hkv + j) * stride;
#pragma unroll 1
  for (int qd = 0; qd < ppw / 4; ++qd) {
    if (pw + qd * 4 >= npages) break;
    if (DMA) {
#pragma unroll
      for (int pg = 0; pg < 4; ++pg) {
        const int32_t page = __shfl(my_page, qd * 4 + pg);
        const uint16_t* base = k_pool + chunk_offset(page, Hkv, j);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int tok = 4 * i + grp;            // row this lane helps fill
          const int c = t ^ tok;                  // chunk that belongs in slot t of that row
          __builtin_amdgcn_global_load_lds(
              (const __attribute__((address_space(1))) void*)(base + tok * AS_HEAD_DIM + c * 8),
              (__attribute__((address_space(3))) void*)(st + pg * 256 + i * 64), 16, 0, NT ? 2 : 0);
        }
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    } else {
      uint4 kb[4][4];
#pragma unroll
      for (int pg = 0; pg < 4; ++pg) {
        const int32_t page = __shfl(my_page, qd * 4 + pg);
        const uint4* base = reinterpret_cast<const uint4*>(k_pool + chunk_offset(page, Hkv, j));
#pragma unroll
        for (int i = 0; i < 4; ++i) kb[pg][i] = ld16<NT>(base + i * 64 + lane);
      }
#pragma unroll
      for (int pg = 0; pg < 4; ++pg)
#pragma unroll
        for (int i = 0; i < 4; ++i) st[pg * 256 + lds_slot(4 * i + grp, t)] = kb[pg][i];
    }
    __builtin_amdgcn_wave_barrier();
    float res[4];
#pragma unroll
    for (int pg = 0; pg < 4; ++pg) {
      uint4 kb[4];
#pragma unroll
      for (int m = 0; m < 4; ++m) kb[m] = st[pg * 256 + lds_slot(t, cmap(grp, m))];
      float v = -INFINITY;
#pragma unroll
      for (int s = 0; s < NSET; ++s) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int m = 0; m < 4; ++m)
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aq[s][m], __builtin_bit_cast(bf16x8, kb[m]), acc, 0, 0, 0);
        v = fmaxf(v, fold_rows(acc));
      }
      res[pg] = group_max(v);
    }
    float outv = grp == 0 ? res[0] : grp == 1 ? res[1] : grp == 2 ? res[2] : res[3];
    const int n = (pw + qd * 4 + grp) * AS_PAGE + t;
    if (n < N) {
      if (NT) __builtin_nontemporal_store(outv + 0.0f, &srow[n]);   // written once, read by another kernel: streaming
      else srow[n] = outv + 0.0f;
    }
    asm volatile("" ::: "memory");
    __builtin_amdgcn_wave_barrier();
  }
}

// Calibration kernel (variant 9): the same paged walk over K with fully coalesced loads and
// no arithmetic beyond an XOR fold; writes one word per token where the scores would go.
// It gives the achievable streaming rate of this access pattern and a known-size reference
// for scaling profiler byte counters.
template <bool NT>
__global__ __launch_bounds__(256) void stream_read_paged(const uint16_t* __restrict__ k_pool,
                                                         const int32_t* __restrict__ block_table,
                                                         const int32_t* __restrict__ ctx_lens,
                                                         float* __restrict__ scores, int64_t stride, int Hkv,
                                                         int max_pages, int32_t last_page, int ppw) {
  const int b = blockIdx.z, j = blockIdx.y;
  const int N = clamp_ctx(ctx_lens[b], max_pages);
  const int npages = (N + AS_PAGE - 1) / AS_PAGE;
  const int p0 = blockIdx.x * (4 * ppw);
  if (p0 >= npages) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int pw = p0 + wave * ppw;
  if (pw >= npages) return;
  int32_t my_page = 0;
  if (lane < ppw && pw + lane < npages) my_page = block_table[(int64_t)b * max_pages + pw + lane];
  my_page = my_page < 0 ? 0 : (my_page > last_page ? last_page : my_page);  // a corrupt table must not leave the pool
  float* srow = scores + ((int64_t)b * Hkv + j) * stride;
#pragma unroll 1
  for (int qd = 0; qd < ppw / 4; ++qd) {
    if (pw + qd * 4 >= npages) break;
    uint4 kb[4][4];
#pragma unroll
    for (int pg = 0; pg < 4; ++pg) {
      const int32_t page = __shfl(my_page, qd * 4 + pg);
      const uint4* base = reinterpret_cast<const uint4*>(k_pool + chunk_offset(page, Hkv, j));
#pragma unroll
      for (int i = 0; i < 4; ++i) kb[pg][i] = ld16<NT>(base + i * 64 + lane);
    }
    uint32_t x = 0;
#pragma unroll
    for (int pg = 0; pg < 4; ++pg)
#pragma unroll
      for (int i = 0; i < 4; ++i) x ^= kb[pg][i].x ^ kb[pg][i].y ^ kb[pg][i].z ^ kb[pg][i].w;
    const int n = (pw + qd * 4) * AS_PAGE + lane;
    if (n < N) srow[n] = __uint_as_float(x & 0x3fffffffu);
  }
}

hipError_t launch_score(int variant, const as_params* p, const as_kv_view* kv, const float* q_hat, float* scores,
                        int64_t stride, hipStream_t s) {
  if (p->batch == 0 || p->max_pages_per_seq == 0) return hipSuccess;
  const int G = p->n_q_heads / p->n_kv_heads;
  const uint16_t* kp = reinterpret_cast<const uint16_t*>(kv->k_pool);
  // pages per wavefront: as many as leave about eight workgroups per compute unit, so that the prologue (the
  // query operand, the page ids) is spread over up to 2048 tokens per workgroup on large batches and small
  // batches still fill the chip
  int ppw = 32;
  while (ppw > 8 && (int64_t)p->batch * p->n_kv_heads * ((p->max_pages_per_seq + 4 * ppw - 1) / (4 * ppw)) < 2048)
    ppw /= 2;
  dim3 grid((p->max_pages_per_seq + 4 * ppw - 1) / (4 * ppw), p->n_kv_heads, p->batch);
  const bool two = (p->agg != AS_AGG_SUM) && G > 8;
  const int32_t last_page = (int32_t)(kv->num_pages > 0 ? kv->num_pages - 1 : 0);
#define AS_SCORE_LAUNCH(KERNEL)                                                                              \
  hipLaunchKernelGGL(KERNEL, grid, dim3(256), 0, s, kp, kv->block_table, kv->ctx_lens, q_hat, scores, stride, \
                     p->n_q_heads, p->n_kv_heads, G, p->agg, p->max_pages_per_seq, last_page, ppw)
  const bool nt = variant >= 10;
  if (p->agg != AS_AGG_SUM && G > 16) {
    // MQA-sized groups: four or eight operand sets of eight heads each; only the product variant is instantiated
    if (G > 32) AS_SCORE_LAUNCH((score_mfma_lds<8, true, true>));
    else AS_SCORE_LAUNCH((score_mfma_lds<4, true, true>));
    return hipGetLastError();
  }
  switch (variant % 10) {
    case 9:
      if (nt)
        hipLaunchKernelGGL(stream_read_paged<true>, grid, dim3(256), 0, s, kp, kv->block_table, kv->ctx_lens, scores,
                           stride, p->n_kv_heads, p->max_pages_per_seq, last_page, ppw);
      else
        hipLaunchKernelGGL(stream_read_paged<false>, grid, dim3(256), 0, s, kp, kv->block_table, kv->ctx_lens, scores,
                           stride, p->n_kv_heads, p->max_pages_per_seq, last_page, ppw);
      break;
    case 1:
      if (two) { if (nt) AS_SCORE_LAUNCH((score_mfma_lds<2, false, true>)); else AS_SCORE_LAUNCH((score_mfma_lds<2, false, false>)); }
      else { if (nt) AS_SCORE_LAUNCH((score_mfma_lds<1, false, true>)); else AS_SCORE_LAUNCH((score_mfma_lds<1, false, false>)); }
      break;
    case 2:
      if (two) { if (nt) AS_SCORE_LAUNCH((score_mfma_lds<2, true, true>)); else AS_SCORE_LAUNCH((score_mfma_lds<2, true, false>)); }
      else { if (nt) AS_SCORE_LAUNCH((score_mfma_lds<1, true, true>)); else AS_SCORE_LAUNCH((score_mfma_lds<1, true, false>)); }
      break;
    default:
      if (two) { if (nt) AS_SCORE_LAUNCH((score_mfma_direct<2, true>)); else AS_SCORE_LAUNCH((score_mfma_direct<2, false>)); }
      else { if (nt) AS_SCORE_LAUNCH((score_mfma_direct<1, true>)); else AS_SCORE_LAUNCH((score_mfma_direct<1, false>)); }
      break;
  }
#undef AS_SCORE_LAUNCH
  return hipGetLastError();
}

}  // namespace asx
