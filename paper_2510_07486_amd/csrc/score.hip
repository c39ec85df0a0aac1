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

// K is read from global memory fully coalesced (a wavefront load covers 1 KB = 4 whole token rows) with
// global_load_lds_dwordx4 straight into a per-wave LDS image (non-temporal; the swizzle is applied on the
// global side: lane l fetches the chunk whose slot it fills) and read back in the MFMA B layout.
template <int NSET>
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
  my_page = clamp_page(my_page, last_page);  // a corrupt table must not leave the pool

  bf16x8 aq[NSET][4];
  build_q_operand<NSET>(q_hat, b, j, Hq, G, agg, lane, aq);

  uint4* st = stage[wave];
  float* srow = scores + ((int64_t)b * Hkv + j) * stride;
#pragma unroll 1
  for (int qd = 0; qd < ppw / 4; ++qd) {
    if (pw + qd * 4 >= npages) break;
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
            (__attribute__((address_space(3))) void*)(st + pg * 256 + i * 64), 16, 0, 2);
      }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
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
      __builtin_nontemporal_store(outv + 0.0f, &srow[n]);   // written once, read by another kernel: streaming
    }
    asm volatile("" ::: "memory");
    __builtin_amdgcn_wave_barrier();
  }
}

// Calibration kernels (as_debug_stream_read_paged / _flat): the same paged walk over K with fully coalesced
// non-temporal loads and no arithmetic beyond an XOR fold.  WORDS = true writes one word per token where the
// scores would go: a known-size reference for scaling profiler byte counters.  WORDS = false writes one word
// per wavefront: the streaming-read rate this access pattern can reach at all.
template <bool WORDS>
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
  my_page = clamp_page(my_page, last_page);  // a corrupt table must not leave the pool
  float* srow = scores + ((int64_t)b * Hkv + j) * stride;
  uint32_t fold = 0;
#pragma unroll 1
  for (int qd = 0; qd < ppw / 4; ++qd) {
    if (pw + qd * 4 >= npages) break;
    uint4 kb[4][4];
#pragma unroll
    for (int pg = 0; pg < 4; ++pg) {
      const int32_t page = __shfl(my_page, qd * 4 + pg);
      const uint4* base = reinterpret_cast<const uint4*>(k_pool + chunk_offset(page, Hkv, j));
#pragma unroll
      for (int i = 0; i < 4; ++i) kb[pg][i] = ld16<true>(base + i * 64 + lane);
    }
    uint32_t x = 0;
#pragma unroll
    for (int pg = 0; pg < 4; ++pg)
#pragma unroll
      for (int i = 0; i < 4; ++i) x ^= kb[pg][i].x ^ kb[pg][i].y ^ kb[pg][i].z ^ kb[pg][i].w;
    const int n = (pw + qd * 4) * AS_PAGE + lane;
    if (WORDS) {
      if (n < N) srow[n] = __uint_as_float(x & 0x3fffffffu);
    } else {
      fold ^= x;
    }
  }
  if (!WORDS) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) fold ^= (uint32_t)__shfl_xor((int)fold, o);
    if (lane == 0) srow[pw * AS_PAGE] = __uint_as_float(fold & 0x3fffffffu);   // pw < npages: inside the row
  }
}

// The plain streaming read: a buffer of n16 16-byte words read front to back, no page table.  Each workgroup
// takes FLAT_TILE contiguous bytes per round (a wavefront load covers 1 KB, eight loads in flight per lane)
// and the workgroups stride over the buffer; one word written per workgroup.  Shape picked from a sweep of
// 1024-16384 workgroups of 256-1024 threads, 4-16 loads in flight, strided and contiguous assignment, plain and
// non-temporal loads: every non-temporal variant lands within 6.65-7.08 TB/s, eight loads per lane at the top;
// plain loads reach 6.0-6.2 TB/s.
static constexpr int FLAT_WGS = 2048;                 // workgroups of the flat read (8 per compute unit)
static constexpr int FLAT_U = 8;                      // 16-byte loads in flight per lane
static constexpr int64_t FLAT_TILE = 256 * FLAT_U;    // 16-byte words per workgroup and round (32 KB)
__global__ __launch_bounds__(256) void stream_read_flat(const uint4* __restrict__ buf, int64_t n16,
                                                        uint32_t* __restrict__ sink) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  uint32_t fold = 0;
  for (int64_t base = (int64_t)blockIdx.x * FLAT_TILE; base < n16; base += (int64_t)gridDim.x * FLAT_TILE) {
    uint4 v[FLAT_U];
    const int64_t w0 = base + (int64_t)wave * (64 * FLAT_U) + lane;   // a wave owns 8 KB of the tile
#pragma unroll
    for (int u = 0; u < FLAT_U; ++u) {
      const int64_t i = w0 + u * 64;
      v[u] = ld16<true>(buf + (i < n16 ? i : n16 - 1));   // the ragged end re-reads the last word
    }
#pragma unroll
    for (int u = 0; u < FLAT_U; ++u) fold ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) fold ^= (uint32_t)__shfl_xor((int)fold, o);
  __shared__ uint32_t part[4];
  if (lane == 0) part[wave] = fold;
  __syncthreads();
  if (tid == 0) sink[blockIdx.x] = part[0] ^ part[1] ^ part[2] ^ part[3];
}

// pages per wavefront: as many as leave about eight workgroups per compute unit, so that the prologue (the
// query operand, the page ids) is spread over up to 2048 tokens per workgroup on large batches and small
// batches still fill the chip
static int pages_per_wave(const as_params* p) {
  int ppw = 32;
  while (ppw > 8 && (int64_t)p->batch * p->n_kv_heads * ((p->max_pages_per_seq + 4 * ppw - 1) / (4 * ppw)) < 2048)
    ppw /= 2;
  return ppw;
}

hipError_t launch_score(const as_params* p, const as_kv_view* kv, const float* q_hat, float* scores, int64_t stride,
                        hipStream_t s) {
  if (p->batch == 0 || p->max_pages_per_seq == 0) return hipSuccess;
  const int G = p->n_q_heads / p->n_kv_heads;
  const uint16_t* kp = reinterpret_cast<const uint16_t*>(kv->k_pool);
  const int ppw = pages_per_wave(p);
  dim3 grid((p->max_pages_per_seq + 4 * ppw - 1) / (4 * ppw), p->n_kv_heads, p->batch);
  const int32_t last_page = (int32_t)(kv->num_pages > 0 ? kv->num_pages - 1 : 0);
#define AS_SCORE_LAUNCH(KERNEL)                                                                              \
  hipLaunchKernelGGL(KERNEL, grid, dim3(256), 0, s, kp, kv->block_table, kv->ctx_lens, q_hat, scores, stride, \
                     p->n_q_heads, p->n_kv_heads, G, p->agg, p->max_pages_per_seq, last_page, ppw)
  // operand sets of eight heads each: one up to 8 heads per KV head, two up to 16, four or eight for MQA-sized groups
  if (p->agg == AS_AGG_SUM || G <= 8) AS_SCORE_LAUNCH(score_mfma_lds<1>);
  else if (G <= 16) AS_SCORE_LAUNCH(score_mfma_lds<2>);
  else if (G <= 32) AS_SCORE_LAUNCH(score_mfma_lds<4>);
  else AS_SCORE_LAUNCH(score_mfma_lds<8>);
#undef AS_SCORE_LAUNCH
  return hipGetLastError();
}

hipError_t launch_stream_read_paged(const as_params* p, const as_kv_view* kv, float* sink, int64_t stride,
                                    bool words_per_token, hipStream_t s) {
  if (p->batch == 0 || p->max_pages_per_seq == 0) return hipSuccess;
  const uint16_t* kp = reinterpret_cast<const uint16_t*>(kv->k_pool);
  const int ppw = pages_per_wave(p);
  dim3 grid((p->max_pages_per_seq + 4 * ppw - 1) / (4 * ppw), p->n_kv_heads, p->batch);
  const int32_t last_page = (int32_t)(kv->num_pages > 0 ? kv->num_pages - 1 : 0);
  if (words_per_token)
    hipLaunchKernelGGL(stream_read_paged<true>, grid, dim3(256), 0, s, kp, kv->block_table, kv->ctx_lens, sink, stride,
                       p->n_kv_heads, p->max_pages_per_seq, last_page, ppw);
  else
    hipLaunchKernelGGL(stream_read_paged<false>, grid, dim3(256), 0, s, kp, kv->block_table, kv->ctx_lens, sink, stride,
                       p->n_kv_heads, p->max_pages_per_seq, last_page, ppw);
  return hipGetLastError();
}

size_t stream_read_flat_sink_words() { return FLAT_WGS; }

hipError_t launch_stream_read_flat(const void* buf, size_t nbytes, uint32_t* sink, hipStream_t s) {
  const int64_t n16 = (int64_t)(nbytes / 16);
  if (n16 == 0) return hipSuccess;
  hipLaunchKernelGGL(stream_read_flat, dim3(FLAT_WGS), dim3(256), 0, s, reinterpret_cast<const uint4*>(buf), n16, sink);
  return hipGetLastError();
}

}  // namespace asx
