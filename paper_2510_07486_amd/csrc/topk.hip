// Per-(sequence, KV head) top-k over the fp32 score row (Sec. 4.3, cache-rank item (2)).
//
// Exact radix select, no sort: scores map to order-preserving 32-bit keys; three LDS
// histogram passes (12 + 12 + 8 bits, most significant first) find the key T of the
// C-th largest score and r, the number of tokens equal to T still to be taken; one
// ordered pass then emits, ascending by token index, every token with key > T and the
// first r tokens with key == T (so ties resolve to the lowest index).  The output slot of
// a token is (#greater before it) + min(#equal before it, r), which needs only wavefront
// ballots and one 16-entry cross-wave prefix per 1024-token chunk.
// One 1024-thread workgroup per row; the row (<= 256 KB) is re-read from L2 each pass.
#include "common.hpp"

namespace asx {

static constexpr int TK_THREADS = 1024;
static constexpr int TK_WAVES = TK_THREADS / 64;
static constexpr int TK_BINS = 4096;

// larger float -> larger key; -0 == +0; NaN -> 0 (below -inf)
__device__ __forceinline__ uint32_t score_key(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0u;
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Finds the bin d (scanning from the highest bin down) with
//   sum_{d' > d} hist[d'] < remaining <= sum_{d' >= d} hist[d'];
// writes d and the count above it to sh_out[0..1].  nb <= 4 * TK_THREADS bins.
__device__ __forceinline__ void find_bin(const uint32_t* hist, int nb, uint32_t remaining, uint32_t* wave_tot,
                                         uint32_t* sh_out) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int per = (nb + TK_THREADS - 1) / TK_THREADS;  // bins per thread, descending order
  uint32_t loc[4];
  uint32_t mine = 0;
  for (int i = 0; i < per; ++i) {
    int rb = tid * per + i;  // reversed bin index
    loc[i] = (rb < nb) ? hist[nb - 1 - rb] : 0u;
    mine += loc[i];
  }
  // inclusive scan across the block
  uint32_t inc = mine;
  for (int o = 1; o < 64; o <<= 1) {
    uint32_t v = __shfl_up(inc, o);
    if (lane >= o) inc += v;
  }
  if (lane == 63) wave_tot[wave] = inc;
  __syncthreads();
  uint32_t off = 0;
  for (int w = 0; w < wave; ++w) off += wave_tot[w];
  uint32_t excl = off + inc - mine;
  for (int i = 0; i < per; ++i) {
    if (excl < remaining && remaining <= excl + loc[i]) {
      sh_out[0] = (uint32_t)(nb - 1 - (tid * per + i));
      sh_out[1] = excl;
    }
    excl += loc[i];
  }
  __syncthreads();
}

__global__ __launch_bounds__(TK_THREADS) void topk_kernel(const float* __restrict__ scores, int64_t stride,
                                                          const int32_t* __restrict__ ctx_lens,
                                                          int32_t* __restrict__ sel_idx,
                                                          int32_t* __restrict__ sel_cnt, int Hkv, int C) {
  __shared__ uint32_t hist[TK_BINS];
  __shared__ uint32_t wave_tot[TK_WAVES];
  __shared__ uint32_t wave_eq[TK_WAVES], wave_gt[TK_WAVES];
  __shared__ uint32_t found[2];

  const int row = blockIdx.x;
  const int b = row / Hkv;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int N = ctx_lens[b];
  const float* s = scores + (int64_t)row * stride;
  int32_t* out = sel_idx + (int64_t)row * C;
  const int keep = N < C ? N : C;
  if (tid == 0) sel_cnt[row] = keep;
  for (int i = keep + tid; i < C; i += TK_THREADS) out[i] = -1;
  if (keep == 0) return;
  if (N <= C) {
    for (int i = tid; i < N; i += TK_THREADS) out[i] = i;
    return;
  }

  // ---- radix select of the keep-th largest key -------------------------------------
  uint32_t prefix = 0, mask = 0, remaining = (uint32_t)keep;
  const int shifts[3] = {20, 8, 0};
  const int widths[3] = {12, 12, 8};
#pragma unroll 1
  for (int pass = 0; pass < 3; ++pass) {
    const int nb = 1 << widths[pass];
    const int sh = shifts[pass];
    for (int i = tid; i < nb; i += TK_THREADS) hist[i] = 0;
    __syncthreads();
    for (int n = tid; n < N; n += TK_THREADS) {
      uint32_t k = score_key(s[n]);
      if ((k & mask) == prefix) atomicAdd(&hist[(k >> sh) & (nb - 1)], 1u);
    }
    __syncthreads();
    find_bin(hist, nb, remaining, wave_tot, found);
    prefix |= found[0] << sh;
    mask |= (uint32_t)(nb - 1) << sh;
    remaining -= found[1];
    __syncthreads();
  }
  const uint32_t T = prefix;
  const uint32_t r = remaining;  // tokens with key == T still to take (>= 1)

  // ---- ordered emission ---------------------------------------------------------------
  uint32_t gt_run = 0, eq_run = 0;
  const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
#pragma unroll 1
  for (int base = 0; base < N; base += TK_THREADS) {
    const int n = base + tid;
    uint32_t k = (n < N) ? score_key(s[n]) : 0u;
    const bool gt = (n < N) && k > T;
    const bool eq = (n < N) && k == T;
    const uint64_t bgt = __ballot(gt), beq = __ballot(eq);
    if (lane == 0) {
      wave_gt[wave] = __popcll(bgt);
      wave_eq[wave] = __popcll(beq);
    }
    __syncthreads();
    uint32_t gt_before = gt_run + __popcll(bgt & lt_mask), eq_before = eq_run + __popcll(beq & lt_mask);
    uint32_t gt_tot = 0, eq_tot = 0;
#pragma unroll
    for (int w = 0; w < TK_WAVES; ++w) {
      const uint32_t g = wave_gt[w], e = wave_eq[w];
      if (w < wave) { gt_before += g; eq_before += e; }
      gt_tot += g;
      eq_tot += e;
    }
    if (gt || (eq && eq_before < r)) out[gt_before + (eq_before < r ? eq_before : r)] = n;
    gt_run += gt_tot;
    eq_run += eq_tot;
    __syncthreads();
  }
}

hipError_t launch_topk(const as_params* p, const float* scores, int64_t stride, const int32_t* ctx_lens,
                       int32_t* sel_idx, int32_t* sel_cnt, hipStream_t s) {
  const int rows = p->batch * p->n_kv_heads;
  if (rows == 0) return hipSuccess;
  hipLaunchKernelGGL(topk_kernel, dim3(rows), dim3(TK_THREADS), 0, s, scores, stride, ctx_lens, sel_idx, sel_cnt,
                     p->n_kv_heads, p->budget);
  return hipGetLastError();
}

}  // namespace asx
