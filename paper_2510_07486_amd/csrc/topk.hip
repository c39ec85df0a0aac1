// Per-(sequence, KV head) top-k over the fp32 score row (Sec. 4.3, cache-rank item (2)).
//
// Exact radix select, no sort: scores map to order-preserving 32-bit keys; three LDS
// histogram passes (12 + 10 + 10 bits, most significant first) find the key T of the
// C-th largest score and r, the number of tokens equal to T still to be taken; one
// ordered pass then emits, ascending by token index, every token with key > T and the
// first r tokens with key == T (so ties resolve to the lowest index).  See block_select.
// One 1024-thread workgroup per row; the row is re-read from L2 each pass.  This is the
// stand-alone stage for rows above 32768 tokens; shorter rows keep their keys in registers
// (topk_regs_kernel below), and the fused selection never materialises the scores (select_fused.hip).
#include "common.hpp"
#include "topk_common.hpp"

namespace asx {


__global__ __launch_bounds__(TK_THREADS) void topk_kernel(const float* __restrict__ scores, int64_t stride,
                                                          const int32_t* __restrict__ ctx_lens,
                                                          int32_t* __restrict__ sel_idx,
                                                          int32_t* __restrict__ sel_cnt, int Hkv, int C,
                                                          int max_pages) {
  __shared__ uint32_t hist[TK_BINS];
  __shared__ __attribute__((aligned(16))) uint32_t xch[TK_XCH];

  const int row = blockIdx.x;
  const int b = row / Hkv;
  const int tid = threadIdx.x;
  const int N = clamp_row(ctx_lens[b], max_pages, stride);   // never past the block table (what the scoring kernel
                                                             // wrote) nor past the score row
  const float* s = scores + (int64_t)row * stride;
  int32_t* out = sel_idx + (int64_t)row * C;
  const int keep = N < C ? N : C;
  if (tid == 0) sel_cnt[row] = keep;
  for (int i = keep + tid; i < C; i += TK_THREADS) out[i] = -1;
  if (keep == 0) return;
  auto key_of = [&](int i, bool& valid) -> uint32_t {
    valid = true;
    return score_key(s[i]);
  };
  auto emit = [&](uint32_t pos, int i, uint32_t) { out[pos] = i; };
  block_select<TK_THREADS, 12>(N, N, keep, false, key4_from_scalar(N, key_of), emit, hist, xch);
}

// Rows of at most NPT * 1024 tokens: the row's keys are read once, coalesced, into registers (token i of the row
// sits in thread i % 1024); the best min(C, N) are marked there (mark_best: radix thresholds on the key, ties by
// token) and put into ascending token order through a bitmap of the row (rank of a token = set bits below it).
// One read of the scores instead of one per radix pass.
template <int NPT>
__global__ __launch_bounds__(TK_THREADS) void topk_regs_kernel(const float* __restrict__ scores, int64_t stride,
                                                               const int32_t* __restrict__ ctx_lens,
                                                               int32_t* __restrict__ sel_idx,
                                                               int32_t* __restrict__ sel_cnt, int Hkv, int C,
                                                               int max_pages) {
  constexpr int WORDS = NPT * TK_THREADS / 32;   // bitmap words, NPT per thread
  __shared__ uint32_t hist[TK_BINS];
  __shared__ uint32_t bitmap[WORDS];
  __shared__ uint32_t wpre[WORDS];               // set bits in the words below
  __shared__ __attribute__((aligned(16))) uint32_t xch[TK_XCH];
  const int row = blockIdx.x;
  const int b = row / Hkv;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int N = clamp_row(ctx_lens[b], max_pages, stride);
  if (N > NPT * TK_THREADS) N = NPT * TK_THREADS;   // the host launches this kernel only when every row fits
  const float* s = scores + (int64_t)row * stride;
  int32_t* out = sel_idx + (int64_t)row * C;
  const int keep = N < C ? N : C;
  if (tid == 0) sel_cnt[row] = keep;
  for (int i = keep + tid; i < C; i += TK_THREADS) out[i] = -1;
  if (keep == 0) return;
  uint32_t key[NPT];
  int32_t tok[NPT];
  bool have[NPT], sel[NPT];
  // every load is issued before the first one is waited for: slots beyond the row re-read its last score (N >= 1
  // here) instead of sitting in a branch of their own, which would serialise the NPT round trips
  float raw[NPT];
#pragma unroll
  for (int e = 0; e < NPT; ++e) {
    tok[e] = tid + e * TK_THREADS;
    have[e] = tok[e] < N;
    raw[e] = s[have[e] ? tok[e] : N - 1];
  }
#pragma unroll
  for (int e = 0; e < NPT; ++e) {
    key[e] = have[e] ? score_key(raw[e]) : 0u;
    sel[e] = have[e];
  }
  if (keep < N) mark_best<TK_THREADS, 12, NPT>(key, tok, have, keep, hist, xch, sel);
  for (int wd = tid; wd < WORDS; wd += TK_THREADS) bitmap[wd] = 0;
  __syncthreads();
#pragma unroll
  for (int e = 0; e < NPT; ++e)
    if (sel[e]) atomicOr(&bitmap[tok[e] >> 5], 1u << (tok[e] & 31));
  __syncthreads();
  // exclusive prefix of the words' bit counts: a thread owns WPT consecutive words
  constexpr int WPT = (WORDS + TK_THREADS - 1) / TK_THREADS;
  uint32_t pc[WPT], mine = 0;
#pragma unroll
  for (int k = 0; k < WPT; ++k) {
    const int wd = tid * WPT + k;
    pc[k] = wd < WORDS ? (uint32_t)__popc(bitmap[wd]) : 0u;
    mine += pc[k];
  }
  const uint32_t inc = wave_incl_scan(mine);
  if (lane == 63) xch[wave] = inc;
  __syncthreads();
  uint32_t woff[1];
  seg_wave_offsets<TK_THREADS / 64, 1>(xch, wave, woff);
  uint32_t run = woff[0] + inc - mine;
#pragma unroll
  for (int k = 0; k < WPT; ++k) {
    const int wd = tid * WPT + k;
    if (wd < WORDS) wpre[wd] = run;
    run += pc[k];
  }
  __syncthreads();
#pragma unroll
  for (int e = 0; e < NPT; ++e)
    if (sel[e]) {
      const uint32_t rank = wpre[tok[e] >> 5] + (uint32_t)__popc(bitmap[tok[e] >> 5] & ((1u << (tok[e] & 31)) - 1u));
      out[rank] = tok[e];
    }
}

hipError_t launch_topk(const as_params* p, const float* scores, int64_t stride, const int32_t* ctx_lens,
                       int32_t* sel_idx, int32_t* sel_cnt, hipStream_t s) {
  const int64_t rows = (int64_t)p->batch * p->n_kv_heads;   // <= 2^31 - 1 (checked with the parameters)
  if (rows == 0) return hipSuccess;
  // rows that fit 32 keys per thread are selected in registers; longer ones by the positional kernel
  const int64_t longest = (int64_t)p->max_pages_per_seq * AS_PAGE < stride ? (int64_t)p->max_pages_per_seq * AS_PAGE : stride;
#define AS_TOPK_REGS(NPT_)                                                                                        \
  hipLaunchKernelGGL(topk_regs_kernel<NPT_>, dim3((unsigned)rows), dim3(TK_THREADS), 0, s, scores, stride, ctx_lens, \
                     sel_idx, sel_cnt, p->n_kv_heads, p->budget, p->max_pages_per_seq)
  if (longest <= 4 * TK_THREADS) AS_TOPK_REGS(4);
  else if (longest <= 8 * TK_THREADS) AS_TOPK_REGS(8);
  else if (longest <= 16 * TK_THREADS) AS_TOPK_REGS(16);
  else if (longest <= 32 * TK_THREADS) AS_TOPK_REGS(32);
  else
    hipLaunchKernelGGL(topk_kernel, dim3((unsigned)rows), dim3(TK_THREADS), 0, s, scores, stride, ctx_lens, sel_idx,
                       sel_cnt, p->n_kv_heads, p->budget, p->max_pages_per_seq);
#undef AS_TOPK_REGS
  return hipGetLastError();
}

}  // namespace asx
