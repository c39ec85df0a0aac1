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

// Rows of at most NPT * 1024 tokens: one read of the scores instead of one per radix pass (topk_regs_row).
template <int NPT>
__global__ __launch_bounds__(TK_THREADS) void topk_regs_kernel(const float* __restrict__ scores, int64_t stride,
                                                               const int32_t* __restrict__ ctx_lens,
                                                               int32_t* __restrict__ sel_idx,
                                                               int32_t* __restrict__ sel_cnt, int Hkv, int C,
                                                               int max_pages) {
  __shared__ __attribute__((aligned(16))) uint32_t hist[4 * TK_BINS];
  __shared__ uint32_t bitmap[NPT * TK_THREADS / 32];
  __shared__ uint32_t wpre[NPT * TK_THREADS / 32];
  __shared__ __attribute__((aligned(16))) uint32_t xch[TK_XCH];
  const int row = blockIdx.x;
  const int b = row / Hkv;
  int N = clamp_row(ctx_lens[b], max_pages, stride);
  if (N > NPT * TK_THREADS) N = NPT * TK_THREADS;   // the host launches this kernel only when every row fits
  const float* s = scores + (int64_t)row * stride;
  topk_regs_row<NPT>([&](int i) { return s[i]; }, N, C, sel_idx + (int64_t)row * C, sel_cnt + row, hist, bitmap, wpre,
                     xch);
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
