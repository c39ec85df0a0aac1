// Per-(sequence, KV head) top-k over the fp32 score row (Sec. 4.3, cache-rank item (2)).
//
// Exact radix select, no sort: scores map to order-preserving 32-bit keys; three LDS
// histogram passes (12 + 10 + 10 bits, most significant first) find the key T of the
// C-th largest score and r, the number of tokens equal to T still to be taken; one
// ordered pass then emits, ascending by token index, every token with key > T and the
// first r tokens with key == T (so ties resolve to the lowest index).  See block_select.
// One 1024-thread workgroup per row; the row is re-read from L2 each pass.  This is the
// stand-alone stage; the fused selection keeps the keys in LDS instead (select_fused.hip).
#include "common.hpp"
#include "topk_common.hpp"

namespace asx {


__global__ __launch_bounds__(TK_THREADS) void topk_kernel(const float* __restrict__ scores, int64_t stride,
                                                          const int32_t* __restrict__ ctx_lens,
                                                          int32_t* __restrict__ sel_idx,
                                                          int32_t* __restrict__ sel_cnt, int Hkv, int C) {
  __shared__ uint32_t hist[TK_BINS];
  __shared__ __attribute__((aligned(16))) uint32_t xch[TK_XCH];

  const int row = blockIdx.x;
  const int b = row / Hkv;
  const int tid = threadIdx.x;
  int N = ctx_lens[b];
  N = N < 0 ? 0 : ((int64_t)N > stride ? (int)stride : N);   // never past the score row
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

hipError_t launch_topk(const as_params* p, const float* scores, int64_t stride, const int32_t* ctx_lens,
                       int32_t* sel_idx, int32_t* sel_cnt, hipStream_t s) {
  const int rows = p->batch * p->n_kv_heads;
  if (rows == 0) return hipSuccess;
  hipLaunchKernelGGL(topk_kernel, dim3(rows), dim3(TK_THREADS), 0, s, scores, stride, ctx_lens, sel_idx, sel_cnt,
                     p->n_kv_heads, p->budget);
  return hipGetLastError();
}

}  // namespace asx
