// Clamps that keep a corrupt caller-owned array (context length, page id, token index, selection count) from
// taking a kernel outside its buffers.  Plain integer functions, usable from host and device code: the kernels
// call them before every dependent address computation, and a host-only build of this header is tested on the CPU
// over negative, oversized and boundary values.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define AS_GUARD_FN __host__ __device__ __forceinline__
#else
#define AS_GUARD_FN static inline
#endif

#define AS_GUARD_PAGE 16 /* tokens per page */

// context length as the kernels use it: never negative, never past the block table row (max_pages pages)
AS_GUARD_FN int clamp_ctx(int n, int max_pages) {
  const int64_t cap = (int64_t)max_pages * AS_GUARD_PAGE;
  return n < 0 ? 0 : ((int64_t)n > cap ? (int)cap : n);
}

// physical page id into [0, last_page] (last_page = num_pages - 1 >= 0)
AS_GUARD_FN int32_t clamp_page(int32_t pg, int32_t last_page) { return pg < 0 ? 0 : (pg > last_page ? last_page : pg); }

// token index into [0, N) for a sequence of N >= 1 tokens (N == 0 gives 0: callers do not dereference then)
AS_GUARD_FN int clamp_token(int n, int N) { return n < 0 ? 0 : (n >= N ? (N > 0 ? N - 1 : 0) : n); }

// selection count into [0, C]; an empty sequence has nothing selected
AS_GUARD_FN int clamp_count(int cnt, int C, int N) { return (cnt < 0 || N == 0) ? 0 : (cnt > C ? C : cnt); }

// start of the dense tail into [0, N]
AS_GUARD_FN int clamp_tail(int tail0, int N) { return tail0 < 0 ? 0 : (tail0 > N ? N : tail0); }

// score-row length: the context clamped to the block table and to the row stride
AS_GUARD_FN int clamp_row(int n, int max_pages, int64_t stride) {
  const int c = clamp_ctx(n, max_pages);
  return (int64_t)c > stride ? (int)stride : c;
}
