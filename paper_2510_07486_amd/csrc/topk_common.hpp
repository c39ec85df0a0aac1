// Device helpers shared by the top-k kernels: order-preserving score keys and the
// block-wide histogram search of the radix select (1024-thread workgroups).
#pragma once
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


// Exact selection of the `keep` largest of the valid keys at virtual positions 0..n-1, emitted
// in ascending position order; equal keys resolve to the lowest position.  Run by a whole
// 1024-thread workgroup.
//   key_of(i, valid) -> key of position i (valid = false marks a hole that is never selected)
//   emit(pos, i, key)   called once per selected position, pos = its rank in ascending order
//   total = number of valid positions (>= keep); keep >= total selects everything.
//   hist0_ready: hist[] already holds the histogram of the top 12 key bits of all valid keys.
// Radix select: three histogram passes (12 + 12 + 8 bits, most significant first) find the key T
// of the keep-th largest and r, how many keys equal to T are still to be taken; the output
// slot of a selected position is (#greater before it) + min(#equal before it, r).
template <class KeyFn, class EmitFn>
__device__ __forceinline__ void block_select(int n, int total, int keep, bool hist0_ready, KeyFn key_of, EmitFn emit,
                                             uint32_t* hist, uint32_t* wave_tot, uint32_t* wave_eq,
                                             uint32_t* wave_gt, uint32_t* found) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bool all = keep >= total;
  uint32_t T = 0, r = 0;
  if (!all) {
    uint32_t prefix = 0, mask = 0, remaining = (uint32_t)keep;
#pragma unroll 1
    for (int pass = 0; pass < 3; ++pass) {
      const int width = pass == 2 ? 8 : 12;
      const int sh = pass == 0 ? 20 : pass == 1 ? 8 : 0;
      const int nb = 1 << width;
      if (!(pass == 0 && hist0_ready)) {
        for (int i = tid; i < nb; i += TK_THREADS) hist[i] = 0;
        __syncthreads();
        for (int i = tid; i < n; i += TK_THREADS) {
          bool valid;
          const uint32_t k = key_of(i, valid);
          if (valid && (k & mask) == prefix) atomicAdd(&hist[(k >> sh) & (nb - 1)], 1u);
        }
        __syncthreads();
      }
      find_bin(hist, nb, remaining, wave_tot, found);
      prefix |= found[0] << sh;
      mask |= (uint32_t)(nb - 1) << sh;
      remaining -= found[1];
      __syncthreads();
    }
    T = prefix;
    r = remaining;
  }
  uint32_t gt_run = 0, eq_run = 0;
  const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
#pragma unroll 1
  for (int base = 0; base < n; base += TK_THREADS) {
    const int i = base + tid;
    bool valid = false;
    uint32_t k = 0;
    if (i < n) k = key_of(i, valid);
    const bool gt = valid && (all || k > T);
    const bool eq = valid && !all && k == T;
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
    if (gt || (eq && eq_before < r)) emit(gt_before + (eq_before < r ? eq_before : r), i, k);
    gt_run += gt_tot;
    eq_run += eq_tot;
    __syncthreads();
  }
}

}  // namespace asx
