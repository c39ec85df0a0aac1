// Device helpers shared by the top-k kernels: order-preserving score keys, an exact block-wide
// positional radix select with ordered emission, and exact marking of the best k among
// register-held (key, token) pairs (radix thresholds on the key, then on the token).
#pragma once
#include "common.hpp"

namespace asx {

static constexpr int TK_THREADS = 1024;   // workgroup size of the stand-alone top-k and merge kernels
static constexpr int TK_BINS = 4096;      // histogram bins they need (12-bit first pass)
static constexpr int TK_XCH = 16 + 128 + 2; // words of LDS exchange space block_select needs

// larger float -> larger key; -0 == +0; NaN -> 0 (below -inf)
__device__ __forceinline__ uint32_t score_key(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0u;
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Inclusive prefix sum over the 64 lanes of a wavefront with six DPP adds: Hillis-Steele
// inside each 16-lane row (row_shr 1, 2, 4, 8), then lane 15 of rows 0 / 2 into rows 1 / 3
// (row_bcast:15) and lane 31 into rows 2-3 (row_bcast:31).
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t x) {
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, false);
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, false);
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xf, 0xf, false);
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xf, 0xf, false);
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x142, 0xa, 0xf, false);
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x143, 0xc, 0xf, false);
  return x;
}

// Exclusive prefix, over (segment, wave) pairs in segment-major order, of NSEG*WAVES <= 64 words
// written by the waves of the workgroup to `words[seg * WAVES + wave]`: every wave loads them
// one per lane, scans with DPP and picks its own NSEG offsets with v_readlane.  Returns the
// grand total.  Call after a barrier that follows the writes.
template <int WAVES, int NSEG>
__device__ __forceinline__ uint32_t seg_wave_offsets(const uint32_t* words, int wave, uint32_t (&off)[NSEG]) {
  const int lane = threadIdx.x & 63;
  const uint32_t w = (lane < NSEG * WAVES) ? words[lane] : 0u;
  const uint32_t inc = wave_incl_scan(w);
  const uint32_t exc = inc - w;
  const int uw = __builtin_amdgcn_readfirstlane(wave);
#pragma unroll
  for (int sgm = 0; sgm < NSEG; ++sgm) off[sgm] = (uint32_t)__builtin_amdgcn_readlane((int)exc, sgm * WAVES + uw);
  return (uint32_t)__builtin_amdgcn_readlane((int)inc, 63);
}

// Finds the bin d (scanning from the highest bin down) with
//   sum_{d' > d} hist[d'] < remaining <= sum_{d' >= d} hist[d'];
// writes d and the count above it to found[0..1].  nb <= 4 * THREADS bins.
// wave_tot: 16 words of LDS.  SPREAD = 4: a bin is the sum of four consecutive words (16-byte aligned), see
// radix_threshold.
template <int THREADS, int SPREAD = 1>
__device__ __forceinline__ void find_bin(const uint32_t* hist, int nb, uint32_t remaining, uint32_t* wave_tot,
                                         uint32_t* found) {
  constexpr int WAVES = THREADS / 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int per = (nb + THREADS - 1) / THREADS;  // bins per thread, descending order
  uint32_t loc[4] = {0u, 0u, 0u, 0u};
  uint32_t mine = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int rb = tid * per + i;  // reversed bin index
    if (i < per && rb < nb) {
      if (SPREAD == 4) {
        const uint4 v = *reinterpret_cast<const uint4*>(hist + 4 * (nb - 1 - rb));
        loc[i] = v.x + v.y + v.z + v.w;
      } else {
        loc[i] = hist[nb - 1 - rb];
      }
    }
    mine += loc[i];
  }
  const uint32_t inc = wave_incl_scan(mine);
  if (lane == 63) wave_tot[wave] = inc;
  __syncthreads();
  uint32_t off[1];
  seg_wave_offsets<WAVES, 1>(wave_tot, wave, off);
  uint32_t excl = off[0] + inc - mine;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (i < per && excl < remaining && remaining <= excl + loc[i]) {
      found[0] = (uint32_t)(nb - 1 - (tid * per + i));
      found[1] = excl;
    }
    excl += loc[i];
  }
  __syncthreads();
}

// Exact selection of the `keep` largest of the valid keys at virtual positions 0..n-1, emitted
// in ascending position order; equal keys resolve to the lowest position.  Run by a whole
// workgroup of THREADS (512 or 1024) threads.
//   key4_of(i4, k, valid)  loads the keys of positions i4..i4+3 (i4 a multiple of 4; positions
//                          >= n must come back invalid); valid = false marks a hole
//   emit(pos, i, key)      called once per selected position, pos = its rank in ascending order
//   total = number of valid positions (>= keep); keep >= total selects everything.
//   hist0_ready: hist[] already holds the histogram of the top B0 key bits of all valid keys.
//   hist: 2^B0 words of LDS (B0 = 11 or 12);  xch: TK_XCH words of LDS.
// Radix select: three histogram passes (B0 bits, then the rest in two halves, most significant
// first) find the key T of the keep-th largest and r, how many keys equal to T are still to be
// taken.  Emission walks 16*THREADS positions per round as four segments; a thread owns four
// consecutive positions of each segment.  The output slot of a selected position is
// (#greater before it) + min(#equal before it, r): packed (greater | equal << 16) counts are
// scanned with DPP inside the wave and across (segment, wave) pairs after one barrier.
template <int THREADS, int B0, class Key4Fn, class EmitFn>
__device__ __forceinline__ void block_select(int n, int total, int keep, bool hist0_ready, Key4Fn key4_of,
                                             EmitFn emit, uint32_t* hist, uint32_t* xch) {
  constexpr int WAVES = THREADS / 64;
  constexpr int B1 = (32 - B0 + 1) / 2, B2 = 32 - B0 - B1;
  constexpr int SEG = 4 * THREADS;  // positions per segment
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  uint32_t* wave_tot = xch;   // [16]
  uint32_t* segw = xch + 16;  // [2][4 * WAVES <= 64] packed counts, double-buffered across rounds
  uint32_t* found = xch + 16 + 128;
  const bool all = keep >= total;
  uint32_t T = 0, r = 0;
  if (!all) {
    uint32_t prefix = 0, mask = 0, remaining = (uint32_t)keep;
#pragma unroll 1
    for (int pass = 0; pass < 3; ++pass) {
      const int width = pass == 0 ? B0 : pass == 1 ? B1 : B2;
      const int sh = pass == 0 ? 32 - B0 : pass == 1 ? B2 : 0;
      const int nb = 1 << width;
      if (!(pass == 0 && hist0_ready)) {
        for (int i = tid; i < nb; i += THREADS) hist[i] = 0;
        __syncthreads();
#pragma unroll 1
        for (int base = 0; base < n; base += 4 * SEG) {
          uint32_t k[4][4];
          bool v[4][4];
#pragma unroll
          for (int sgm = 0; sgm < 4; ++sgm) key4_of(base + sgm * SEG + 4 * tid, k[sgm], v[sgm]);
#pragma unroll
          for (int sgm = 0; sgm < 4; ++sgm)
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (v[sgm][e] && (k[sgm][e] & mask) == prefix) atomicAdd(&hist[(k[sgm][e] >> sh) & (nb - 1)], 1u);
        }
        __syncthreads();
      }
      find_bin<THREADS>(hist, nb, remaining, wave_tot, found);
      prefix |= found[0] << sh;
      mask |= (uint32_t)(nb - 1) << sh;
      remaining -= found[1];
    }
    T = prefix;
    r = remaining;
  }
  uint32_t gt_run = 0, eq_run = 0;
  int round = 0;
#pragma unroll 1
  for (int base = 0; base < n; base += 4 * SEG, ++round) {
    uint32_t k[4][4];
    bool v[4][4];
    uint32_t p[4], inc[4];
#pragma unroll
    for (int sgm = 0; sgm < 4; ++sgm) key4_of(base + sgm * SEG + 4 * tid, k[sgm], v[sgm]);
    uint32_t* x = segw + (round & 1) * 64;  // double-buffered: one barrier per round
#pragma unroll
    for (int sgm = 0; sgm < 4; ++sgm) {
      uint32_t c = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool gt = v[sgm][e] && (all || k[sgm][e] > T);
        const bool eq = v[sgm][e] && !all && k[sgm][e] == T;
        c += (gt ? 1u : 0u) + (eq ? 0x10000u : 0u);
      }
      p[sgm] = c;
      inc[sgm] = wave_incl_scan(c);
      if (lane == 63) x[sgm * WAVES + wave] = inc[sgm];
    }
    __syncthreads();
    uint32_t off[4];
    const uint32_t tot = seg_wave_offsets<WAVES, 4>(x, wave, off);  // fields stay below 2^15: no carry
#pragma unroll
    for (int sgm = 0; sgm < 4; ++sgm) {
      const uint32_t before = off[sgm] + inc[sgm] - p[sgm];
      uint32_t g = gt_run + (before & 0xffffu), q = eq_run + (before >> 16);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const bool gt = v[sgm][e] && (all || k[sgm][e] > T);
        const bool eq = v[sgm][e] && !all && k[sgm][e] == T;
        if (gt || (eq && q < r)) emit(g + (q < r ? q : r), base + sgm * SEG + 4 * tid + e, k[sgm][e]);
        g += gt ? 1u : 0u;
        q += eq ? 1u : 0u;
      }
    }
    gt_run += tot & 0xffffu;
    eq_run += tot >> 16;
  }
}

// adapts a per-position key function to the four-at-a-time interface
template <class KeyFn>
__device__ __forceinline__ auto key4_from_scalar(int n, KeyFn key_of) {
  return [=](int i4, uint32_t (&k)[4], bool (&v)[4]) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      v[e] = false;
      k[e] = 0;
      if (i4 + e < n) k[e] = key_of(i4 + e, v[e]);
    }
  };
}

// ---- exact selection over an unordered candidate buffer ----------------------------------------
// Candidates are (key, token) pairs in arbitrary order.  Tokens are unique, so the pairs are totally
// ordered by (key descending, token ascending) and "the best `keep`" is unique: every pair with
// key > T, plus the r pairs with the lowest tokens among those with key == T.

// Value of the want-th largest of the (up to NPT per thread) values held in registers, over the
// whole workgroup: three histogram passes (B0 bits, then the rest in two halves).  Returns T;
// `r` = how many values equal to T are still wanted, `ties` = how many values equal T.
// SPREAD = 4 (hist then has 4 << B0 words, 16-byte aligned): in the first pass, where every value is counted and
// scores crowd into a few dozen bins (sign, exponent, three mantissa bits), a bin is four words in four LDS banks and
// a lane adds to word lane % 4, so a wavefront's adds to one bin serialise a quarter as long.  (The 32-keys-per-thread
// top-k spills three dwords per lane with it and is still faster: 20.3 against 22.7 us for a 32768-token row.)
template <int THREADS, int B0, int NPT, int SPREAD = 1>
__device__ __forceinline__ uint32_t radix_threshold(const uint32_t (&val)[NPT], const bool (&ok)[NPT], uint32_t want,
                                                    uint32_t* hist, uint32_t* xch, uint32_t& r, uint32_t& ties) {
  constexpr int B1 = (32 - B0 + 1) / 2, B2 = 32 - B0 - B1;
  const int tid = threadIdx.x;
  uint32_t* wave_tot = xch;
  uint32_t* found = xch + 16 + 128;
  uint32_t prefix = 0, mask = 0, remaining = want;
#pragma unroll 1
  for (int pass = 0; pass < 3; ++pass) {
    const int width = pass == 0 ? B0 : pass == 1 ? B1 : B2;
    const int sh = pass == 0 ? 32 - B0 : pass == 1 ? B2 : 0;
    const int nb = 1 << width;
    if (SPREAD == 4 && pass == 0) {
      for (int i = tid; i < 4 * nb; i += THREADS) hist[i] = 0;
      __syncthreads();
#pragma unroll
      for (int e = 0; e < NPT; ++e)
        if (ok[e]) atomicAdd(&hist[4 * (val[e] >> sh) + (tid & 3)], 1u);
      __syncthreads();
      find_bin<THREADS, SPREAD>(hist, nb, remaining, wave_tot, found);
    } else {
    for (int i = tid; i < nb; i += THREADS) hist[i] = 0;
    __syncthreads();
#pragma unroll
    for (int e = 0; e < NPT; ++e)
      if (ok[e] && (val[e] & mask) == prefix) atomicAdd(&hist[(val[e] >> sh) & (nb - 1)], 1u);
    __syncthreads();
    find_bin<THREADS>(hist, nb, remaining, wave_tot, found);
    }
    prefix |= found[0] << sh;
    mask |= (uint32_t)(nb - 1) << sh;
    remaining -= found[1];
    if (pass == 2) ties = hist[found[0]];
  }
  __syncthreads();   // hist and found may be reused by the caller
  r = remaining;
  return prefix;
}

// Marks, among this thread's NPT candidates, the ones that belong to the best `keep` of the `total`
// candidates of the workgroup (keep < total).  Returns the key threshold T; tie_inv (optional) receives the
// cut among the pairs with key == T: such a pair is kept iff ~token >= *tie_inv (0 when every one of them is).
template <int THREADS, int B0, int NPT, int SPREAD = 1>
__device__ __forceinline__ uint32_t mark_best(const uint32_t (&key)[NPT], const int32_t (&tok)[NPT],
                                              const bool (&have)[NPT], int keep, uint32_t* hist, uint32_t* xch,
                                              bool (&sel)[NPT], uint32_t* tie_inv = nullptr) {
  uint32_t r, ties;
  const uint32_t T = radix_threshold<THREADS, B0, NPT, SPREAD>(key, have, (uint32_t)keep, hist, xch, r, ties);
  uint32_t I = 0;   // threshold on ~token among the pairs with key == T
  if (r < ties) {   // uniform: not every tie fits, the lowest tokens win
    uint32_t inv[NPT];
    bool tie[NPT];
#pragma unroll
    for (int e = 0; e < NPT; ++e) {
      inv[e] = ~(uint32_t)tok[e];
      tie[e] = have[e] && key[e] == T;
    }
    uint32_t r2, t2;
    I = radix_threshold<THREADS, B0, NPT, SPREAD>(inv, tie, r, hist, xch, r2, t2);
  }
#pragma unroll
  for (int e = 0; e < NPT; ++e)
    sel[e] = have[e] && (key[e] > T || (key[e] == T && ~(uint32_t)tok[e] >= I));
  if (tie_inv) *tie_inv = I;
  return T;
}

// Top-C of one row of at most NPT * TK_THREADS scores, by a whole workgroup of TK_THREADS threads.  The row's keys
// are read once, coalesced, into registers (token i sits in thread i % 1024: load(i) returns its score); the best
// min(C, N) are marked there (mark_best: radix thresholds on the key, ties by token) and put into ascending token
// order through a bitmap of the row (rank of a token = set bits below it).  A wavefront's 64 tokens of one
// register slot are two whole bitmap words, so the bitmap is written from ballots, without atomics.
//   out: C token indices (-1 beyond the count); cnt_out: the count
//   hist: 4 * TK_BINS words, 16-byte aligned; bitmap, wpre: NPT * TK_THREADS / 32 words each; xch: TK_XCH words (all LDS)
template <int NPT, class LoadFn>
__device__ __forceinline__ void topk_regs_row(LoadFn load, int N, int C, int32_t* __restrict__ out,
                                              int32_t* __restrict__ cnt_out, uint32_t* hist, uint32_t* bitmap,
                                              uint32_t* wpre, uint32_t* xch) {
  constexpr int WORDS = NPT * TK_THREADS / 32;   // bitmap words
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int keep = N < C ? N : C;
  if (tid == 0) *cnt_out = keep;
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
    raw[e] = load(have[e] ? tok[e] : N - 1);
  }
#pragma unroll
  for (int e = 0; e < NPT; ++e) {
    key[e] = have[e] ? score_key(raw[e]) : 0u;
    sel[e] = have[e];
  }
  if (keep < N) mark_best<TK_THREADS, 12, NPT, 4>(key, tok, have, keep, hist, xch, sel);
#pragma unroll
  for (int e = 0; e < NPT; ++e) {   // tokens e * 1024 + wave * 64 + 0..63: words e * 32 + 2 * wave and the next
    const unsigned long long m = __ballot(sel[e]);
    if (lane == 0) {
      bitmap[e * (TK_THREADS / 32) + 2 * wave] = (uint32_t)m;
      bitmap[e * (TK_THREADS / 32) + 2 * wave + 1] = (uint32_t)(m >> 32);
    }
  }
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

}  // namespace asx
