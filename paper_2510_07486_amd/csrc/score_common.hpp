// Device helpers shared by the key-scoring kernels: the MFMA operand layout of the predicted
// queries, the bank-conflict-free LDS image of a 16-token K page, and streaming loads.
#pragma once
#include "common.hpp"

namespace asx {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));


// Lane (t = lane & 15, grp = lane >> 4) of MFMA step m contracts the 8 dims of chunk
// `cmap(grp, m)`; the same map is used for the Q rows and the K columns, so any
// bijection onto 0..15 is valid.  Chunks 4*grp..4*grp+3 make each lane read 64
// contiguous bytes of its token.
__device__ __forceinline__ int cmap(int grp, int m) { return grp * 4 + m; }

// Builds the A operand (rows = hi/lo parts of the group's queries) for this lane.
//   row r = lane & 15:  head slot 2*(r>>2) + (r&1), part (r>>1)&1  (0 = hi, 1 = lo)
//   operand set s (of NSET, counted from s_base) holds head slots (s_base + s) * 8 .. + 7, wrapped modulo G
template <int NSET>
__device__ __forceinline__ void build_q_operand(const float* __restrict__ q_hat, int b, int j, int Hq, int G,
                                                int agg, int lane, bf16x8 (&aq)[NSET][4], int s_base = 0) {
  const int r = lane & 15, grp = lane >> 4;
  const int slot = 2 * (r >> 2) + (r & 1);
  const int part = (r >> 1) & 1;
  const float* qb = q_hat + ((int64_t)b * Hq + (int64_t)j * G) * AS_HEAD_DIM;
  // all loads of an operand set are issued before the first conversion (one round trip, not one per chunk)
#pragma unroll
  for (int s = 0; s < NSET; ++s) {
    float v[4][8];
    if (agg == AS_AGG_SUM) {
#pragma unroll
      for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int e = 0; e < 8; ++e) v[m][e] = 0.f;
      for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int m = 0; m < 4; ++m)
#pragma unroll
          for (int e = 0; e < 8; ++e) v[m][e] += qb[g * AS_HEAD_DIM + cmap(grp, m) * 8 + e];
      }
    } else {
      const int g = ((s_base + s) * 8 + slot) % G;
#pragma unroll
      for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int e = 0; e < 8; ++e) v[m][e] = qb[g * AS_HEAD_DIM + cmap(grp, m) * 8 + e];
    }
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      uint32_t w[4];
#pragma unroll
      for (int e = 0; e < 8; e += 2) {
        uint32_t h0 = f32_to_bf16_rne(v[m][e]), h1 = f32_to_bf16_rne(v[m][e + 1]);
        if (part) {
          h0 = f32_to_bf16_rne(v[m][e] - __uint_as_float(h0 << 16));
          h1 = f32_to_bf16_rne(v[m][e + 1] - __uint_as_float(h1 << 16));
        }
        w[e >> 1] = h0 | (h1 << 16);
      }
      uint4 u = make_uint4(w[0], w[1], w[2], w[3]);
      aq[s][m] = __builtin_bit_cast(bf16x8, u);
    }
  }
}

// 16-byte global load; NT marks the line as streaming (read once, do not keep in cache)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
template <bool NT>
__device__ __forceinline__ uint4 ld16(const void* p) {
  if (NT) {
    u32x4 r = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return make_uint4(r.x, r.y, r.z, r.w);
  }
  return *reinterpret_cast<const uint4*>(p);
}

// a lane's four accumulators -> max over its heads of (hi + lo)
__device__ __forceinline__ float fold_rows(const f32x4& d) { return fmaxf(d[0] + d[2], d[1] + d[3]); }
__device__ __forceinline__ float group_max(float v) {
  v = fmaxf(v, __shfl_xor(v, 16));
  v = fmaxf(v, __shfl_xor(v, 32));
  return v;
}

// LDS slot of chunk c of token t inside a 4 KB page image: rows of 256 B, 16-byte slots
// XOR-swizzled by the token so that both the row-wise (coalesced) fill and the
// column-wise MFMA-layout read touch all 64 banks exactly once per 16 lanes.
__device__ __forceinline__ int lds_slot(int t, int c) { return t * 16 + (c ^ t); }


}  // namespace asx
