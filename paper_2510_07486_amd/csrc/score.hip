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

namespace asx {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

static constexpr int SC_PPW = 8;            // pages per wave
static constexpr int SC_TP = 4 * SC_PPW;    // pages per 256-thread block

// Lane (t = lane & 15, grp = lane >> 4) of MFMA step m contracts the 8 dims of chunk
// `cmap(grp, m)`; the same map is used for the Q rows and the K columns, so any
// bijection onto 0..15 is valid.  Chunks 4*grp..4*grp+3 make each lane read 64
// contiguous bytes of its token.
__device__ __forceinline__ int cmap(int grp, int m) { return grp * 4 + m; }

// Builds the A operand (rows = hi/lo parts of the group's queries) for this lane.
//   row r = lane & 15:  head slot 2*(r>>2) + (r&1), part (r>>1)&1  (0 = hi, 1 = lo)
template <int NSET>
__device__ __forceinline__ void build_q_operand(const float* __restrict__ q_hat, int b, int j, int Hq, int G,
                                                int agg, int lane, bf16x8 (&aq)[NSET][4]) {
  const int r = lane & 15, grp = lane >> 4;
  const int slot = 2 * (r >> 2) + (r & 1);
  const int part = (r >> 1) & 1;
  const float* qb = q_hat + ((int64_t)b * Hq + (int64_t)j * G) * AS_HEAD_DIM;
#pragma unroll
  for (int s = 0; s < NSET; ++s) {
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const int c = cmap(grp, m);
      float v[8];
      if (agg == AS_AGG_SUM) {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = 0.f;
        for (int g = 0; g < G; ++g) {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += qb[g * AS_HEAD_DIM + c * 8 + e];
        }
      } else {
        const int g = (s * 8 + slot) % G;
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = qb[g * AS_HEAD_DIM + c * 8 + e];
      }
      uint32_t w[4];
#pragma unroll
      for (int e = 0; e < 8; e += 2) {
        uint32_t h0 = f32_to_bf16_rne(v[e]), h1 = f32_to_bf16_rne(v[e + 1]);
        if (part) {
          h0 = f32_to_bf16_rne(v[e] - __uint_as_float(h0 << 16));
          h1 = f32_to_bf16_rne(v[e + 1] - __uint_as_float(h1 << 16));
        }
        w[e >> 1] = h0 | (h1 << 16);
      }
      uint4 u = make_uint4(w[0], w[1], w[2], w[3]);
      aq[s][m] = __builtin_bit_cast(bf16x8, u);
    }
  }
}

// a lane's four accumulators -> max over its heads of (hi + lo)
__device__ __forceinline__ float fold_rows(const f32x4& d) { return fmaxf(d[0] + d[2], d[1] + d[3]); }
__device__ __forceinline__ float group_max(float v) {
  v = fmaxf(v, __shfl_xor(v, 16));
  v = fmaxf(v, __shfl_xor(v, 32));
  return v;
}

// Variant 0: K is read from global memory directly in the MFMA B layout (lane = token,
// 64 contiguous bytes per lane across the four steps).
template <int NSET>
__global__ __launch_bounds__(256) void score_mfma_direct(const uint16_t* __restrict__ k_pool,
                                                         const int32_t* __restrict__ block_table,
                                                         const int32_t* __restrict__ ctx_lens,
                                                         const float* __restrict__ q_hat, float* __restrict__ scores,
                                                         int64_t stride, int Hq, int Hkv, int G, int agg,
                                                         int max_pages) {
  const int b = blockIdx.z, j = blockIdx.y;
  const int N = ctx_lens[b];
  const int npages = (N + AS_PAGE - 1) / AS_PAGE;
  const int p0 = blockIdx.x * SC_TP;
  if (p0 >= npages) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int t = lane & 15, grp = lane >> 4;
  const int pw = p0 + wave * SC_PPW;  // first page of this wave
  if (pw >= npages) return;

  int32_t my_page = 0;
  if (lane < SC_PPW && pw + lane < npages) my_page = block_table[(int64_t)b * max_pages + pw + lane];

  bf16x8 aq[NSET][4];
  build_q_operand<NSET>(q_hat, b, j, Hq, G, agg, lane, aq);

  float* srow = scores + ((int64_t)b * Hkv + j) * stride;
#pragma unroll 1
  for (int qd = 0; qd < SC_PPW / 4; ++qd) {
    if (pw + qd * 4 >= npages) break;
    uint4 kb[4][4];
#pragma unroll
    for (int pg = 0; pg < 4; ++pg) {
      const int32_t page = __shfl(my_page, qd * 4 + pg);
      const uint16_t* base = k_pool + chunk_offset(page, Hkv, j) + t * AS_HEAD_DIM;
#pragma unroll
      for (int m = 0; m < 4; ++m) kb[pg][m] = *reinterpret_cast<const uint4*>(base + cmap(grp, m) * 8);
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

hipError_t launch_score(int variant, const as_params* p, const as_kv_view* kv, const float* q_hat, float* scores,
                        int64_t stride, hipStream_t s) {
  if (p->batch == 0 || p->max_pages_per_seq == 0) return hipSuccess;
  const int G = p->n_q_heads / p->n_kv_heads;
  const uint16_t* kp = reinterpret_cast<const uint16_t*>(kv->k_pool);
  dim3 grid((p->max_pages_per_seq + SC_TP - 1) / SC_TP, p->n_kv_heads, p->batch);
  const bool two = (p->agg != AS_AGG_SUM) && G > 8;
  (void)variant;
  if (two)
    hipLaunchKernelGGL(score_mfma_direct<2>, grid, dim3(256), 0, s, kp, kv->block_table, kv->ctx_lens, q_hat, scores,
                       stride, p->n_q_heads, p->n_kv_heads, G, p->agg, p->max_pages_per_seq);
  else
    hipLaunchKernelGGL(score_mfma_direct<1>, grid, dim3(256), 0, s, kp, kv->block_table, kv->ctx_lens, q_hat, scores,
                       stride, p->n_q_heads, p->n_kv_heads, G, p->agg, p->max_pages_per_seq);
  return hipGetLastError();
}

}  // namespace asx
