// Sparse decode attention on the matrix cores (Sec. 4.1; the 4*q*h*C term of Appendix B).
//
// A vector-ALU formulation (v_dot2c_f32_bf16 + DPP reductions) is issue-bound: about 75 instructions
// per gathered row and head group of 4, twice that at group size 8, which capped it near 4 TB/s and
// 2.4 TB/s when it was measured.  Here both contractions of a 32-token step run as v_mfma_f32_16x16x32_bf16 and the whole GQA
// group (up to 16 heads) shares every gathered row at no extra cost:
//   S^T[token][head] = K_tile[16 x 128] * Q^T[128 x 16]     (two 16-token tiles, 4 MFMAs each)
//   O[head][dim]    += P[16 x 32] * V[32 x 128]             (8 dim tiles, P split hi + lo)
// K and V rows arrive with the same coalesced 256-byte row gathers (16 lanes per row,
// non-temporal), are staged in per-wave LDS images and read back in operand layout: K with
// the XOR-swizzled 128-bit reads of the scoring kernel, V with ds_read_b64_tr_b16, the
// transposing LDS read that hands a lane four tokens of one dim.  The S^T accumulator layout
// (lane = head, 4 tokens per tile and lane group) IS the A-operand layout of P for the PV
// product, so probabilities go from registers straight back into the matrix core.  Each
// wavefront keeps its own online-softmax state (no barrier in the loop); the waves of a workgroup
// (four or eight, chosen by the host so that about eight wavefronts per compute unit each get the
// same number of steps) merge once at the end.  A row that is not split across workgroups is
// finished there (normalised, rounded to bf16, lse written); otherwise the workgroup writes one
// partial (m, l, o) per head and split, which attn_combine_kernel (attn.hip) reduces.
#include "common.hpp"
#include "score_common.hpp"

namespace asx {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_m __attribute__((ext_vector_type(4)));

static constexpr int AM_STEP = 32;          // tokens per wave step
static constexpr int AM_VROW = 288;         // bytes per V row in LDS (256 + 32: spreads the tr reads over banks)
static constexpr int AM_KIMG = 256;         // uint4 per 16-token K image
static constexpr int AM_WAVE_LDS = AM_STEP * AM_VROW;   // 9 KB per wave: the V rows of a step; the 4 KB K tile image
                                                        // of the S phase lives in the same bytes (three workgroups per CU)

__device__ __forceinline__ uint4 am_ld16_nt(const void* p) {
  const u32x4_m r = __builtin_nontemporal_load(reinterpret_cast<const u32x4_m*>(p));
  return make_uint4(r.x, r.y, r.z, r.w);
}

// Measured and not kept: a second register set per wavefront, so that the rows of the next step are requested before
// the current one is computed (252 registers, two steps = 32 KB in flight per wavefront).  Batch 32, 32/8 heads,
// budget 2048: 51.2 us against 49.1 us.  While all workgroups run the kernel already moves 6.3 TB/s (the rate of
// full attention over long contexts); what is left is the spread between the fastest and the slowest compute unit
// at the end (38.7 / 42.6 / 48.0 us for the first, median and last workgroup), which more loads in flight do not shorten.
// WAVES = 4: 37 KB of LDS, three workgroups fit a compute unit; WAVES = 8: 73 KB, two fit.  (Padding the LDS
// request so that a compute unit cannot take more than its even share of a grid was measured: nothing gained
// alone, and beside the selection kernel, whose workgroups own a compute unit each, attention then waits for
// whole compute units instead of packing into the free ones: batch 16, 64/8 heads, 216 -> 253 us per layer-step.)
template <int WAVES> struct am_shape {
  static constexpr int LDS = WAVES * AM_WAVE_LDS < WAVES * 16 * AS_HEAD_DIM * 4 ? WAVES * 16 * AS_HEAD_DIM * 4 : WAVES * AM_WAVE_LDS;
  // Block-table rows of up to this many pages are copied into LDS at the start of the kernel, in the same round trip as
  // the first token indices: the chain index -> page id -> row address then has two dependent global loads, not three.
  static constexpr int BT_CAP = WAVES == 8 ? 4096 : 2048;   // 16 KB / 8 KB (three four-wavefront workgroups still fit a compute unit)
};

template <int WAVES>
__global__ __launch_bounds__(WAVES * 64, WAVES == 4 ? 3 : 1) void attn_mfma_kernel(
    const uint16_t* __restrict__ k_pool, const uint16_t* __restrict__ v_pool, const int32_t* __restrict__ block_table,
    const int32_t* __restrict__ ctx_lens, const uint16_t* __restrict__ q, const int32_t* __restrict__ sel_idx,
    const int32_t* __restrict__ sel_cnt, const int32_t* __restrict__ sel_ctx_lens, float* __restrict__ part_o,
    float* __restrict__ part_ml, uint16_t* __restrict__ out, float* __restrict__ lse, int Hq, int Hkv, int G, int C,
    int max_pages, float sm_scale, int nsplit, int list_len, int32_t last_page, wg_timeline tl) {
  const long long t_in = timeline_begin(tl);
  __shared__ __attribute__((aligned(16))) unsigned char lds_raw[am_shape<WAVES>::LDS];
  __shared__ float m_sh[WAVES][16], l_sh[WAVES][16], l_fin[16];
  __shared__ __attribute__((aligned(16))) int32_t bt_sh[am_shape<WAVES>::BT_CAP];

  // a workgroup serves up to 16 heads of a group: larger groups (MQA) take several head blocks per KV head
  const int hblocks = (G + 15) / 16;
  const int b = blockIdx.z, j = blockIdx.y / hblocks, g0 = (blockIdx.y % hblocks) * 16, split = blockIdx.x;
  const int Gb = G - g0 < 16 ? G - g0 : 16;   // heads of this block
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int t = lane & 15, grp = lane >> 4;   // operand coordinates: row / column index, k group
  const int slot = grp, c = t;                // gather coordinates: row within a 4-row load, 16-byte chunk

  const int32_t* idx_row = sel_idx + ((int64_t)b * Hkv + j) * C;
  // lane l (< 32, upper half mirrors) resolves token l of a 32-token step of this wave
  // Balanced partition of the logical token list: split s starts at s * list_len / nsplit rounded down to a
  // whole 32-token step, the last split also takes whatever lies beyond list_len (the dense tail).
  const int t_begin = (int)((int64_t)split * list_len / nsplit) & ~(AM_STEP - 1);
  const int t_next = (int)((int64_t)(split + 1) * list_len / nsplit) & ~(AM_STEP - 1);
  auto step_token = [&](int step) -> int { return t_begin + step * AM_STEP + (lane & 31); };
  auto fetch_index = [&](int step) -> int {
    const int ti = step_token(step);
    return (ti < C) ? idx_row[ti] : 0;
  };
  const int raw_first = fetch_index(w);       // speculative: validated once the lengths are known
  const bool bt_in_lds = max_pages <= am_shape<WAVES>::BT_CAP;   // uniform
  if (bt_in_lds) {                            // the whole table row of the sequence (it is max_pages entries long)
    const int32_t* src = block_table + (int64_t)b * max_pages;
    for (int i = tid; i < max_pages; i += WAVES * 64) bt_sh[i] = src[i];
  }

  const int N = clamp_ctx(ctx_lens[b], max_pages);
  int cnt = sel_cnt ? sel_cnt[b * Hkv + j] : 0;   // no selection arrays: dense attention over [0, N)
  cnt = clamp_count(cnt, C, N);   // an empty sequence has nothing to select from
  int tail0 = sel_idx ? (sel_ctx_lens ? sel_ctx_lens[b] : N) : 0;
  tail0 = clamp_tail(tail0, N);
  const int L = cnt + (N - tail0);
  const int t_end = (split == nsplit - 1) ? L : (t_next < L ? t_next : L);
  const int64_t pbase = ((int64_t)b * Hq + (int64_t)j * G + g0) * nsplit + split;  // + g * nsplit per head
  const bool direct = nsplit == 1;                                            // the whole row is this workgroup's
  const int64_t obase = (int64_t)b * Hq + (int64_t)j * G + g0;                // + g per head
  if (t_begin >= t_end) {                                                     // nothing here: mark empty
    if (direct) {
      for (int i = tid; i < Gb * AS_HEAD_DIM; i += WAVES * 64) out[obase * AS_HEAD_DIM + i] = 0;
      if (lse && tid < Gb) lse[obase + tid] = -INFINITY;
    } else if (tid < Gb) {
      part_ml[(pbase + (int64_t)tid * nsplit) * 2 + 0] = -INFINITY;
      part_ml[(pbase + (int64_t)tid * nsplit) * 2 + 1] = 0.f;
    }
  } else {
  const int nsteps = (t_end - t_begin + AM_STEP - 1) / AM_STEP;

  // Q^T as the B operand of S^T = K Q^T: lane (head t, k group grp), step m holds the 8 dims of
  // chunk cmap(grp, m) of head t (zero for t >= G)
  bf16x8 qb[4];
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    uint4 u = make_uint4(0, 0, 0, 0);
    if (t < Gb) u = *reinterpret_cast<const uint4*>(q + ((int64_t)b * Hq + (int64_t)j * G + g0 + t) * AS_HEAD_DIM + cmap(grp, m) * 8);
    qb[m] = __builtin_bit_cast(bf16x8, u);
  }

  unsigned char* my_lds = lds_raw + w * AM_WAVE_LDS;
  uint4* kimg = reinterpret_cast<uint4*>(my_lds);                       // [256] swizzled 16-byte slots, one 16-token tile
  unsigned char* vimg = my_lds;                                         // [32][AM_VROW], written once S is done
  const int32_t* bt_row = block_table + (int64_t)b * max_pages;

  auto page_of = [&](int step, int raw) -> uint32_t {
    const int ti = step_token(step);
    int n = 0;
    if (ti < t_end) n = (ti < cnt) ? raw : tail0 + (ti - cnt);
    n = clamp_token(n, N);                                              // keeps a bad index inside the sequence
    int32_t pg = bt_in_lds ? bt_sh[n >> 4] : bt_row[n >> 4];
    pg = clamp_page(pg, last_page);                                     // a corrupt table must not leave the pool
    return ((uint32_t)pg << 4) | (uint32_t)(n & 15);
  };

  f32x4 o_acc[8];                       // O[head 4*grp+i][dim 16*nt + t]
#pragma unroll
  for (int nt = 0; nt < 8; ++nt) o_acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f; // softmax state of head t (replicated in the 4 lane groups)

  if (bt_in_lds) __syncthreads();       // the table row has landed (uniform branch; every wave of a workgroup with tokens is here)
  uint32_t my_pk = (w < nsteps) ? page_of(w, raw_first) : 0u;
#pragma unroll 1
  for (int step = w; step < nsteps; step += WAVES) {
    // next step's index is requested now, its page id after this step's rows are on their way
    const bool more = step + WAVES < nsteps;
    int raw_next = 0;
    if (more) raw_next = fetch_index(step + WAVES);
    // ---- gather the 32 K and V rows of the step (8 loads of 4 rows each) ----
    uint4 kr[8], vr[8];
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const uint32_t pk = __shfl(my_pk, it * 4 + slot);
      const int64_t off = chunk_offset((int32_t)(pk >> 4), Hkv, j) + (int64_t)(pk & 15) * AS_HEAD_DIM + c * 8;
      kr[it] = am_ld16_nt(k_pool + off);
      vr[it] = am_ld16_nt(v_pool + off);
    }
    uint32_t pk_next = 0;
    if (more) pk_next = page_of(step + WAVES, raw_next);
    // ---- S^T = K Q^T for the two tiles (K goes through one 16-token image, tile after tile): lane (head t, grp) gets tokens tile*16 + 4*grp + i ----
    float s[8];
#pragma unroll
    for (int tile = 0; tile < 2; ++tile) {
#pragma unroll
      for (int it = 0; it < 4; ++it) kimg[lds_slot(it * 4 + slot, c)] = kr[tile * 4 + it];
      __builtin_amdgcn_wave_barrier();
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        const uint4 kk = kimg[lds_slot(t, cmap(grp, m))];
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kk), qb[m], acc, 0, 0, 0);
      }
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int tok = t_begin + step * AM_STEP + tile * 16 + 4 * grp + i;
        s[tile * 4 + i] = (tok < t_end) ? acc[i] * sm_scale : -INFINITY;
      }
    }
    // ---- the K image is dead: stage V (padded rows) over it ----
#pragma unroll
    for (int it = 0; it < 8; ++it) *reinterpret_cast<uint4*>(vimg + (it * 4 + slot) * AM_VROW + c * 16) = vr[it];
    __builtin_amdgcn_wave_barrier();
    // ---- online softmax of head t over the step's 32 tokens ----
    float mx = s[0];
#pragma unroll
    for (int e = 1; e < 8; ++e) mx = fmaxf(mx, s[e]);
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);                               // finite: the step holds a valid token
    const float scl = (m_run == -INFINITY) ? 0.f : __expf(m_run - m_new);
    float p[8], ps = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      p[e] = __expf(s[e] - m_new);                                      // exp(-inf) = 0 for masked tokens
      ps += p[e];
    }
    ps += __shfl_xor(ps, 16);
    ps += __shfl_xor(ps, 32);
    l_run = l_run * scl + ps;
    m_run = m_new;
    // P as A operand (row = head t, k slots e = tokens tile (e>>2), 4*grp + (e&3)), split hi + lo
    uint32_t ph[4], pl[4];
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      const uint32_t h0 = f32_to_bf16_rne(p[e]), h1 = f32_to_bf16_rne(p[e + 1]);
      const uint32_t l0 = f32_to_bf16_rne(p[e] - __uint_as_float(h0 << 16));
      const uint32_t l1 = f32_to_bf16_rne(p[e + 1] - __uint_as_float(h1 << 16));
      ph[e >> 1] = h0 | (h1 << 16);
      pl[e >> 1] = l0 | (l1 << 16);
    }
    const bf16x8 pa_hi = __builtin_bit_cast(bf16x8, make_uint4(ph[0], ph[1], ph[2], ph[3]));
    const bf16x8 pa_lo = __builtin_bit_cast(bf16x8, make_uint4(pl[0], pl[1], pl[2], pl[3]));
    // rescale O: this lane holds heads 4*grp + i, whose factors live in lanes (t = head)
    float rs[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) rs[i] = __shfl(scl, 4 * grp + i);
    // ---- O += P V: V^T fragments through the transposing LDS read ----
    // lane rho = t of a 16-lane block points at token (tile*16 + 4*grp + (rho>>2)), dims 16*nt + 4*(rho&3);
    // it receives dims 16*nt + t of tokens tile*16 + 4*grp + 0..3
    const unsigned char* vbase = vimg + (4 * grp + (t >> 2)) * AM_VROW + (t & 3) * 8;
#pragma unroll
    for (int nt = 0; nt < 8; ++nt) {
      const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) s16x4*)(vbase + nt * 32));
      const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) s16x4*)(vbase + 16 * AM_VROW + nt * 32));
      struct { s16x4 a, b; } pr = {v0, v1};
      const bf16x8 vb = __builtin_bit_cast(bf16x8, pr);
      f32x4 acc = o_acc[nt];
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] *= rs[i];
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa_hi, vb, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa_lo, vb, acc, 0, 0, 0);
      o_acc[nt] = acc;
    }
    __builtin_amdgcn_wave_barrier();
    my_pk = pk_next;
  }

  // ---- merge the waves: common max per head, rescale, sum ----
  if (grp == 0) {
    m_sh[w][t] = m_run;
    l_sh[w][t] = l_run;
  }
  __syncthreads();                      // also: every wave is done with its LDS images
  float M = -INFINITY, Ls = 0.f;
#pragma unroll
  for (int ww = 0; ww < WAVES; ++ww) M = fmaxf(M, m_sh[ww][t]);
#pragma unroll
  for (int ww = 0; ww < WAVES; ++ww) Ls += (m_sh[ww][t] == -INFINITY) ? 0.f : l_sh[ww][t] * __expf(m_sh[ww][t] - M);
  const float wgt = (m_run == -INFINITY) ? 0.f : __expf(m_run - M);   // this wave's factor for head t
  float* red = reinterpret_cast<float*>(lds_raw);                      // [WAVES][16 heads][128] fp32
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float f = __shfl(wgt, 4 * grp + i);
    const int head = 4 * grp + i;
    if (head < Gb) {                     // rows of the zero-padded heads are never read
#pragma unroll
      for (int nt = 0; nt < 8; ++nt) red[(w * 16 + head) * AS_HEAD_DIM + nt * 16 + t] = o_acc[nt][i] * f;
    }
  }
  if (w == 0 && grp == 0) l_fin[t] = Ls;   // the merged normaliser of head t
  __syncthreads();
  for (int i = tid; i < Gb * AS_HEAD_DIM; i += WAVES * 64) {
    const int g = i / AS_HEAD_DIM, d = i % AS_HEAD_DIM;
    float v = 0.f;
#pragma unroll
    for (int ww = 0; ww < WAVES; ++ww) v += red[(ww * 16 + g) * AS_HEAD_DIM + d];
    if (direct) {
      const float lg = l_fin[g];
      out[(obase + g) * AS_HEAD_DIM + d] = (uint16_t)f32_to_bf16_rne(lg > 0.f ? v / lg : 0.f);
    } else {
      part_o[(pbase + (int64_t)g * nsplit) * AS_HEAD_DIM + d] = v;
    }
  }
  if (w == 0 && grp == 0 && t < Gb) {
    if (direct) {
      if (lse) lse[obase + t] = (Ls > 0.f) ? M + logf(Ls) : -INFINITY;
    } else {
      part_ml[(pbase + (int64_t)t * nsplit) * 2 + 0] = M;
      part_ml[(pbase + (int64_t)t * nsplit) * 2 + 1] = Ls;
    }
  }
  }   // this split had tokens
  timeline_end(tl, t_in);
}

hipError_t launch_attn_mfma(const as_params* p, const as_kv_view* kv, const uint16_t* q, const int32_t* sel_idx,
                            const int32_t* sel_cnt, const int32_t* sel_ctx_lens, float* part_o, float* part_ml,
                            uint16_t* out, float* lse, int nsplit, int waves, int list_len, wg_timeline tl,
                            hipStream_t s) {
  const int G = p->n_q_heads / p->n_kv_heads;
  dim3 grid(nsplit, p->n_kv_heads * ((G + 15) / 16), p->batch);
#define AS_ATTN_LAUNCH(WAVES_)                                                                                        \
  hipLaunchKernelGGL(attn_mfma_kernel<WAVES_>, grid, dim3(WAVES_ * 64), 0, s,                                         \
                     reinterpret_cast<const uint16_t*>(kv->k_pool), reinterpret_cast<const uint16_t*>(kv->v_pool),    \
                     kv->block_table, kv->ctx_lens, q, sel_idx, sel_cnt, sel_ctx_lens, part_o, part_ml, out, lse,     \
                     p->n_q_heads, p->n_kv_heads, G, sel_idx ? p->budget : 0, p->max_pages_per_seq, p->sm_scale,      \
                     nsplit, list_len, (int32_t)(kv->num_pages > 0 ? kv->num_pages - 1 : 0), tl)
  if (waves == 8) AS_ATTN_LAUNCH(8); else AS_ATTN_LAUNCH(4);
#undef AS_ATTN_LAUNCH
  return hipGetLastError();
}

}  // namespace asx
