// Selection for shapes with few (sequence, KV head) rows, in one launch (Sec. 4.3, cache-rank items (1)-(2)).
//
// When a layer has so few rows that the fused selection kernel would have to cut them into shares no longer than
// the budget, nothing can be pruned per share and the work is "score everything, then one top-k per row".  As two
// launches that costs a launch gap and a second ramp-up, which at these sizes (a few MiB of K) is a quarter of the
// time.  Here one grid does both: every workgroup scores its share of a row into the row's fp32 score buffer with
// device-scope stores and counts itself in; the workgroup that completes a row's count reads the row back with
// device-scope loads and selects (topk_regs_row).  The scores and therefore the selection are bit-identical to
// those of the two stand-alone kernels (same operands, same MFMA order).  With the launch gap gone the form also beats
// the fused kernel on mid-size shapes whose shares could prune (select_rows_preferred), and it takes the rows of a
// whole pack of layers in one grid (depth-wise packing, Sec. 4.3) like the fused kernel does.
#include "common.hpp"
#include "devscope.hpp"
#include "score_common.hpp"
#include "topk_common.hpp"

namespace asx {

static constexpr int SR_WAVES = TK_THREADS / 64;   // 16
static constexpr int SR_MAX_SHARE = 64 * SR_WAVES; // a lane holds one page id of its wavefront: 64 pages per wavefront

// SR_PG: pages a wavefront has in flight per iteration
template <int NSET, int NPT, int SR_PG>
__global__ __launch_bounds__(TK_THREADS) void select_rows_kernel(
    sel_tab tab, int B, float* __restrict__ scores, int64_t stride, int32_t* __restrict__ arrivals, int Hq, int Hkv,
    int G, int agg, int C, int max_pages, int share_pages) {
  __shared__ uint4 stage[SR_WAVES][256];   // per wavefront: one 4 KB page image
  __shared__ __attribute__((aligned(16))) uint32_t hist[4 * TK_BINS];
  __shared__ uint32_t bitmap[NPT * TK_THREADS / 32];
  __shared__ uint32_t wpre[NPT * TK_THREADS / 32];
  __shared__ __attribute__((aligned(16))) uint32_t xch[TK_XCH];
  __shared__ int last_sh;

  // grid z runs over (layer of the pack, sequence); the layer is uniform, so its table entry comes in through
  // scalar loads from the kernel arguments
  const int layer = blockIdx.z / B;
  const int b = blockIdx.z - layer * B, j = blockIdx.y;
  const uint16_t* __restrict__ k_pool = tab.k_pool[layer];
  const int32_t* __restrict__ block_table = tab.block_table[layer];
  const int32_t* __restrict__ ctx_lens = tab.ctx_lens[layer];
  const float* __restrict__ q_hat = tab.q_hat[layer];
  int32_t* __restrict__ sel_idx = tab.sel_idx[layer];
  int32_t* __restrict__ sel_cnt = tab.sel_cnt[layer];
  const int32_t last_page = tab.last_page[layer];
  const int64_t row = (int64_t)b * Hkv + j;                      // row of this layer's outputs
  const int64_t crow = ((int64_t)layer * B + b) * Hkv + j;        // row of the pack-wide score rows and counters
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int t = lane & 15, grp = lane >> 4;
  int N = clamp_row(ctx_lens[b], max_pages, stride);
  if (N > NPT * TK_THREADS) N = NPT * TK_THREADS;   // the host takes this route only when every row fits
  const int npages = (N + AS_PAGE - 1) / AS_PAGE;
  const int p0 = blockIdx.x * share_pages;
  const int p_end = p0 + share_pages < npages ? p0 + share_pages : npages;   // this workgroup scores pages [p0, p_end)
  float* srow = scores + crow * stride;

  if (p0 + wave * SR_PG < p_end) {   // wavefront-uniform: this wavefront has pages
    // lane l holds the page id of the wavefront's l-th page: iteration l / SR_PG, page l % SR_PG of it
    const int my_idx = p0 + (wave + SR_WAVES * (lane / SR_PG)) * SR_PG + lane % SR_PG;
    int32_t my_page = 0;
    if (my_idx < p_end) my_page = block_table[(int64_t)b * max_pages + my_idx];
    my_page = clamp_page(my_page, last_page);   // a corrupt table must not leave the pool

    bf16x8 aq[NSET][4];
    build_q_operand<NSET>(q_hat, b, j, Hq, G, agg, lane, aq);
    uint4* st = stage[wave];
#pragma unroll 1
    for (int it = 0; p0 + (wave + SR_WAVES * it) * SR_PG < p_end; ++it) {
      const int pg0 = p0 + (wave + SR_WAVES * it) * SR_PG;   // first page of this iteration
      uint4 kb[SR_PG][4];
#pragma unroll
      for (int pg = 0; pg < SR_PG; ++pg) {
        const int32_t page = __shfl(my_page, it * SR_PG + pg);   // pages beyond p_end read page 0's id: valid memory
        const uint4* base = reinterpret_cast<const uint4*>(k_pool + chunk_offset(page, Hkv, j));
#pragma unroll
        for (int i = 0; i < 4; ++i) kb[pg][i] = ld16<true>(base + i * 64 + lane);
      }
      float res[SR_PG];
#pragma unroll
      for (int pg = 0; pg < SR_PG; ++pg) {
#pragma unroll
        for (int i = 0; i < 4; ++i) st[lds_slot(4 * i + grp, t)] = kb[pg][i];
        __builtin_amdgcn_wave_barrier();
        uint4 kk[4];
#pragma unroll
        for (int m = 0; m < 4; ++m) kk[m] = st[lds_slot(t, cmap(grp, m))];
        __builtin_amdgcn_wave_barrier();
        float v = -INFINITY;
#pragma unroll
        for (int s = 0; s < NSET; ++s) {
          f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int m = 0; m < 4; ++m)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aq[s][m], __builtin_bit_cast(bf16x8, kk[m]), acc, 0, 0, 0);
          v = fmaxf(v, fold_rows(acc));
        }
        res[pg] = group_max(v);
      }
      // lane group g < SR_PG writes token t of page g
      const float outv = grp == 0 ? res[0] : grp == 1 ? res[1] : grp == 2 ? res[SR_PG > 2 ? 2 : 0] : res[SR_PG - 1];
      const int n = (pg0 + grp) * AS_PAGE + t;
      if (grp < SR_PG && pg0 + grp < p_end && n < N)
        st_dev(reinterpret_cast<uint32_t*>(srow) + n, __float_as_uint(outv + 0.0f));
    }
  }

  // every workgroup of the grid counts itself in, with or without pages
  if (!arrive_last(arrivals + crow, (int)gridDim.x, &last_sh)) return;
  const __amdgpu_buffer_rsrc_t rs = dev_rsrc(srow);
  topk_regs_row<NPT>([&](int i) { return __uint_as_float(ld_dev(rs, (uint32_t)i * 4u)); }, N, C, sel_idx + row * C,
                     sel_cnt + row, hist, bitmap, wpre, xch);
}

int select_rows_share_pages(const as_params* p, int n_layers) {
  // as many shares per row as keep the whole grid within one workgroup per compute unit, in whole workgroup
  // iterations (two pages per wavefront and iteration; four were measured too, for shares of 128 pages and more:
  // no faster, and the 16- and 32-key instances then spill)
  const int64_t rows = (int64_t)p->batch * p->n_kv_heads * n_layers;
  const int64_t pages = p->max_pages_per_seq > 0 ? p->max_pages_per_seq : 1;
  int64_t nshares = rows > 0 ? 256 / rows : 1;
  if (nshares < 1) nshares = 1;
  int64_t sp = (pages + nshares - 1) / nshares;
  const int64_t round = SR_WAVES * 2;
  sp = (sp + round - 1) / round * round;
  return sp > SR_MAX_SHARE ? 0 : (int)sp;
}

// Whether the one-launch form serves this shape (n_layers layers in one grid): plain aggregation with at most two
// operand sets (groups of up to 16 heads), rows that fit the register top-k, as many arrival counters as rows, and
// shares within what a wavefront's lanes can index.
bool select_rows_ok(const as_params* p, int n_layers) {
  const int G = p->n_kv_heads > 0 ? p->n_q_heads / p->n_kv_heads : 0;
  if (p->agg == AS_AGG_SOFTMAX_SUM) return false;
  if (!(p->agg == AS_AGG_SUM || G <= 16)) return false;
  if ((int64_t)p->max_pages_per_seq * AS_PAGE > 32 * TK_THREADS) return false;
  if ((int64_t)p->batch * p->n_kv_heads * n_layers > AS_SEL_COUNTERS) return false;
  if ((int64_t)p->batch * n_layers > 65535 || p->n_kv_heads > 65535) return false;
  return select_rows_share_pages(p, n_layers) > 0;
}

// Shapes where this form beats the fused selection kernel even though that kernel's shares could prune: at most
// half a chip's worth of rows (128) and at most 2^20 tokens in all (256 MiB of K), counted over the pack.  Measured,
// one-launch against fused, per as_score_topk call: batch 8 at 8192 tokens 35.0 / 41.8 us, batch 8 at 16384 61.2 / 64.5,
// batch 4 at 32768 69.1 / 72.4, batch 16 at 4096 32.9 / 38.5, 64/8 heads batch 16 at 8192 58.8 / 65.1; beyond either
// bound the fused kernel wins (batch 6 at 32768: 93.1 / 85.7, batch 32 at 4096: 56.5 / 54.0, batch 8 at 32768:
// 113.9 / 106.0).
bool select_rows_preferred(const as_params* p, int n_layers) {
  const int64_t rows = (int64_t)p->batch * p->n_kv_heads * n_layers;
  return rows <= 128 && rows * p->max_pages_per_seq * AS_PAGE <= ((int64_t)1 << 20);
}

// bytes of the pack-wide score rows
size_t select_rows_score_bytes(const as_params* p, int n_layers) {
  return (size_t)p->batch * p->n_kv_heads * n_layers * (size_t)p->max_pages_per_seq * AS_PAGE * sizeof(float);
}

// scores: [n_layers * batch * n_kv_heads][stride]; arrivals: one zeroed counter per such row
hipError_t launch_select_rows(const as_params* p, int n_layers, const sel_tab& tab, float* scores, int64_t stride,
                              int32_t* arrivals, hipStream_t s) {
  if (p->batch == 0) return hipSuccess;
  const int G = p->n_q_heads / p->n_kv_heads;
  const int sp = select_rows_share_pages(p, n_layers);
  const int nshares = p->max_pages_per_seq > 0 ? (p->max_pages_per_seq + sp - 1) / sp : 1;   // >= 1: every row is selected
  const dim3 grid(nshares, p->n_kv_heads, p->batch * n_layers);
  const int64_t longest = (int64_t)p->max_pages_per_seq * AS_PAGE;
#define AS_ROWS_LAUNCH(NSET_, NPT_)                                                                                  \
  hipLaunchKernelGGL((select_rows_kernel<NSET_, NPT_, 2>), grid, dim3(TK_THREADS), 0, s, tab, p->batch, scores,      \
                     stride, arrivals, p->n_q_heads, p->n_kv_heads, G, p->agg, p->budget, p->max_pages_per_seq, sp)
#define AS_ROWS_NPT(NSET_)                                      \
  do {                                                          \
    if (longest <= 4 * TK_THREADS) AS_ROWS_LAUNCH(NSET_, 4);    \
    else if (longest <= 8 * TK_THREADS) AS_ROWS_LAUNCH(NSET_, 8);   \
    else if (longest <= 16 * TK_THREADS) AS_ROWS_LAUNCH(NSET_, 16); \
    else AS_ROWS_LAUNCH(NSET_, 32);                             \
  } while (0)
  if (p->agg == AS_AGG_SUM || G <= 8) AS_ROWS_NPT(1);
  else AS_ROWS_NPT(2);
#undef AS_ROWS_NPT
#undef AS_ROWS_LAUNCH
  return hipGetLastError();
}

}  // namespace asx
