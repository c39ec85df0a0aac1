// Fused key scoring + top-k for one layer-step (Alg. 1 step 7 followed by the cache rank's
// top-k, Sec. 4.3 items (1)-(2)), without ever writing the per-token scores to HBM
// (interleaving 4 B/token of score writes with the K stream costs about 15 % of the read rate).
//
// Each (sequence, KV head) row is cut into shares; one workgroup owns a share.  It streams the
// K pages (coalesced non-temporal 128-bit loads, transposed through a per-wave 4 KB LDS image into
// the MFMA operand layout, see score_common.hpp) and appends (order-preserving 32-bit key, token)
// pairs to an unordered candidate buffer in LDS (one LDS atomic per wavefront reserves the slots).
// When the buffer is nearly full, a prune keeps exactly the best C pairs (radix threshold on the
// key over register-held candidates, ties resolved by a second radix threshold on the token) and
// its threshold then filters the stream: a token seen later can only matter if it beats the worst
// kept pair (a larger key, or the same key and a lower token index), so the inflow decays like
// C / tokens-seen and a 32768-token share typically needs one prune and the final selection,
// instead of one selection per 8192 tokens.  Because tokens are unique, the pairs are totally
// ordered by (key descending, token ascending): the result depends neither on the order in which
// wavefronts appended nor on the order in which the share's pages are visited, and every workgroup
// starts its walk at a different page (regularly laid out caches would otherwise have all
// workgroups, advancing in lockstep, on the same memory channels).  The final selection is put into ascending token order
// through a bitmap of the share (rank of a token = set bits below it) and goes out: straight into
// sel_idx when the row has a single share, otherwise as (key, token) candidates that a small merge
// kernel reduces to the row's top-C.  The top-C of a row is contained in the union of the top-C of
// its parts and every level resolves equal keys to the lowest token, so the result equals a full
// sort of the row.  HBM traffic: one read of K plus 8 B per candidate of a multi-share row.
//
// Pruning needs C <= half the buffer (2048 / 4096 pairs for 512 / 1024 threads); larger budgets
// use shares that fit the buffer whole.  The first sub-slice of a long share has a pseudo-random
// shorter length so that the prune phases of different compute units do not coincide.
#include "common.hpp"
#include "predict_common.hpp"
#include "score_common.hpp"
#include "topk_common.hpp"
#include "devscope.hpp"

namespace asx {

template <int THREADS> struct fs_shape {
  static constexpr int WAVES = THREADS / 64;
  static constexpr int CAP = THREADS * 8;                 // candidate buffer, (key, token) pairs
  static constexpr int RCAP = THREADS * 4;                // largest budget served by pruning (a prune frees >= CAP / 2)
  static constexpr int B0 = 11;                           // bits of the first radix pass
  static constexpr int BINS = 1 << B0;
  static constexpr int SHARE_CAP = THREADS * (THREADS == 1024 ? 64 : 32);   // tokens per share: the bitmap that orders
                                                          // a share's selection has one bit per token (8 KB / 2 KB)
};
static constexpr int FS_PG = 2;             // pages a wave loads per iteration (8 KB in flight per wave)
static constexpr int FS_PG4 = 4;            // ... of the four-operand-set instance: its 512-thread workgroups leave a compute
                                            // unit with 8 wavefronts instead of 16, so each keeps twice the bytes in flight
static constexpr int FS_MAX_SLICES = 1024;  // shares per row the merge kernel can index (one per thread)

static int device_cus() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
      cus = n;
    else
      cus = 256;
  }
  return cus;
}

// Picks how many shares a row is cut into with a small cost model (microseconds), evaluated for
// the longest context the block table allows.  Workgroups run in rounds of one resident set;
// a full round streams at the chip's rate (HBM-bound, T_SHARED per token and workgroup), a
// partly filled last round at the rate one compute unit can pull alone (T_ALONE).  Every share
// pays a fixed start-up, its selections (typically one prune and the final one when it is longer than
// the candidate buffer) and, when a row has several shares, its candidates through HBM plus the merge kernel.  Constants are measured on MI355X.
static select_plan plan_for(const as_params* p, int thr, int n_layers) {
  select_plan pl;
  const int64_t rows = (int64_t)p->batch * p->n_kv_heads * n_layers;
  const int64_t max_ctx = (int64_t)p->max_pages_per_seq * AS_PAGE;
  const int ssub = thr * 8, rcap = thr * 4, share_cap = thr == 1024 ? fs_shape<1024>::SHARE_CAP : fs_shape<512>::SHARE_CAP;
  const int64_t slots = (int64_t)device_cus() * (thr == 1024 ? 1 : 2);
  const double T_SHARED = 9.5e-3 * 256.0 / (double)device_cus() * (thr == 1024 ? 1.0 : 2.0);
  const double T_ALONE = 7.2e-3 * (thr == 1024 ? 1.0 : 2.0);
  const double T_FIX = 7.0, T_SELECT = 5.0, T_MERGE = 12.0, T_CAND_PER_MIB = 2.1;
  double best = 1e30;
  int64_t best_sl = 256;
  for (int64_t st = 1; st <= 4096; st = st < 8 ? st + 1 : st + st / 4) {
    int64_t sl = (max_ctx + st - 1) / st;
    sl = (sl + 63) / 64 * 64;
    if (sl < 256) sl = 256;
    if (sl > share_cap) sl = share_cap;
    if (p->budget > rcap && sl > ssub) sl = ssub;   // pruning needs C <= half the buffer: else one sub-slice per share
    const int64_t nsh = (max_ctx + sl - 1) / sl > 0 ? (max_ctx + sl - 1) / sl : 1;
    if (nsh > FS_MAX_SLICES) continue;
    const int64_t nsub = sl > ssub ? 2 : 1;         // typical selections per share: one prune + the final one
    double t = 0.0;
    for (int64_t left = rows * nsh; left > 0; left -= slots) {
      const double fill = (double)(left < slots ? left : slots) / (double)slots;
      const double per_tok = T_SHARED * fill > T_ALONE ? T_SHARED * fill : T_ALONE;
      t += (double)sl * per_tok + T_FIX + (double)nsub * T_SELECT;
    }
    if (nsh > 1) {
      const double ccap = (double)(p->budget < sl ? p->budget : sl);
      t += (double)rows * (double)nsh * ccap * 8.0 / 1048576.0 * T_CAND_PER_MIB;
      t += T_MERGE * (double)((rows + device_cus() - 1) / device_cus()) * (1.0 + (double)nsh * ccap / 16384.0);
    }
    if (t < best) {
      best = t;
      best_sl = sl;
    }
    if (sl == 256) break;
  }
  pl.slice_len = (int)best_sl;
  pl.nslices = (int)((max_ctx + best_sl - 1) / best_sl);
  if (pl.nslices < 1) pl.nslices = 1;
  pl.ccap = p->budget < pl.slice_len ? p->budget : pl.slice_len;
  return pl;
}

// Groups above 16 heads (MQA) keep four or eight MFMA operand sets in registers: that needs the register budget
// of the 512-thread shape (two waves per SIMD).
static int slice_threads_for(const as_params* p) {
  const int G = p->n_q_heads / p->n_kv_heads;
  return (p->agg != AS_AGG_SUM && G > 16) ? 512 : 1024;
}

select_plan plan_select(const as_params* p, int n_layers) { return plan_for(p, slice_threads_for(p), n_layers); }

// false when no share plan fits: a budget above half the candidate buffer forces buffer-sized shares, and the merge
// kernel indexes at most FS_MAX_SLICES of them per row (contexts beyond 4-8 million tokens at such budgets)
bool select_plan_ok(const as_params* p, int n_layers) { return plan_select(p, n_layers).nslices <= FS_MAX_SLICES; }

// A single layer with so few rows that the plan cuts them into shares not much longer than the budget: the shares
// can discard little or nothing, most tokens would travel to the merge kernel as 8-byte candidates and the merge
// would be a top-k over (nearly) the whole row.  The stand-alone stages do the same work with 4-byte scores and
// keys held in registers (batch 1, 16384 tokens, budget 2048: 10 + 17 us against 15 + 22 us; batch 1, 4096 tokens,
// budget 256: 9 + 9 us against 15 + 9 us).  Chosen when at least half of a row would reach the merge and the row
// fits the register top-k; rows beyond that only when no share could discard anything at all.
bool select_prefers_stages(const as_params* p) {
  if (p->agg == AS_AGG_SOFTMAX_SUM) return false;   // needs the row-wide normalisers of the fused passes
  const select_plan pl = plan_select(p, 1);
  if (pl.nslices <= 1) return false;
  if (pl.ccap == pl.slice_len) return true;
  const int64_t max_ctx = (int64_t)p->max_pages_per_seq * AS_PAGE;
  return max_ctx <= 32 * TK_THREADS && (int64_t)pl.nslices * pl.ccap * 2 >= max_ctx;
}

// bytes of the candidate arrays (rows cut into several shares) and, behind them, of the per-share (max, sum)
// pairs of the softmax-normalised aggregation
static size_t cand_bytes(const as_params* p, const select_plan& pl, int n_layers) {
  if (pl.nslices <= 1 || pl.nslices > FS_MAX_SLICES) return 0;   // one share per row, or no share plan at all
  const size_t rows = (size_t)p->batch * p->n_kv_heads * n_layers;
  return (rows * pl.nslices * ((size_t)pl.ccap * 8 + 4) + 15) / 16 * 16;
}
static size_t lse_bytes(const as_params* p, const select_plan& pl, int n_layers) {
  if (p->agg != AS_AGG_SOFTMAX_SUM || pl.nslices > FS_MAX_SLICES) return 0;
  return (size_t)p->batch * p->n_q_heads * n_layers * pl.nslices * sizeof(float2);
}

size_t select_workspace_bytes(const as_params* p, int n_layers) {
  const select_plan pl = plan_select(p, n_layers);
  return cand_bytes(p, pl, n_layers) + lse_bytes(p, pl, n_layers);
}

// ---- rows cut into several shares, merged inside the slice kernel ---------------------------------
// The last workgroup of a row to finish merges the row's per-share candidates itself (merge_row_lds below)
// instead of a second launch doing it; the hand-over between workgroups is the one of devscope.hpp.
// Top-C of one row from its shares' candidates (token order within and across shares), at most 8 * THREADS of
// them in all: the candidates are compacted into LDS, marked in registers (mark_best) and compacted in order.
//   row_key / row_idx: [nslices][ccap] candidates of the row; row_cnt: [nslices]
//   lkey / lidx: 8 * THREADS words of LDS each; cnt_sh / pre_sh: nslices words each; hist: 2^B0 words
template <int THREADS, int B0>
__device__ __forceinline__ void merge_row_lds(const uint32_t* row_key, const int32_t* row_idx, const int32_t* row_cnt,
                                              int nslices, int ccap, int C, int32_t* __restrict__ out_idx,
                                              int32_t* __restrict__ out_cnt, uint32_t* lkey, int32_t* lidx,
                                              int32_t* cnt_sh, int32_t* pre_sh, uint32_t* hist, uint32_t* xch) {
  constexpr int NPT = 8, WAVES = THREADS / 64;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(row_key), 0, 0x7fffffff, 0x00020000);
  const __amdgpu_buffer_rsrc_t ri = __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t*>(row_idx), 0, 0x7fffffff, 0x00020000);
  const __amdgpu_buffer_rsrc_t rc = __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t*>(row_cnt), 0, 0x7fffffff, 0x00020000);
  // counts and their exclusive prefix over shares: thread s owns share s, THREADS shares per round
  uint32_t run = 0;
  for (int s0 = 0; s0 < nslices; s0 += THREADS) {
    const int sl = s0 + tid;
    const uint32_t mine = sl < nslices ? ld_dev(rc, (uint32_t)sl * 4u) : 0u;
    const uint32_t inc = wave_incl_scan(mine);
    __syncthreads();
    if (lane == 63) xch[wave] = inc;
    __syncthreads();
    uint32_t woff[1];
    const uint32_t tot = seg_wave_offsets<WAVES, 1>(xch, wave, woff);
    if (sl < nslices) {
      cnt_sh[sl] = (int32_t)mine;
      pre_sh[sl] = (int32_t)(run + woff[0] + inc - mine);
    }
    run += tot;
  }
  __syncthreads();
  const int total = (int)run;                 // <= nslices * ccap <= NPT * THREADS (host check)
  const int keep = total < C ? total : C;
  const int nvirt = nslices * ccap;
  if (keep > 0) {
#pragma unroll 1
    for (int base = 0; base < nvirt; base += NPT * THREADS) {
      uint32_t k[NPT];
      int32_t ix[NPT];
      int pos[NPT];
#pragma unroll
      for (int u = 0; u < NPT; ++u) {   // every load issued before the first is used; empty slots re-read candidate 0
        const int v = base + u * THREADS + tid;
        const int sl = v < nvirt ? v / ccap : 0;
        const int i = v - sl * ccap;
        const bool ok = v < nvirt && i < cnt_sh[sl];
        pos[u] = ok ? pre_sh[sl] + i : -1;
        k[u] = ld_dev(rk, (uint32_t)(ok ? v : 0) * 4u);
        ix[u] = (int32_t)ld_dev(ri, (uint32_t)(ok ? v : 0) * 4u);
      }
#pragma unroll
      for (int u = 0; u < NPT; ++u)
        if (pos[u] >= 0) {
          lkey[pos[u]] = k[u];
          lidx[pos[u]] = ix[u];
        }
    }
    __syncthreads();
    uint32_t key[NPT];
    int32_t tok[NPT];
    bool have[NPT], sel[NPT];
#pragma unroll
    for (int e = 0; e < NPT; ++e) {
      const int i = tid * NPT + e;              // < NPT * THREADS
      have[e] = i < total;
      const uint32_t k = lkey[i];
      const int32_t tk = lidx[i];
      key[e] = have[e] ? k : 0u;
      tok[e] = have[e] ? tk : 0;
      sel[e] = have[e];
    }
    if (keep < total) mark_best<THREADS, B0, NPT>(key, tok, have, keep, hist, xch, sel);
    uint32_t c = 0;
#pragma unroll
    for (int e = 0; e < NPT; ++e) c += sel[e] ? 1u : 0u;
    const uint32_t sinc = wave_incl_scan(c);
    __syncthreads();                 // every thread has its candidates in registers: lidx becomes the output stage
    if (lane == 63) xch[wave] = sinc;
    __syncthreads();
    uint32_t soff[1];
    seg_wave_offsets<WAVES, 1>(xch, wave, soff);
    uint32_t at = soff[0] + sinc - c;
#pragma unroll
    for (int e = 0; e < NPT; ++e)
      if (sel[e]) lidx[at++] = tok[e];
    __syncthreads();
    for (int i = tid; i < keep; i += THREADS) out_idx[i] = lidx[i];
  }
  for (int i = keep + tid; i < C; i += THREADS) out_idx[i] = -1;
  if (tid == 0) *out_cnt = keep;
}

// MODE 0: scores are the max (or the pre-summed query's logit) over the group.  MODES 1 and 2 are the two passes
// of the softmax-normalised aggregation s[n] = sum_g exp(scale * l[g][n] - LSE_g): pass 1 streams the share and
// leaves one (max, sum) pair per head in lse_part, pass 2 merges the pairs of all shares of its row into LSE_g
// and then selects exactly like mode 0 with s[n] as the score.
// PRED: the query predictor (Sec. 4.2) runs in the prologue: up to eight wavefronts at a time each predict one head
// of the group from its window (predict_wave, fp64; their scratch borrows the page images and the candidate
// buffer, which are idle until the stream starts) and leave q_hat in LDS, where the MFMA operand is built from.
template <int NSET, int FS_THREADS, int PG, int MODE, bool PRED>
__global__ __launch_bounds__(FS_THREADS) void select_slice_kernel(
    const sel_tab tab, int B, int Hq, int Hkv, int G, int agg, int max_pages, int share_len, int nshares, int C,
    int ccap, uint32_t* __restrict__ cand_key, int32_t* __restrict__ cand_idx, int32_t* __restrict__ cand_cnt,
    float sm_scale, float2* __restrict__ lse_part, int32_t* __restrict__ arrivals) {
  using shape = fs_shape<FS_THREADS>;
  constexpr int FS_WAVES = shape::WAVES, CAP = shape::CAP, NPT = CAP / FS_THREADS;
  constexpr int FS_B0 = shape::B0, FS_BINS = shape::BINS, BM_WORDS = shape::SHARE_CAP / 32;
  constexpr int BM_WPT = (BM_WORDS + FS_THREADS - 1) / FS_THREADS;   // consecutive bitmap words a thread scans
  static_assert(BM_WORDS <= FS_BINS, "the prefixes of the bitmap words alias hist");
  __shared__ __attribute__((aligned(16))) uint32_t c_key[CAP];   // candidate buffer: keys ...
  __shared__ __attribute__((aligned(16))) int32_t c_tok[CAP];    // ... and their token indices
  __shared__ uint4 stage[FS_WAVES][256];  // per-wave page images while streaming; ordered output at the end
  __shared__ uint32_t hist[FS_BINS];      // radix histograms; prefix counts of the bitmap words at the end
  __shared__ uint32_t bitmap[BM_WORDS];   // one bit per token of the share: orders the selected tokens
  __shared__ __attribute__((aligned(16))) uint32_t xch[TK_XCH];
  __shared__ uint32_t c_cnt;              // candidates in the buffer
  // Groups of 33-64 heads (eight operand sets), plain selection: the sets stay in LDS and a wavefront holds one half
  // (four sets, 64 registers) at a time; the pages of an iteration are kept in registers and scored against one
  // half, the other half is loaded, the same pages are scored again, and the next iteration starts with the half
  // that is already loaded: one half-load (16 KB per wavefront) per PG pages, and room for PG = 4 pages in flight.
  constexpr bool HALF = NSET == 8 && MODE == 0;
  constexpr int NREG = HALF ? 4 : NSET;   // operand sets held in registers
  __shared__ uint4 aq_lds[HALF ? 8 * 4 * 64 : 1];
  __shared__ int last_sh;                 // this workgroup completed its row's arrival count

  // Grid = (KV head, layer * B + batch slot, share).  Consecutive workgroup ids go round-robin over the 8 XCDs
  // and, inside an XCD, over its shader arrays: any index whose upper values are empty for short
  // sequences (the share) must vary slowest, or the workgroups that do have work pile up on half
  // of the compute units.
  const long long t_in = timeline_begin(tab.timeline);
  const int j = blockIdx.x, sh = blockIdx.z;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int t = lane & 15, grp = lane >> 4;
  // Longest sequences first: workgroups are dispatched in blockIdx order, so the y-th dispatched
  // batch slot takes the sequence of length rank y (ties by index) and the short ones fill the tail.
  const int layer = blockIdx.y / B;   // uniform: the layer's table entry comes in through scalar loads
  const int slot = blockIdx.y - layer * B;
  const uint16_t* __restrict__ k_pool = tab.k_pool[layer];
  const int32_t* __restrict__ block_table = tab.block_table[layer];
  const int32_t* __restrict__ ctx_lens = tab.ctx_lens[layer];
  const float* __restrict__ q_hat = tab.q_hat[layer];
  int32_t* __restrict__ sel_idx = tab.sel_idx[layer];
  int32_t* __restrict__ sel_cnt = tab.sel_cnt[layer];
  const int32_t last_page = tab.last_page[layer];
  int b = slot;
  if (tid == 0) c_cnt = 0;
  if (B > 1 && B <= CAP) {
    int32_t* lens = c_tok;
    for (int i = tid; i < B; i += FS_THREADS) lens[i] = ctx_lens[i];
    __syncthreads();
    for (int u = tid; u < B; u += FS_THREADS) {
      const int lu = lens[u];
      int rank = 0;
      for (int v = 0; v < B; ++v) rank += (lens[v] > lu) || (lens[v] == lu && v < u);
      if (rank == slot) xch[0] = (uint32_t)u;
    }
    __syncthreads();
    b = __builtin_amdgcn_readfirstlane((int)xch[0]);   // uniform: keeps the row's addresses in scalar registers
  }
  __syncthreads();
  const int64_t row = (int64_t)b * Hkv + j;                      // row of this layer's outputs
  const int64_t crow = ((int64_t)layer * B + b) * Hkv + j;        // row of the pack-wide candidate arrays
  const int N = clamp_ctx(ctx_lens[b], max_pages);
  const int tok0 = sh * share_len;
  int n_share = N - tok0;
  n_share = n_share < 0 ? 0 : (n_share > share_len ? share_len : n_share);
  const bool final_out = (nshares == 1);
  // rows with several shares and an arrival counter: called by every workgroup of the row once its candidates (and
  // their count) are stored; the one that completes the count merges the row
  auto arrive_and_merge = [&]() {
    if (!arrive_last(arrivals + crow, nshares, &last_sh)) return;
    static_assert(BM_WORDS >= 512, "share counts and their prefixes live in the bitmap words");
    merge_row_lds<FS_THREADS, FS_B0>(cand_key + crow * nshares * (int64_t)ccap, cand_idx + crow * nshares * (int64_t)ccap,
                                     cand_cnt + crow * nshares, nshares, ccap, C, sel_idx + row * C, sel_cnt + row,
                                     c_key, c_tok, reinterpret_cast<int32_t*>(bitmap),
                                     reinterpret_cast<int32_t*>(bitmap) + BM_WORDS / 2, hist, xch);
  };
  if (MODE == 1 && n_share == 0) {
    if (tid < G) lse_part[(crow * nshares + sh) * G + tid] = make_float2(-INFINITY, 0.f);
    timeline_end(tab.timeline, t_in);
    return;
  }
  if (n_share == 0) {
    if (final_out) {
      for (int i = tid; i < C; i += FS_THREADS) sel_idx[row * C + i] = -1;
      if (tid == 0) sel_cnt[row] = 0;
    } else if (arrivals) {
      if (tid == 0) st_dev(&cand_cnt[crow * nshares + sh], 0);
      arrive_and_merge();
    } else if (tid == 0) {
      cand_cnt[crow * nshares + sh] = 0;
    }
    timeline_end(tab.timeline, t_in);
    return;
  }

  // The share is streamed in sub-slices that are known to fit the free part of the candidate buffer.
  // The first one of a long share has a pseudo-random length, so that the prune phases of different
  // compute units do not coincide (all of them pausing their K stream at once would idle the HBM).
  int n_sub = (n_share + AS_PAGE - 1) / AS_PAGE * AS_PAGE;   // whole pages; tokens beyond the share are masked
  if (n_sub > CAP) {
    const uint32_t wg = (uint32_t)((blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x);
    n_sub = CAP / 2 + 64 * (int)((wg * 2654435761u >> 16) % (CAP / 128));
  }
  const int share_pages = (n_share + AS_PAGE - 1) / AS_PAGE;
  const int n_pad = share_pages * AS_PAGE;   // the share in whole pages: what the stream walks
  const int32_t* bt_row = block_table + (int64_t)b * max_pages + tok0 / AS_PAGE;
  // The pages of the share are visited in rotated order, starting at a page that differs from workgroup to
  // workgroup (the selection does not depend on the order in which tokens are seen): workgroups that
  // advance in lockstep over regularly laid out sequences would otherwise keep hitting the same memory channels.
  // (the KV heads of a sequence share the start: their workgroups then read the eight 4 KB chunks of one page
  // record at about the same time)
  const uint32_t rot_id = (uint32_t)(blockIdx.z * gridDim.y + blockIdx.y);
  const int rot = (int)((rot_id * 2246822519u >> 12) % (uint32_t)share_pages);
  auto real_page = [&](int vpage) -> int {   // vpage < share_pages
    const int rp = vpage + rot;
    return rp >= share_pages ? rp - share_pages : rp;
  };
  // lane l keeps the page id of (iteration l / PG, page l % PG) of the sub-slice that starts at token `pos`
  // (a sub-slice has at most CAP tokens = 64 pages per wave)
  auto load_pages = [&](int pos) -> int32_t {
    const int lp = ((lane / PG) * FS_WAVES + wave) * PG + (lane % PG);
    const int pi = pos / AS_PAGE + lp;
    const int32_t pg = pi < share_pages ? bt_row[real_page(pi)] : 0;
    return clamp_page(pg, last_page);   // a corrupt table must not leave the pool
  };
  int pos = 0;
  int32_t my_page = load_pages(0);

  bf16x8 aq[NREG][4];
  if constexpr (HALF) {
    static_assert(FS_WAVES == 8, "wavefront w builds operand set w");
    bf16x8 one[1][4];
    build_q_operand<1>(q_hat, b, j, Hq, G, agg, lane, one, wave);
#pragma unroll
    for (int m = 0; m < 4; ++m) aq_lds[(wave * 4 + m) * 64 + lane] = __builtin_bit_cast(uint4, one[0][m]);
    __syncthreads();
#pragma unroll
    for (int s2 = 0; s2 < 4; ++s2)
#pragma unroll
      for (int m = 0; m < 4; ++m) aq[s2][m] = __builtin_bit_cast(bf16x8, aq_lds[(s2 * 4 + m) * 64 + lane]);
  } else if constexpr (PRED) {
    static_assert(MODE == 0 && NSET <= 2 && FS_THREADS == 1024, "hist holds q_hat of up to 16 heads; eight scratch areas");
    static_assert(sizeof(predict_lds<16>) <= 16384, "four areas in the page images, two each in the candidate arrays");
    float* qh_sh = reinterpret_cast<float*>(hist);   // [G][128]; hist is next written by a prune, behind a barrier
    unsigned char* area = wave < 4 ? reinterpret_cast<unsigned char*>(&stage[0][0]) + wave * 16384
                          : wave < 6 ? reinterpret_cast<unsigned char*>(c_key) + (wave - 4) * 16384
                                     : reinterpret_cast<unsigned char*>(c_tok) + (wave - 6) * 16384;
    const int W = tab.pred_window;
#pragma unroll 1
    for (int h0 = 0; h0 < G; h0 += 8) {
      const int h = h0 + wave;
      if (wave < 8 && h < G) {
        const int64_t bh = (int64_t)b * Hq + (int64_t)j * G + h;
        predict_wave<16, true>(reinterpret_cast<const uint32_t*>(tab.q_win[layer] + bh * W * AS_HEAD_DIM),
                               reinterpret_cast<const uint32_t*>(tab.q_cur[layer] + bh * AS_HEAD_DIM), W, tab.pred_eps,
                               tab.pred_beta, tab.pred_single, *reinterpret_cast<predict_lds<16>*>(area),
                               qh_sh + h * AS_HEAD_DIM);
      }
    }
    __syncthreads();
    build_q_operand<NREG>(qh_sh, 0, 0, 0, G, agg, lane, aq);   // the group's rows start at qh_sh
    __syncthreads();   // the scratch areas become page images and candidates again
  } else {
    build_q_operand<NREG>(q_hat, b, j, Hq, G, agg, lane, aq);
  }
  int cur_half = 0;   // HALF: which half of the operand sets aq holds

  // softmax modes: the lane's accumulators of operand set s belong to heads s*8 + 2*grp and s*8 + 2*grp + 1
  float hm[NSET][2], hl[NSET][2];   // pass 1: running (max, sum of exp) of this lane's token column; pass 2: hm = LSE
#pragma unroll
  for (int s = 0; s < NSET; ++s)
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      hm[s][e] = MODE == 2 ? INFINITY : -INFINITY;
      hl[s][e] = 0.f;
    }
  if (MODE == 2) {
    // LSE of the group's heads over the whole row: wave w merges the per-share pairs of heads w, w + WAVES, ...
    float* lse_sh = reinterpret_cast<float*>(hist);
    for (int h = wave; h < G; h += FS_WAVES) {
      float m = -INFINITY;
      for (int s2 = lane; s2 < nshares; s2 += 64) m = fmaxf(m, lse_part[(crow * nshares + s2) * G + h].x);
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
      float l = 0.f;
      for (int s2 = lane; s2 < nshares; s2 += 64) {
        const float2 v = lse_part[(crow * nshares + s2) * G + h];
        l += v.y > 0.f ? v.y * __expf(v.x - m) : 0.f;
      }
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) l += __shfl_xor(l, o);
      if (lane == 0) lse_sh[h] = m + __logf(l);
    }
    __syncthreads();
#pragma unroll
    for (int s = 0; s < NSET; ++s)
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int h = s * 8 + 2 * grp + e;
        if (h < G) hm[s][e] = lse_sh[h];
      }
    // hist is next written by a prune, which every wave reaches only through the barrier after its first sub-slice
  }

  uint4* st = stage[wave];
  bool have_tau = false;   // after the first prune: only keys above tau can still make the best C
  uint32_t tau = 0, tau_inv = 0;   // a pair (tau, token) still matters iff ~token >= tau_inv
  int cnt = 0;             // candidates in the buffer (uniform copy of c_cnt)
#pragma unroll 1
  while (true) {
    // ---- stream the sub-slice: score, filter, append ----
    const int npages_sub = (n_sub + AS_PAGE - 1) / AS_PAGE;
    const int ngroups = (npages_sub + PG - 1) / PG;   // a wave takes PG pages per iteration
#pragma unroll 1
    for (int it = 0; wave + FS_WAVES * it < ngroups; ++it) {
      const int q = wave + FS_WAVES * it;
      uint4 kb[PG][4];
#pragma unroll
      for (int pg = 0; pg < PG; ++pg) {
        const int32_t page = __shfl(my_page, it * PG + pg);
        const uint4* base = reinterpret_cast<const uint4*>(k_pool + chunk_offset(page, Hkv, j));
#pragma unroll
        for (int i = 0; i < 4; ++i) kb[pg][i] = ld16<true>(base + i * 64 + lane);
      }
      float res[PG];
      if constexpr (HALF) {
        uint4 kkh[PG][4];
        float vpart[PG];
#pragma unroll
        for (int pg = 0; pg < PG; ++pg) {
#pragma unroll
          for (int i = 0; i < 4; ++i) st[lds_slot(4 * i + grp, t)] = kb[pg][i];
          __builtin_amdgcn_wave_barrier();
#pragma unroll
          for (int m = 0; m < 4; ++m) kkh[pg][m] = st[lds_slot(t, cmap(grp, m))];
          __builtin_amdgcn_wave_barrier();
          float v = -INFINITY;
#pragma unroll
          for (int s2 = 0; s2 < 4; ++s2) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int m = 0; m < 4; ++m)
              acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aq[s2][m], __builtin_bit_cast(bf16x8, kkh[pg][m]), acc, 0, 0, 0);
            v = fmaxf(v, fold_rows(acc));
          }
          vpart[pg] = v;
        }
        cur_half ^= 1;
#pragma unroll
        for (int s2 = 0; s2 < 4; ++s2)
#pragma unroll
          for (int m = 0; m < 4; ++m)
            aq[s2][m] = __builtin_bit_cast(bf16x8, aq_lds[((cur_half * 4 + s2) * 4 + m) * 64 + lane]);
#pragma unroll
        for (int pg = 0; pg < PG; ++pg) {
          float v = vpart[pg];
#pragma unroll
          for (int s2 = 0; s2 < 4; ++s2) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int m = 0; m < 4; ++m)
              acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aq[s2][m], __builtin_bit_cast(bf16x8, kkh[pg][m]), acc, 0, 0, 0);
            v = fmaxf(v, fold_rows(acc));
          }
          res[pg] = group_max(v);
        }
      } else {
#pragma unroll
      for (int pg = 0; pg < PG; ++pg) {
#pragma unroll
        for (int i = 0; i < 4; ++i) st[lds_slot(4 * i + grp, t)] = kb[pg][i];
        __builtin_amdgcn_wave_barrier();
        uint4 kk[4];
#pragma unroll
        for (int m = 0; m < 4; ++m) kk[m] = st[lds_slot(t, cmap(grp, m))];
        __builtin_amdgcn_wave_barrier();
        float v = MODE == 0 ? -INFINITY : 0.f;
        const int vp_pg = pos / AS_PAGE + q * PG + pg;             // this page, in visiting order
        const bool tok_ok = vp_pg < share_pages && real_page(vp_pg < share_pages ? vp_pg : 0) * AS_PAGE + t < n_share;
#pragma unroll
        for (int s = 0; s < NSET; ++s) {
          f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int m = 0; m < 4; ++m)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aq[s][m], __builtin_bit_cast(bf16x8, kk[m]), acc, 0, 0, 0);
          if (MODE == 0) {
            v = fmaxf(v, fold_rows(acc));
          } else {
            const float x[2] = {(acc[0] + acc[2]) * sm_scale, (acc[1] + acc[3]) * sm_scale};
#pragma unroll
            for (int e = 0; e < 2; ++e) {
              if (MODE == 1) {
                if (tok_ok) {
                  const float mn = fmaxf(hm[s][e], x[e]);
                  hl[s][e] = hl[s][e] * __expf(hm[s][e] - mn) + __expf(x[e] - mn);
                  hm[s][e] = mn;
                }
              } else {
                v += __expf(x[e] - hm[s][e]);   // hm = +inf for head slots beyond the group: contributes 0
              }
            }
          }
        }
        if (MODE == 0) {
          res[pg] = group_max(v);
        } else if (MODE == 2) {
          v += __shfl_xor(v, 16);
          v += __shfl_xor(v, 32);
          res[pg] = v;
        } else {
          res[pg] = 0.f;
        }
      }
      }   // !HALF
      if (MODE == 1) continue;   // pass 1 keeps no candidates
      float outv = res[0];
#pragma unroll
      for (int pg = 1; pg < PG; ++pg) outv = grp == pg ? res[pg] : outv;
      const int vp = pos / AS_PAGE + q * PG + grp;  // page of this lane's token, in visiting order
      const int rel = real_page(vp < share_pages ? vp : 0) * AS_PAGE + t;   // token within the share
      const uint32_t key = score_key(outv + 0.0f);
      const bool pass = grp < PG && vp < share_pages && rel < n_share &&
                        (!have_tau || key > tau || (key == tau && ~(uint32_t)(tok0 + rel) >= tau_inv));
      const uint64_t m = __ballot(pass);
      if (m) {   // uniform: one LDS atomic per wave reserves the slots
        const int leader = __ffsll((long long)m) - 1;
        uint32_t base = 0;
        if (lane == leader) base = atomicAdd(&c_cnt, (uint32_t)__popcll(m));
        base = (uint32_t)__builtin_amdgcn_readlane((int)base, leader);
        if (pass) {
          const uint32_t at = base + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
          c_key[at] = key;
          c_tok[at] = tok0 + rel;
        }
      }
    }
    pos += n_sub;
    const bool last = pos >= n_pad;
    if (!last) my_page = load_pages(pos);   // page ids of the next sub-slice travel during the barrier / prune
    if (MODE == 1) {                        // no candidate buffer to watch: whole-buffer-sized sub-slices, no barrier
      if (last) break;
      n_sub = (n_pad - pos) < CAP ? (n_pad - pos) : CAP;
      continue;
    }
    __syncthreads();
    cnt = (int)c_cnt;
    if (last) break;
    if (CAP - cnt < CAP / 4 && C < cnt) {
      // ---- prune: keep the best C (C <= CAP / 2 < cnt here), unordered, and raise the filter threshold ----
      uint32_t key[NPT];
      int32_t tok[NPT];
      bool have[NPT], sel[NPT];
#pragma unroll
      for (int e = 0; e < NPT; ++e) {
        const int i = tid + e * FS_THREADS;      // < CAP: the read needs no guard, stale slots are masked
        have[e] = i < cnt;
        const uint32_t k = c_key[i];
        const int32_t tk = c_tok[i];
        key[e] = have[e] ? k : 0u;
        tok[e] = have[e] ? tk : 0;
      }
      tau = mark_best<FS_THREADS, FS_B0, NPT>(key, tok, have, C, hist, xch, sel, &tau_inv);
      have_tau = true;
      if (tid == 0) c_cnt = 0;
      __syncthreads();     // every thread holds its candidates in registers: the buffer can be rewritten
#pragma unroll
      for (int e = 0; e < NPT; ++e) {
        const uint64_t m = __ballot(sel[e]);
        if (m) {
          const int leader = __ffsll((long long)m) - 1;
          uint32_t base = 0;
          if (lane == leader) base = atomicAdd(&c_cnt, (uint32_t)__popcll(m));
          base = (uint32_t)__builtin_amdgcn_readlane((int)base, leader);
          if (sel[e]) {
            const uint32_t at = base + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
            c_key[at] = key[e];
            c_tok[at] = tok[e];
          }
        }
      }
      __syncthreads();
      cnt = (int)c_cnt;    // == C
    }
    __syncthreads();   // every wave holds the same count before the next sub-slice starts to append
    const int room = (CAP - cnt) & ~63;
    if (room <= 0) break;   // unreachable while the host plan keeps C <= CAP / 2 for multi-sub-slice shares
    n_sub = (n_pad - pos) < room ? (n_pad - pos) : room;
  }

  if (MODE == 1) {
    // ---- merge the token columns (16 lanes), then the waves, and leave one (max, sum) pair per head ----
    float2* red = reinterpret_cast<float2*>(hist);   // [FS_WAVES][64 heads]
#pragma unroll
    for (int s = 0; s < NSET; ++s)
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        float m = hm[s][e], l = hl[s][e];
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) {
          const float m2 = __shfl_xor(m, o), l2 = __shfl_xor(l, o);
          const float mn = fmaxf(m, m2);
          l = (m == -INFINITY ? 0.f : l * __expf(m - mn)) + (m2 == -INFINITY ? 0.f : l2 * __expf(m2 - mn));
          m = mn;
        }
        const int h = s * 8 + 2 * grp + e;
        if (t == 0 && h < 64) red[wave * 64 + h] = make_float2(m, l);
      }
    __syncthreads();
    if (tid < G) {
      float m = -INFINITY;
      for (int w2 = 0; w2 < FS_WAVES; ++w2) m = fmaxf(m, red[w2 * 64 + tid].x);
      float l = 0.f;
      for (int w2 = 0; w2 < FS_WAVES; ++w2) {
        const float2 v = red[w2 * 64 + tid];
        l += v.x == -INFINITY ? 0.f : v.y * __expf(v.x - m);
      }
      lse_part[(crow * nshares + sh) * G + tid] = make_float2(m, l);
    }
    timeline_end(tab.timeline, t_in);
    return;
  }

  // ---- the share's best min(C, cnt), in ascending token order ----
  const int keep = cnt < C ? cnt : C;
  {
    uint32_t key[NPT];
    int32_t tok[NPT];
    bool have[NPT], sel[NPT];
#pragma unroll
    for (int e = 0; e < NPT; ++e) {
      const int i = tid + e * FS_THREADS;        // < CAP
      have[e] = i < cnt;
      const uint32_t k = c_key[i];
      const int32_t tk = c_tok[i];
      key[e] = have[e] ? k : 0u;
      tok[e] = have[e] ? tk : 0;
      sel[e] = have[e];
    }
    if (keep < cnt) mark_best<FS_THREADS, FS_B0, NPT>(key, tok, have, keep, hist, xch, sel);
    // order by token through a bitmap of the share: rank of a token = set bits below it
    for (int wd = tid; wd < BM_WORDS; wd += FS_THREADS) bitmap[wd] = 0;
    __syncthreads();
#pragma unroll
    for (int e = 0; e < NPT; ++e)
      if (sel[e]) atomicOr(&bitmap[(tok[e] - tok0) >> 5], 1u << ((tok[e] - tok0) & 31));
    __syncthreads();
    uint32_t pcw[BM_WPT], pc = 0;
#pragma unroll
    for (int k = 0; k < BM_WPT; ++k) {
      const int wd = tid * BM_WPT + k;
      pcw[k] = wd < BM_WORDS ? (uint32_t)__popc(bitmap[wd]) : 0u;
      pc += pcw[k];
    }
    const uint32_t inc = wave_incl_scan(pc);
    if (lane == 63) xch[wave] = inc;
    __syncthreads();
    uint32_t woff[1];
    seg_wave_offsets<FS_WAVES, 1>(xch, wave, woff);
    uint32_t below = woff[0] + inc - pc;                  // set bits in the words below this thread's first one
#pragma unroll
    for (int k = 0; k < BM_WPT; ++k) {
      const int wd = tid * BM_WPT + k;
      if (wd < BM_WORDS) hist[wd] = below;
      below += pcw[k];
    }
    __syncthreads();
    uint32_t* o_key = reinterpret_cast<uint32_t*>(&stage[0][0]);   // [CAP] + [CAP] words fit: the page images are dead
    int32_t* o_tok = reinterpret_cast<int32_t*>(o_key + CAP);
#pragma unroll
    for (int e = 0; e < NPT; ++e)
      if (sel[e]) {
        const int rel = tok[e] - tok0;
        const uint32_t at = hist[rel >> 5] + (uint32_t)__popc(bitmap[rel >> 5] & ((1u << (rel & 31)) - 1u));
        o_key[at] = key[e];
        o_tok[at] = tok[e];
      }
    __syncthreads();
    // ---- write out, coalesced ----
    if (final_out) {
      for (int i = tid; i < C; i += FS_THREADS) sel_idx[row * C + i] = i < keep ? o_tok[i] : -1;
      if (tid == 0) sel_cnt[row] = keep;
    } else {
      const int64_t cbase = (crow * nshares + sh) * (int64_t)ccap;
      if (arrivals) {
        for (int i = tid; i < keep; i += FS_THREADS) {
          st_dev(&cand_key[cbase + i], o_key[i]);
          st_dev(&cand_idx[cbase + i], o_tok[i]);
        }
        if (tid == 0) st_dev(&cand_cnt[crow * nshares + sh], keep);
      } else {
        for (int i = tid; i < keep; i += FS_THREADS) {
          cand_key[cbase + i] = o_key[i];
          cand_idx[cbase + i] = o_tok[i];
        }
        if (tid == 0) cand_cnt[crow * nshares + sh] = keep;
      }
    }
  }
  if (!final_out && arrivals) arrive_and_merge();
  timeline_end(tab.timeline, t_in);
}

// Reduces a row's per-slice candidates (ascending token order within and across slices) to
// its top-C, again ascending and with ties to the lowest index.  Rows with at most
// MG_LDS candidates are first compacted into LDS (one read of the candidates), marked in
// registers (mark_best) and compacted in order; larger rows run the positional radix select
// of the stand-alone top-k over the global arrays.
// MG_NPT = candidates per thread the LDS path can hold (4, 8 or 16: 32 / 64 / 128 KB of pairs), chosen by the
// host from the most candidates a row can have, so that short rows do not pay for slots they never fill.
template <int MG_NPT>
__global__ __launch_bounds__(TK_THREADS) void select_merge_kernel(const sel_tab tab, int rows_per_layer,
                                                                  const uint32_t* __restrict__ cand_key,
                                                                  const int32_t* __restrict__ cand_idx,
                                                                  const int32_t* __restrict__ cand_cnt, int nslices,
                                                                  int ccap, int C) {
  constexpr int MG_LDS = MG_NPT * TK_THREADS;
  __shared__ int32_t cnt_sh[FS_MAX_SLICES];
  __shared__ int32_t pre_sh[FS_MAX_SLICES];
  __shared__ __attribute__((aligned(16))) uint32_t lkey[MG_LDS];
  __shared__ int32_t lidx[MG_LDS];
  __shared__ uint32_t hist[TK_BINS];
  __shared__ __attribute__((aligned(16))) uint32_t xch[TK_XCH];
  const int64_t crow = blockIdx.x;                         // row of the pack-wide candidate arrays
  const int layer = blockIdx.x / rows_per_layer;
  const int64_t row = crow - (int64_t)layer * rows_per_layer;  // row of this layer's outputs
  int32_t* __restrict__ sel_idx = tab.sel_idx[layer];
  int32_t* __restrict__ sel_cnt = tab.sel_cnt[layer];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // counts and their exclusive prefix over slices: thread s owns slice s
  static_assert(FS_MAX_SLICES <= TK_THREADS, "one slice per thread");
  const uint32_t mine = tid < nslices ? (uint32_t)cand_cnt[crow * nslices + tid] : 0u;
  const uint32_t inc = wave_incl_scan(mine);
  if (lane == 63) xch[wave] = inc;
  __syncthreads();
  uint32_t woff[1];
  const int total = (int)seg_wave_offsets<TK_THREADS / 64, 1>(xch, wave, woff);
  if (tid < nslices) {
    cnt_sh[tid] = (int32_t)mine;
    pre_sh[tid] = (int32_t)(woff[0] + inc - mine);
  }
  __syncthreads();
  const int keep = total < C ? total : C;
  const int64_t cbase = crow * nslices * (int64_t)ccap;
  const int nvirt = nslices * ccap;
  if (keep > 0) {
    if (total <= MG_LDS) {
      // eight candidates per thread and round, every load issued before the first is waited for (empty slots
      // re-read candidate 0 of the row: a guarded load would sit in a branch with a wait of its own)
      constexpr int MG_U = 8;
#pragma unroll 1
      for (int base = 0; base < nvirt; base += MG_U * TK_THREADS) {
        uint32_t k[MG_U];
        int32_t ix[MG_U];
        int pos[MG_U];
#pragma unroll
        for (int u = 0; u < MG_U; ++u) {
          const int v = base + u * TK_THREADS + tid;
          const int sl = v < nvirt ? v / ccap : 0;
          const int i = v - sl * ccap;
          const bool ok = v < nvirt && i < cnt_sh[sl];
          pos[u] = ok ? pre_sh[sl] + i : -1;
          k[u] = cand_key[cbase + (ok ? v : 0)];
          ix[u] = cand_idx[cbase + (ok ? v : 0)];
        }
#pragma unroll
        for (int u = 0; u < MG_U; ++u)
          if (pos[u] >= 0) {
            lkey[pos[u]] = k[u];
            lidx[pos[u]] = ix[u];
          }
      }
      __syncthreads();
      // a thread owns MG_NPT consecutive candidates (token order): exact marking of the best `keep` in registers,
      // then an ordered compaction of the marked ones
      uint32_t key[MG_NPT];
      int32_t tok[MG_NPT];
      bool have[MG_NPT], sel[MG_NPT];
#pragma unroll
      for (int e = 0; e < MG_NPT; ++e) {
        const int i = tid * MG_NPT + e;            // < MG_LDS
        have[e] = i < total;
        const uint32_t k = lkey[i];
        const int32_t tk = lidx[i];
        key[e] = have[e] ? k : 0u;
        tok[e] = have[e] ? tk : 0;
        sel[e] = have[e];
      }
      if (keep < total) mark_best<TK_THREADS, 12, MG_NPT>(key, tok, have, keep, hist, xch, sel);
      uint32_t c = 0;
#pragma unroll
      for (int e = 0; e < MG_NPT; ++e) c += sel[e] ? 1u : 0u;
      const uint32_t sinc = wave_incl_scan(c);
      __syncthreads();                 // every thread has its candidates in registers: lidx becomes the output stage
      if (lane == 63) xch[wave] = sinc;
      __syncthreads();
      uint32_t soff[1];
      seg_wave_offsets<TK_THREADS / 64, 1>(xch, wave, soff);
      uint32_t at = soff[0] + sinc - c;
#pragma unroll
      for (int e = 0; e < MG_NPT; ++e)
        if (sel[e]) lidx[at++] = tok[e];
      __syncthreads();
      for (int i = tid; i < keep; i += TK_THREADS) sel_idx[row * C + i] = lidx[i];
    } else {
      auto key_of = [&](int v, bool& valid) -> uint32_t {
        valid = (v % ccap) < cnt_sh[v / ccap];
        return valid ? cand_key[cbase + v] : 0u;
      };
      auto emit = [&](uint32_t pos, int v, uint32_t) { sel_idx[row * C + pos] = cand_idx[cbase + v]; };
      block_select<TK_THREADS, 12>(nvirt, total, keep, false, key4_from_scalar(nvirt, key_of), emit, hist, xch);
    }
  }
  for (int i = keep + tid; i < C; i += TK_THREADS) sel_idx[row * C + i] = -1;
  if (tid == 0) sel_cnt[row] = keep;
}

// The prologue form keeps q_hat of the whole group in 8 KB of LDS: groups of up to 16 heads, whatever the aggregation.
bool select_can_predict(const as_params* p) {
  const int G = p->n_q_heads / p->n_kv_heads;
  return p->window <= 16 && p->agg != AS_AGG_SOFTMAX_SUM && G <= 16;
}

hipError_t launch_select_pack(const as_params* p, int n_layers, const sel_tab& tab_in, void* ws, int32_t* arrivals,
                              bool fuse_predict, hipStream_t s) {
  const int64_t rows = (int64_t)p->batch * p->n_kv_heads * n_layers;
  if (rows == 0) return hipSuccess;
  if ((int64_t)p->batch * n_layers > 65535) return hipErrorInvalidValue;   // grid.y
  if (fuse_predict && !select_can_predict(p)) return hipErrorInvalidValue;
  sel_tab tab = tab_in;
  tab.pred_window = p->window;
  tab.pred_single = p->predictor == AS_PRED_SINGLE_SOLVE ? 1 : 0;
  tab.pred_eps = (double)p->ridge_eps;
  tab.pred_beta = (double)p->softmax_beta;
  const select_plan pl = plan_select(p, n_layers);
  const int G = p->n_q_heads / p->n_kv_heads;
  uint32_t* cand_key = nullptr;
  int32_t *cand_idx = nullptr, *cand_cnt = nullptr;
  if (pl.nslices > 1) {
    const size_t n = (size_t)rows * pl.nslices * pl.ccap;
    cand_key = reinterpret_cast<uint32_t*>(ws);
    cand_idx = reinterpret_cast<int32_t*>(cand_key + n);
    cand_cnt = cand_idx + n;
  }
  dim3 grid(p->n_kv_heads, p->batch * n_layers, pl.nslices);
  const int nset = (p->agg == AS_AGG_SUM || G <= 8) ? 1 : G <= 16 ? 2 : G <= 32 ? 4 : 8;
  // Rows cut into several shares are merged by the last workgroup of the row inside the slice kernel when there
  // is an arrival counter per row and the row's candidates fit the kernel's LDS candidate buffer; else by a
  // second launch.
  const int thr = nset > 2 ? 512 : 1024;
  const bool merge_in_kernel = arrivals != nullptr && pl.nslices > 1 && rows <= AS_SEL_COUNTERS &&
                               (int64_t)pl.nslices * pl.ccap <= 8 * thr && pl.nslices <= thr / 4 &&
                               (int64_t)rows * pl.nslices * pl.ccap * 8 < 0x7fffffffLL;
  int32_t* arr = merge_in_kernel ? arrivals : nullptr;
  float2* lse_part = reinterpret_cast<float2*>(static_cast<char*>(ws) + cand_bytes(p, pl, n_layers));
#define AS_SLICE_LAUNCH(NSET_, THR_, MODE_, PRED_)                                                                \
  hipLaunchKernelGGL((select_slice_kernel<NSET_, THR_, (NSET_ == 4 || (NSET_ == 8 && MODE_ == 0) ? FS_PG4 : FS_PG), MODE_, PRED_>), grid, dim3(THR_), 0, s, tab, \
                     p->batch, p->n_q_heads, p->n_kv_heads, G, p->agg, p->max_pages_per_seq, pl.slice_len,        \
                     pl.nslices, p->budget, pl.ccap, cand_key, cand_idx, cand_cnt, p->sm_scale, lse_part, arr)
  // groups of up to 16 heads (one or two operand sets) run 1024-thread workgroups, larger ones the 512-thread shape
  if (p->agg == AS_AGG_SOFTMAX_SUM) {
    // two passes over K with the same grid: per-share (max, sum) pairs, then selection on the normalised scores
    if (nset == 8) { AS_SLICE_LAUNCH(8, 512, 1, false); AS_SLICE_LAUNCH(8, 512, 2, false); }
    else if (nset == 4) { AS_SLICE_LAUNCH(4, 512, 1, false); AS_SLICE_LAUNCH(4, 512, 2, false); }
    else if (nset == 2) { AS_SLICE_LAUNCH(2, 1024, 1, false); AS_SLICE_LAUNCH(2, 1024, 2, false); }
    else { AS_SLICE_LAUNCH(1, 1024, 1, false); AS_SLICE_LAUNCH(1, 1024, 2, false); }
  } else if (nset == 8) AS_SLICE_LAUNCH(8, 512, 0, false);
  else if (nset == 4) AS_SLICE_LAUNCH(4, 512, 0, false);
  else if (nset == 2) { if (fuse_predict) AS_SLICE_LAUNCH(2, 1024, 0, true); else AS_SLICE_LAUNCH(2, 1024, 0, false); }
  else { if (fuse_predict) AS_SLICE_LAUNCH(1, 1024, 0, true); else AS_SLICE_LAUNCH(1, 1024, 0, false); }
#undef AS_SLICE_LAUNCH
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || pl.nslices == 1 || merge_in_kernel) return e;
  const int64_t most = (int64_t)pl.nslices * pl.ccap;   // candidates a row can have
#define AS_MERGE_LAUNCH(NPT_)                                                                                   \
  hipLaunchKernelGGL(select_merge_kernel<NPT_>, dim3((unsigned)rows), dim3(TK_THREADS), 0, s, tab,              \
                     p->batch * p->n_kv_heads, cand_key, cand_idx, cand_cnt, pl.nslices, pl.ccap, p->budget)
  if (most <= 4 * TK_THREADS) AS_MERGE_LAUNCH(4);
  else if (most <= 8 * TK_THREADS) AS_MERGE_LAUNCH(8);
  else AS_MERGE_LAUNCH(16);
#undef AS_MERGE_LAUNCH
  return hipGetLastError();
}

hipError_t launch_select_fused(const as_params* p, const as_kv_view* kv, const float* q_hat, const uint16_t* q_win,
                               const uint16_t* q_cur, void* ws, int32_t* arrivals, int32_t* sel_idx, int32_t* sel_cnt,
                               wg_timeline tl, hipStream_t s) {
  sel_tab tab = {};
  tab.timeline = tl;
  tab.q_win[0] = q_win;
  tab.q_cur[0] = q_cur;
  tab.k_pool[0] = reinterpret_cast<const uint16_t*>(kv->k_pool);
  tab.block_table[0] = kv->block_table;
  tab.ctx_lens[0] = kv->ctx_lens;
  tab.q_hat[0] = q_hat;
  tab.sel_idx[0] = sel_idx;
  tab.sel_cnt[0] = sel_cnt;
  tab.last_page[0] = (int32_t)(kv->num_pages > 0 ? kv->num_pages - 1 : 0);
  return launch_select_pack(p, 1, tab, ws, arrivals, q_win != nullptr, s);
}

}  // namespace asx
