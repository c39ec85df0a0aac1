/*
 * Plain-C caller of the C ABI (no C++, no PyTorch): allocates a two-page bf16 KV cache with the HIP runtime,
 * runs predict -> fused selection -> sparse attention on a hand-checkable case and verifies the results:
 *   keys    first component (3, 1, 2, 3, 0, ...), so with q_hat = e_0 the scores are (3, 1, 2, 3, 0, ...);
 *   budget 2 keeps tokens {0, 3} (Sec. 4.3 item (2), ties to the lowest index do not even arise);
 *   values  first component (10, 20, 30, 50): attention with q = e_0 over {0, 3} gives (10 + 50) / 2 = 30 (Sec. 4.1).
 * The query window holds Q_{t-1} = e_1 and Q_t = e_0 with W = 1, so the predictor returns Q_t itself (Eq. 4, k = 1).
 * Prints "abi_demo: OK" and exits 0 on success.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "asyncspade.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "HIP error %d at %s:%d\n", (int)e_, __FILE__, __LINE__); return 2; } } while (0)
#define CHECK_AS(x) do { as_status s_ = (x); if (s_ != AS_OK) { fprintf(stderr, "%s -> %s\n", #x, as_status_str(s_)); return 3; } } while (0)

static uint16_t bf16(float f) { uint32_t u; memcpy(&u, &f, 4); return (uint16_t)(u >> 16); }   /* exact for small integers */
static float bf16_to_f(uint16_t h) { uint32_t u = (uint32_t)h << 16; float f; memcpy(&f, &u, 4); return f; }

int main(void) {
  enum { HKV = 1, HQ = 1, D = 128, P = 16, PAGES = 2, N = 20, C = 2, W = 1 };
  static uint16_t k[PAGES * HKV * P * D], v[PAGES * HKV * P * D], qwin[W * D], qcur[D], out_h[D];
  const float kvals[4] = {3.f, 1.f, 2.f, 3.f}, vvals[4] = {10.f, 20.f, 30.f, 50.f};
  /* logical page 0 lives in physical page 1 and vice versa */
  int32_t table[PAGES] = {1, 0}, lens[1] = {N}, sel_h[C], cnt_h[1];
  for (int n = 0; n < 4; ++n) {
    k[(1 * P + n) * D + 0] = bf16(kvals[n]);
    v[(1 * P + n) * D + 0] = bf16(vvals[n]);
  }
  qwin[1] = bf16(1.f);
  qcur[0] = bf16(1.f);

  void *dk, *dv, *dqw, *dqc, *dout;
  int32_t *dtab, *dlens, *dsel, *dcnt;
  float* dlse;
  CHECK_HIP(hipSetDevice(0));
  CHECK_HIP(hipMalloc(&dk, sizeof k));
  CHECK_HIP(hipMalloc(&dv, sizeof v));
  CHECK_HIP(hipMalloc(&dqw, sizeof qwin));
  CHECK_HIP(hipMalloc(&dqc, sizeof qcur));
  CHECK_HIP(hipMalloc(&dout, sizeof out_h));
  CHECK_HIP(hipMalloc((void**)&dtab, sizeof table));
  CHECK_HIP(hipMalloc((void**)&dlens, sizeof lens));
  CHECK_HIP(hipMalloc((void**)&dsel, sizeof sel_h));
  CHECK_HIP(hipMalloc((void**)&dcnt, sizeof cnt_h));
  CHECK_HIP(hipMalloc((void**)&dlse, sizeof(float)));
  CHECK_HIP(hipMemcpy(dk, k, sizeof k, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dv, v, sizeof v, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dqw, qwin, sizeof qwin, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dqc, qcur, sizeof qcur, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dtab, table, sizeof table, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dlens, lens, sizeof lens, hipMemcpyHostToDevice));

  as_params p;
  memset(&p, 0, sizeof p);
  p.batch = 1; p.n_q_heads = HQ; p.n_kv_heads = HKV; p.head_dim = D; p.page_size = P; p.window = W; p.budget = C;
  p.max_pages_per_seq = PAGES; p.ridge_eps = 0.01f; p.softmax_beta = 1.f; p.sm_scale = 1.f;
  p.agg = AS_AGG_MAX; p.predictor = AS_PRED_PER_WINDOW;
  as_kv_view kv = {dk, dv, dtab, dlens, PAGES};
  as_ctx* ctx = NULL;
  CHECK_AS(as_create(&ctx, 0, as_workspace_bytes(&p)));
  CHECK_AS(as_select_step(ctx, &p, &kv, dqw, dqc, dsel, dcnt, NULL));
  CHECK_AS(as_sparse_decode_attn(ctx, &p, &kv, dqc, dsel, dcnt, NULL, dout, dlse, NULL));
  CHECK_HIP(hipDeviceSynchronize());
  float lse_h;
  CHECK_HIP(hipMemcpy(sel_h, dsel, sizeof sel_h, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(cnt_h, dcnt, sizeof cnt_h, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(out_h, dout, sizeof out_h, hipMemcpyDeviceToHost));
  CHECK_HIP(hipMemcpy(&lse_h, dlse, sizeof lse_h, hipMemcpyDeviceToHost));
  CHECK_AS(as_destroy(ctx));
  const float o0 = bf16_to_f(out_h[0]);
  printf("abi_demo: selected %d tokens [%d, %d], out[0] = %g, lse = %g\n", cnt_h[0], sel_h[0], sel_h[1], o0, lse_h);
  if (cnt_h[0] != 2 || sel_h[0] != 0 || sel_h[1] != 3 || o0 != 30.f || out_h[1] != 0 ||
      lse_h < 3.6931f || lse_h > 3.6932f) {
    fprintf(stderr, "abi_demo: MISMATCH\n");
    return 1;
  }
  printf("abi_demo: OK\n");
  return 0;
}
