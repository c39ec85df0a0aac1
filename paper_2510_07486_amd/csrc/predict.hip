// Query predictor (Sec. 4.2: Eq. 2-3 ridge + softmax, Eq. 4 single-token shift, Eq. 5 mean
// over window sizes; Appendix C Alg. 1 steps 1-6).
//
// One wavefront per (sequence, query head).  The window is reordered newest-first so that
// window size k is the LEADING k x k block of one W x W Gram matrix: a single fp64
// factorisation (Cholesky in the general kernel, L D L^T in the fixed-window one) and a single
// forward solve then serve every k (both are prefix-consistent), and lane k-1 finishes its own
// size-k back-substitution, softmax and weight row independently.  Everything W x W is fp64; the
// result is
//   q_hat = sum_i a_i S_i,  a_i = (1/W) sum_{k>=i} w^{(k)}_i,  S = (Q_t, Q_{t-1}, ..., Q_{t-W+1}).
// Latency-bound and tiny (about 50 kflop per head at W = 16): one dependent chain per head.
#include "common.hpp"
#include "predict_common.hpp"

namespace asx {

static constexpr int RS = AS_HEAD_DIM + 1;  // padded fp32 row stride (bank spread)

__host__ __device__ inline size_t predict_lds_bytes(int W) {
  size_t dbl = (size_t)W * (W + 1) * 2 + 3 * (size_t)W;  // A, Om, bv, yv, av
  return dbl * sizeof(double) + (size_t)(W + 1) * RS * sizeof(float);
}

__global__ __launch_bounds__(64) void predict_kernel(const pred_tab tab, int heads_per_layer, int W, double eps,
                                                     double beta, int single) {
  extern __shared__ double smem_d[];
  double* A = smem_d;                    // [W][W+1] lower Cholesky factor in place
  double* Om = A + (size_t)W * (W + 1);  // [W][W+1] row k-1: omega^{(k)} then w^{(k)}
  double* bv = Om + (size_t)W * (W + 1);
  double* yv = bv + W;
  double* av = yv + W;
  float* Rf = reinterpret_cast<float*>(av + W);  // [W+1][RS]; row i<W = Q_{t-1-i}, row W = Q_t

  const int lane = threadIdx.x;
  const int layer = blockIdx.x / heads_per_layer;          // uniform: the table entry is read with scalar loads
  const int64_t bh = blockIdx.x - layer * heads_per_layer;
  float* __restrict__ q_hat = tab.q_hat[layer];
  const uint32_t* win = reinterpret_cast<const uint32_t*>(tab.q_win[layer] + bh * (int64_t)W * AS_HEAD_DIM);
  const uint32_t* cur = reinterpret_cast<const uint32_t*>(tab.q_cur[layer] + bh * (int64_t)AS_HEAD_DIM);

  // 1. stage the window newest-first (lane holds dims 2*lane, 2*lane+1)
  for (int i = 0; i < W; ++i) {
    uint32_t w2 = win[(int64_t)(W - 1 - i) * (AS_HEAD_DIM / 2) + lane];
    Rf[i * RS + 2 * lane] = bf16lo(w2);
    Rf[i * RS + 2 * lane + 1] = bf16hi(w2);
  }
  {
    uint32_t w2 = cur[lane];
    Rf[W * RS + 2 * lane] = bf16lo(w2);
    Rf[W * RS + 2 * lane + 1] = bf16hi(w2);
  }
  __syncthreads();

  // 2. Gram matrix of the W predecessors (+ eps on the diagonal) and rhs b_i = <Q_{t-i}, Q_t>
  const int npairs = (W + 1) * (W + 2) / 2;
  for (int p = lane; p < npairs; p += 64) {
    int i = (int)((sqrtf(8.0f * (float)p + 1.0f) - 1.0f) * 0.5f);
    while (i * (i + 1) / 2 > p) --i;
    while ((i + 1) * (i + 2) / 2 <= p) ++i;
    int j = p - i * (i + 1) / 2;
    const float* ri = Rf + i * RS;
    const float* rj = Rf + j * RS;
    double s = 0.0;
    for (int d = 0; d < AS_HEAD_DIM; ++d) s += (double)ri[d] * (double)rj[d];
    if (i < W) A[i * (W + 1) + j] = s + (i == j ? eps : 0.0);
    else if (j < W) bv[j] = s;
  }

  // 3. Cholesky, lane = row
  const int r = lane;
  for (int j = 0; j < W; ++j) {
    __syncthreads();
    double djj = sqrt(A[j * (W + 1) + j]);
    double lij = 0.0;
    if (r > j && r < W) {
      lij = A[r * (W + 1) + j] / djj;
      A[r * (W + 1) + j] = lij;
    }
    __syncthreads();
    if (r == j) A[j * (W + 1) + j] = djj;
    if (r > j && r < W)
      for (int k = j + 1; k <= r; ++k) A[r * (W + 1) + k] -= lij * A[k * (W + 1) + j];
  }
  __syncthreads();

  // 4. forward solve y = L^-1 b (prefix-consistent: y_{1:k} solves the size-k system)
  {
    double rr = (r < W) ? bv[r] : 0.0;
    double y = 0.0;
    for (int j = 0; j < W; ++j) {
      double yj = __shfl(rr, j) / A[j * (W + 1) + j];
      if (r == j) y = yj;
      if (r > j && r < W) rr -= A[r * (W + 1) + j] * yj;
    }
    if (r < W) yv[r] = y;
  }
  __syncthreads();

  // 5. lane kk solves L_k^T omega = y_{1:k} for k = kk+1 (single-solve mode: the full system for every lane,
  //    of which lane kk keeps the kk+1 newest entries), then softmax(beta * omega)
  if (r < W) {
    const int kk = r;
    const int ks = single ? W - 1 : kk;
    double* om = Om + kk * (W + 1);
    for (int i = ks; i >= 0; --i) {
      double s = yv[i];
      for (int m = i + 1; m <= ks; ++m) s -= A[m * (W + 1) + i] * om[m];
      om[i] = s / A[i * (W + 1) + i];
    }
    double mx = beta * om[0];
    for (int i = 1; i <= kk; ++i) mx = fmax(mx, beta * om[i]);
    double z = 0.0;
    for (int i = 0; i <= kk; ++i) {
      double e = exp(beta * om[i] - mx);
      om[i] = e;
      z += e;
    }
    for (int i = 0; i <= kk; ++i) om[i] /= z;
  }
  __syncthreads();

  // 6. pooled weight of shifted element i: a_i = (1/W) sum_{k > i} w^{(k)}_i
  if (r < W) {
    double a = 0.0;
    for (int kk = r; kk < W; ++kk) a += Om[kk * (W + 1) + r];
    av[r] = a / (double)W;
  }
  __syncthreads();

  // 7. q_hat = a_0 Q_t + sum_{i>=1} a_i Q_{t-i}
  for (int d = lane; d < AS_HEAD_DIM; d += 64) {
    double acc = av[0] * (double)Rf[W * RS + d];
    for (int i = 1; i < W; ++i) acc += av[i] * (double)Rf[(i - 1) * RS + d];
    q_hat[bh * AS_HEAD_DIM + d] = (float)acc;
  }
}

// Window sizes known at compile time (the paper profiles W = 16), W <= 16: one wavefront per workgroup runs
// predict_wave (predict_common.hpp).
template <int W>
__global__ __launch_bounds__(64) void predict_kernel_w(const pred_tab tab, int heads_per_layer, double eps,
                                                       double beta, int single) {
  __shared__ predict_lds<W> S;
  const int layer = blockIdx.x / heads_per_layer;
  const int64_t bh = blockIdx.x - layer * heads_per_layer;
  const uint32_t* win = reinterpret_cast<const uint32_t*>(tab.q_win[layer] + bh * (int64_t)W * AS_HEAD_DIM);
  const uint32_t* cur = reinterpret_cast<const uint32_t*>(tab.q_cur[layer] + bh * (int64_t)AS_HEAD_DIM);
  predict_wave<W, false>(win, cur, W, eps, beta, single, S, tab.q_hat[layer] + bh * AS_HEAD_DIM);
}

hipError_t launch_predict_pack(const as_params* p, int n_layers, const pred_tab& tab, hipStream_t s) {
  const int64_t per_layer = (int64_t)p->batch * p->n_q_heads;
  const int64_t heads = per_layer * n_layers;
  if (heads == 0) return hipSuccess;
  if (heads > 0x7fffffff) return hipErrorInvalidValue;
  const int hpl = (int)per_layer;
  const int single = p->predictor == AS_PRED_SINGLE_SOLVE ? 1 : 0;
#define AS_PREDICT_W(W_)                                                                                  \
  case W_:                                                                                               \
    hipLaunchKernelGGL(predict_kernel_w<W_>, dim3((unsigned)heads), dim3(64), 0, s, tab, hpl,            \
                       (double)p->ridge_eps, (double)p->softmax_beta, single);                           \
    return hipGetLastError();
  switch (p->window) {   // windows of up to 16 queries: the Gram matrix fits one matrix-core tile
    AS_PREDICT_W(1) AS_PREDICT_W(2) AS_PREDICT_W(3) AS_PREDICT_W(4) AS_PREDICT_W(5) AS_PREDICT_W(6)
    AS_PREDICT_W(7) AS_PREDICT_W(8) AS_PREDICT_W(9) AS_PREDICT_W(10) AS_PREDICT_W(11) AS_PREDICT_W(12)
    AS_PREDICT_W(13) AS_PREDICT_W(14) AS_PREDICT_W(15) AS_PREDICT_W(16)
    default: break;
  }
#undef AS_PREDICT_W
  size_t lds = predict_lds_bytes(p->window);
  if (lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(predict_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(predict_kernel, dim3((unsigned)heads), dim3(64), lds, s, tab, hpl, p->window,
                     (double)p->ridge_eps, (double)p->softmax_beta, single);
  return hipGetLastError();
}

hipError_t launch_predict(const as_params* p, const uint16_t* q_win, const uint16_t* q_cur, float* q_hat,
                          hipStream_t s) {
  pred_tab tab = {};
  tab.q_win[0] = q_win;
  tab.q_cur[0] = q_cur;
  tab.q_hat[0] = q_hat;
  return launch_predict_pack(p, 1, tab, s);
}

}  // namespace asx
