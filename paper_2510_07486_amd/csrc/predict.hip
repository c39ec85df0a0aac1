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

// Window sizes known at compile time (the paper profiles W = 16), W <= 16.  Same algorithm, laid out for one
// wavefront:
//  * the Gram matrix of the W predecessors is one chain of 32 fp64 matrix-core instructions
//    (v_mfma_f64_16x16x4: G += X_s X_s^T over 32 slices of four dims; lane l supplies X[l % 16][4s + l / 16] as
//    both operands); the result lands with lane (r = l % 16, q = l / 16) holding G[r][q + 4v], v = 0..3, i.e.
//    every row spread over four lanes, which is the distribution the factorisation below works in;
//  * G + eps I = L D L^T (unit lower L, no square roots) by right-looking elimination on the full symmetric
//    trailing block: per step one reciprocal, the pivot row and column fetched with cross-lane reads, at most four
//    multiply-adds per lane.  The right-hand side b rides along, so z = L^-1 b and y = D^-1 z come out of the
//    same loop.  Leading blocks of L and D factor the leading blocks of G: one factorisation serves every window size;
//  * lane k-1 then back-substitutes L_k^T omega = y_{1:k} on its own, the W(W+1)/2 softmax exponentials are
//    spread over the 64 lanes.
template <int W>
__global__ __launch_bounds__(64) void predict_kernel_w(const pred_tab tab, int heads_per_layer, double eps,
                                                       double beta, int single) {
  static_assert(W >= 1 && W <= 16, "one 16 x 16 matrix-core tile holds the Gram matrix");
  typedef double f64x4 __attribute__((ext_vector_type(4)));
  constexpr int RW = AS_HEAD_DIM + 4;  // row stride of the staged window: lanes (r, q) read banks 4r + q
  __shared__ float Rf[(W + 1) * RW];   // row i < W = Q_{t-1-i}, row W = Q_t
  __shared__ double Ls[W][W + 1];      // L below the diagonal
  __shared__ double Om[W][W + 1];      // row k-1: beta*omega^{(k)} - max, then exp of it
  __shared__ double yv[W], zinv[W], av[W];

  const int lane = threadIdx.x;
  const int r = lane & 15, q = lane >> 4;
  const int layer = blockIdx.x / heads_per_layer;
  const int64_t bh = blockIdx.x - layer * heads_per_layer;
  float* __restrict__ q_hat = tab.q_hat[layer];
  const uint32_t* win = reinterpret_cast<const uint32_t*>(tab.q_win[layer] + bh * (int64_t)W * AS_HEAD_DIM);
  const uint32_t* cur = reinterpret_cast<const uint32_t*>(tab.q_cur[layer] + bh * (int64_t)AS_HEAD_DIM);
#pragma unroll
  for (int i = 0; i < W; ++i) {
    const uint32_t w2 = win[(int64_t)(W - 1 - i) * (AS_HEAD_DIM / 2) + lane];
    Rf[i * RW + 2 * lane] = bf16lo(w2);
    Rf[i * RW + 2 * lane + 1] = bf16hi(w2);
  }
  {
    const uint32_t w2 = cur[lane];
    Rf[W * RW + 2 * lane] = bf16lo(w2);
    Rf[W * RW + 2 * lane + 1] = bf16hi(w2);
  }
  __syncthreads();

  // Gram matrix on the matrix cores; the rhs b_r = <Q_{t-1-r}, Q_t> from the same operand values
  f64x4 acc = {0.0, 0.0, 0.0, 0.0};
  double b = 0.0;
  {
    const float* xr = Rf + (r < W ? r : 0) * RW + q;
    const float* tr = Rf + W * RW + q;
#pragma unroll 8
    for (int s4 = 0; s4 < AS_HEAD_DIM; s4 += 4) {
      const double x = r < W ? (double)xr[s4] : 0.0;
      acc = __builtin_amdgcn_mfma_f64_16x16x4f64(x, x, acc, 0, 0, 0);
      b += x * (double)tr[s4];
    }
    b += __shfl_xor(b, 16);
    b += __shfl_xor(b, 32);
  }
  double a[4];   // a[v] = (G + eps I)[r][q + 4v]
#pragma unroll
  for (int v = 0; v < 4; ++v) a[v] = acc[v] + (q + 4 * v == r ? eps : 0.0);

  // L D L^T with the rhs carried along
  auto from_lane = [](double x, int src) -> double {   // src uniform
    const int lo = __builtin_amdgcn_readlane(__double2loint(x), src);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(x), src);
    return __hiloint2double(hi, lo);
  };
#pragma unroll
  for (int j = 0; j < W; ++j) {
    const int jq = j & 3, jv = j >> 2;                       // column j sits in lanes q = jq, register jv
    const double inv = 1.0 / from_lane(a[jv], j + 16 * jq);  // pivot D_j
    const double zj = from_lane(b, j);
    const double cr = __shfl(a[jv], r + 16 * jq);            // (G)[r][j] after the earlier steps
    const double lr = r > j ? cr * inv : 0.0;                // L[r][j]
#pragma unroll
    for (int v = 0; v < 4; ++v)
      if (4 * v + 3 > j) {                                   // some lane's column q + 4v lies right of j
        const double rj = __shfl(a[v], j + 16 * q);          // row j, this lane's column
        if (q + 4 * v > j) a[v] -= lr * rj;
      }
    b -= lr * zj;
    if (q == 0 && r > j && r < W) Ls[r][j] = lr;
    if (lane == 0) yv[j] = zj * inv;
  }
  __syncthreads();

  // lane kk: L_k^T omega = y_{1:k} for k = kk+1, weights stay zero above kk (single-solve mode: every lane
  // solves the full system; only its kk+1 newest entries enter the softmax below)
  const int kk = lane;
  double om[W];
#pragma unroll
  for (int i = 0; i < W; ++i) om[i] = 0.0;
#pragma unroll
  for (int i = W - 1; i >= 0; --i) {
    double s = yv[i];
#pragma unroll
    for (int m = i + 1; m < W; ++m) s -= Ls[m][i] * om[m];
    om[i] = (single || i <= kk) ? s : 0.0;
  }
  if (kk < W) {
    double mx = beta * om[0];
#pragma unroll
    for (int i = 1; i < W; ++i)
      if (i <= kk) mx = fmax(mx, beta * om[i]);
#pragma unroll
    for (int i = 0; i < W; ++i) Om[kk][i] = beta * om[i] - mx;
  }
  __syncthreads();
  // exponentials of the W(W+1)/2 (k, i) pairs, spread over the lanes
  for (int p = lane; p < W * (W + 1) / 2; p += 64) {
    int k = (int)((sqrtf(8.0f * (float)p + 1.0f) - 1.0f) * 0.5f);
    while (k * (k + 1) / 2 > p) --k;
    while ((k + 1) * (k + 2) / 2 <= p) ++k;
    const int i = p - k * (k + 1) / 2;
    Om[k][i] = exp(Om[k][i]);
  }
  __syncthreads();
  if (kk < W) {
    double z = 0.0;
#pragma unroll
    for (int i = 0; i < W; ++i)
      if (i <= kk) z += Om[kk][i];
    zinv[kk] = 1.0 / z;
  }
  __syncthreads();
  if (kk < W) {
    double sum = 0.0;
#pragma unroll
    for (int k2 = 0; k2 < W; ++k2)
      if (k2 >= kk) sum += Om[k2][kk] * zinv[k2];
    av[kk] = sum / (double)W;
  }
  __syncthreads();
  for (int d = lane; d < AS_HEAD_DIM; d += 64) {
    double o = av[0] * (double)Rf[W * RW + d];
#pragma unroll
    for (int i = 1; i < W; ++i) o += av[i] * (double)Rf[(i - 1) * RW + d];
    q_hat[bh * AS_HEAD_DIM + d] = (float)o;
  }
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
