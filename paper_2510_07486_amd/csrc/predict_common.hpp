// The query predictor for windows of up to 16 queries as a device function that ONE wavefront runs on its own
// (Sec. 4.2: Eq. 2-3 ridge + softmax, Eq. 4 single-token shift, Eq. 5 mean over window sizes; Appendix C Alg. 1
// steps 1-6).  Used by the stand-alone predictor kernel (one wavefront per workgroup) and by the prologue of the
// fused selection kernel (the wavefronts of a workgroup predict the queries of their own KV head's group).
//
// Laid out for one wavefront:
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
// WC is the compile-time bound of the window (loops are unrolled to it).  With RT = false the window is WC itself;
// with RT = true the window is the run-time w_rt <= WC and the rows beyond it are exact zeros that drop out of
// every sum, so both forms compute the same values in the same order.
#pragma once
#include "common.hpp"

namespace asx {

template <int WC> struct predict_lds {
  static constexpr int RW = AS_HEAD_DIM + 4;  // row stride of the staged window: lanes (r, q) read banks 4r + q
  float Rf[(WC + 1) * RW];                    // row i < W = Q_{t-1-i}, row WC = Q_t
  double Ls[WC][WC + 1];                      // L below the diagonal
  double Om[WC][WC + 1];                      // row k-1: beta*omega^{(k)} - max, then exp of it
  double yv[WC], zinv[WC], av[WC];
};

// win: the head's window, bf16 pairs, [W][64] oldest first; cur: Q_t, [64].  out: 128 floats (any address space).
// Every lane of the wavefront must call it; S is wave-private LDS.  Memory operations of one wavefront on LDS
// complete in program order, so the phases are separated by scheduling barriers only.
template <int WC, bool RT>
__device__ __forceinline__ void predict_wave(const uint32_t* __restrict__ win, const uint32_t* __restrict__ cur,
                                             int w_rt, double eps, double beta, int single, predict_lds<WC>& S,
                                             float* out) {
  static_assert(WC >= 1 && WC <= 16, "one 16 x 16 matrix-core tile holds the Gram matrix");
  typedef double f64x4 __attribute__((ext_vector_type(4)));
  constexpr int RW = predict_lds<WC>::RW;
  const int W = RT ? w_rt : WC;
  const int lane = threadIdx.x & 63;
  const int r = lane & 15, q = lane >> 4;
#pragma unroll
  for (int i = 0; i < WC; ++i)
    if (!RT || i < W) {
      const uint32_t w2 = win[(int64_t)(W - 1 - i) * (AS_HEAD_DIM / 2) + lane];
      S.Rf[i * RW + 2 * lane] = bf16lo(w2);
      S.Rf[i * RW + 2 * lane + 1] = bf16hi(w2);
    }
  {
    const uint32_t w2 = cur[lane];
    S.Rf[WC * RW + 2 * lane] = bf16lo(w2);
    S.Rf[WC * RW + 2 * lane + 1] = bf16hi(w2);
  }
  __builtin_amdgcn_wave_barrier();

  // Gram matrix on the matrix cores; the rhs b_r = <Q_{t-1-r}, Q_t> from the same operand values
  f64x4 acc = {0.0, 0.0, 0.0, 0.0};
  double b = 0.0;
  {
    const float* xr = S.Rf + (r < W ? r : 0) * RW + q;
    const float* tr = S.Rf + WC * RW + q;
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
  for (int j = 0; j < WC; ++j) {
    const int jq = j & 3, jv = j >> 2;                       // column j sits in lanes q = jq, register jv
    const double inv = 1.0 / from_lane(a[jv], j + 16 * jq);  // pivot D_j (eps for a row beyond the window)
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
    if (q == 0 && r > j && r < WC) S.Ls[r][j] = lr;
    if (lane == 0) S.yv[j] = zj * inv;
  }
  __builtin_amdgcn_wave_barrier();

  // lane kk: L_k^T omega = y_{1:k} for k = kk+1, weights stay zero above kk (single-solve mode: every lane
  // solves the full system; only its kk+1 newest entries enter the softmax below).  Two forms with the same
  // arithmetic in the same order.  RT = false (the stand-alone kernel): fully unrolled, omega in registers
  // (134 registers at W = 16).  RT = true (the prologue of the fused selection kernel, whose 1024-thread
  // workgroups allow 128 registers): the loop over the unknowns stays rolled and the solved entries are read
  // back from the lane's own row of Om.
  const int kk = lane;
  if constexpr (!RT) {
    double om[WC];
#pragma unroll
    for (int i = 0; i < WC; ++i) om[i] = 0.0;
#pragma unroll
    for (int i = WC - 1; i >= 0; --i) {
      double s = S.yv[i];
#pragma unroll
      for (int m = i + 1; m < WC; ++m) s -= S.Ls[m][i] * om[m];
      om[i] = (single || i <= kk) ? s : 0.0;
    }
    if (kk < W) {
      double mx = beta * om[0];
#pragma unroll
      for (int i = 1; i < WC; ++i)
        if (i <= kk) mx = fmax(mx, beta * om[i]);
#pragma unroll
      for (int i = 0; i < WC; ++i) S.Om[kk][i] = beta * om[i] - mx;
    }
  } else if (kk < W) {
#pragma unroll 1
    for (int i = WC - 1; i >= 0; --i) {
      double s = S.yv[i];
#pragma unroll
      for (int m = 1; m < WC; ++m)
        if (m > i) s -= S.Ls[m][i] * S.Om[kk][m];       // entries m > i of this lane's row were stored below
      S.Om[kk][i] = ((single && i < W) || i <= kk) ? s : 0.0;
    }
    double mx = beta * S.Om[kk][0];
#pragma unroll 1
    for (int i = 1; i <= kk; ++i) mx = fmax(mx, beta * S.Om[kk][i]);
#pragma unroll
    for (int i = 0; i < WC; ++i) S.Om[kk][i] = beta * S.Om[kk][i] - mx;
  }
  __builtin_amdgcn_wave_barrier();
  // exponentials of the W(W+1)/2 (k, i) pairs, spread over the lanes
  for (int p = lane; p < W * (W + 1) / 2; p += 64) {
    int k = (int)((sqrtf(8.0f * (float)p + 1.0f) - 1.0f) * 0.5f);
    while (k * (k + 1) / 2 > p) --k;
    while ((k + 1) * (k + 2) / 2 <= p) ++k;
    const int i = p - k * (k + 1) / 2;
    S.Om[k][i] = exp(S.Om[k][i]);
  }
  __builtin_amdgcn_wave_barrier();
  if (kk < W) {
    double z = 0.0;
#pragma unroll
    for (int i = 0; i < WC; ++i)
      if (i <= kk) z += S.Om[kk][i];
    S.zinv[kk] = 1.0 / z;
  }
  __builtin_amdgcn_wave_barrier();
  if (kk < W) {
    double sum = 0.0;
#pragma unroll
    for (int k2 = 0; k2 < WC; ++k2)
      if (k2 >= kk && (!RT || k2 < W)) sum += S.Om[k2][kk] * S.zinv[k2];
    S.av[kk] = sum / (double)W;
  }
  __builtin_amdgcn_wave_barrier();
  for (int d = lane; d < AS_HEAD_DIM; d += 64) {
    double o = S.av[0] * (double)S.Rf[WC * RW + d];
#pragma unroll
    for (int i = 1; i < WC; ++i)
      if (!RT || i < W) o += S.av[i] * (double)S.Rf[(i - 1) * RW + d];
    out[d] = (float)o;
  }
  __builtin_amdgcn_wave_barrier();
}

}  // namespace asx
