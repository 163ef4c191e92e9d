// Rows stage for kernels in which 16 lanes share one sample: lane m of the 16 holds the logits of classes
// m, 16 + m, ... of its row.  Probabilities with the log-sum-exp shift (Sections 2.2, 2.6), the row of D
// (eq. matrix-c) or of P - Y, the row loss, optional stores of P and of the logits; the sums over a row's
// classes are rotations inside the 16 lanes.
#pragma once

#include "nadmm_internal.h"
#include "nadmm_mfma.h"

namespace nadmm {
namespace rows16 {

// Which classes a lane holds: class 16 nb + m if that is below C-1 (valid), else the last class again so that
// loads stay inside the row.
template <int NB>
struct LaneClasses {
  int cl[NB];
  bool cv[NB];
  __device__ __forceinline__ LaneClasses(int m, int NC) {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      cv[nb] = 16 * nb + m < NC;
      cl[nb] = cv[nb] ? 16 * nb + m : NC - 1;
    }
  }
};

// One row.  z, w: the row's logits A X and A V (whichever operands the call has); pin: the cached probabilities
// (used when the call has no X); label: the row's class (kinds with a loss).  Returns the row loss in the lane
// with m == 0 of a valid row, 0 elsewhere and for kinds without a loss.
template <int NB>
__device__ __forceinline__ double finish(const RowArgs& a, int64_t row, int m, const LaneClasses<NB>& lc, bool has0,
                                         bool has1, const float (&z)[NB], const float (&w)[NB], const float (&pin)[NB],
                                         int label) {
  using mfma_detail::row16_max;
  using mfma_detail::row16_sum;
  const int NC = a.NC;
  const bool valid = row < a.n;
  const size_t ro = (size_t)(valid ? row : a.n - 1) * NC;
  if (a.kind == kRowsLogits) {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
      if (valid && lc.cv[nb]) {
        if (has0 && a.Z0out) a.Z0out[ro + lc.cl[nb]] = z[nb];
        if (has1 && a.Z1out) a.Z1out[ro + lc.cl[nb]] = w[nb];
      }
    return 0.0;
  }
  float P[NB];
  float M = 0.f, alpha = 1.f;
  if (has0) {
    float mx = 0.f;  // the reference class has logit 0
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) mx = fmaxf(mx, lc.cv[nb] ? z[nb] : 0.f);
    M = row16_max(mx);
    float es = 0.f;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      P[nb] = lc.cv[nb] ? expf(z[nb] - M) : 0.f;
      es += P[nb];
    }
    alpha = row16_sum(es) + expf(-M);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) P[nb] = P[nb] / alpha;
  } else {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) P[nb] = lc.cv[nb] ? pin[nb] : 0.f;
  }
  if (a.kind == kRowsHv) {
    float t = 0.f;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) t = fmaf(P[nb], w[nb], t);
    t = row16_sum(t);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
      if (valid && lc.cv[nb]) {
        a.rows_out[ro + lc.cl[nb]] = P[nb] * (w[nb] - t);
        if (a.Pout) a.Pout[ro + lc.cl[nb]] = P[nb];
      }
    return 0.0;
  }
  float zb = 0.f;
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const bool mine = lc.cv[nb] && 16 * nb + m == label;
    zb += mine ? z[nb] : 0.f;
    if (valid && lc.cv[nb]) {
      if (a.kind == kRowsGrad && a.rows_out) a.rows_out[ro + lc.cl[nb]] = P[nb] - (mine ? 1.f : 0.f);
      if (a.Pout) a.Pout[ro + lc.cl[nb]] = P[nb];
      if (a.Z0out) a.Z0out[ro + lc.cl[nb]] = z[nb];
    }
  }
  zb = row16_sum(zb);
  return (valid && m == 0) ? (double)M + (double)logf(alpha) - (double)zb : 0.0;
}

}  // namespace rows16
}  // namespace nadmm
