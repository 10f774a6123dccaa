// Scalar tail of BLEU on the device: closest reference length, brevity penalty, smoothing and
// the weighted geometric mean (paper Section 3.4 and the BLEU equation of Section 2.1), fp32.
#pragma once

#include "tb_common.h"

namespace tb {

// Reference length closest to c; the shorter one on ties.  R >= 1.
__device__ __forceinline__ int closest_ref_len(int c, const int32_t* ref_len, int R,
                                               int64_t ref_stride, int32_t* status) {
  int best = clamped_len(ref_len[0], ref_stride, status);
  int bd = abs(best - c);
  for (int j = 1; j < R; ++j) {
    int l = clamped_len(ref_len[j], ref_stride, status);
    int d = abs(l - c);
    if (d < bd || (d == bd && l < best)) {
      best = l;
      bd = d;
    }
  }
  return best;
}

// BP * exp(sum_n w_n log p_n) from integer statistics.  `clipped` / `total` are read through
// a functor-free pair of arrays of any integer type convertible to float.
template <typename IntT>
__device__ __forceinline__ float bleu_from_stats(const IntT* clipped, const IntT* total, IntT c,
                                                 IntT r, const ScoreParams& sp) {
  if (c == 0 || clipped[0] == 0) return 0.0f;
  float logsum = 0.0f;
  int zeros_seen = 0;
#pragma unroll
  for (int n = 1; n <= 4; ++n) {
    if (n > sp.N) break;
    const IntT cn = clipped[n - 1];
    const IntT tn = total[n - 1];
    const float num = float(cn);
    const float den = float(tn < 1 ? IntT(1) : tn);
    float p;
    if (sp.smoothing == TB_SMOOTH_FLOOR) {
      p = (cn == 0) ? sp.param / den : num / den;
    } else if (sp.smoothing == TB_SMOOTH_ADD_K) {
      p = (n >= 2) ? (num + sp.param) / (den + sp.param) : num / den;
    } else if (sp.smoothing == TB_SMOOTH_EXP) {
      if (cn == 0) {
        zeros_seen += 1;
        p = 1.0f / (ldexpf(1.0f, zeros_seen) * den);
      } else {
        p = num / den;
      }
    } else {
      p = num / den;
    }
    const float w = sp.w[n - 1];
    if (w == 0.0f) continue;
    if (!(p > 0.0f)) return 0.0f;
    logsum += w * logf(p);
  }
  const float bp = (c > r) ? 1.0f : expf(1.0f - float(r) / float(c));
  return bp * expf(logsum);
}

}  // namespace tb
