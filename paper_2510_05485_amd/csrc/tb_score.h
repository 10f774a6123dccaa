// Scalar tail of BLEU on the device: closest reference length, brevity penalty, smoothing and
// the weighted geometric mean (paper Section 3.4 and the BLEU equation of Section 2.1), fp32.
#pragma once

#include "tb_common.h"

namespace tb {

// Reference length closest to c; the shorter one on ties.  No reference at all (possible with
// CSR reference lists only): 0.
__device__ __forceinline__ int closest_ref_len(int c, const int32_t* ref_len, int R,
                                               int64_t ref_stride, int32_t* status) {
  if (R < 1) return 0;
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

// w_n * log p_n for order n (1-based), with p_n the smoothed modified precision.
// zeros_seen: how many of the orders 1..n have a zero numerator (used by the 'exp' smoothing).
// Returns 0 when w_n = 0 (the order is skipped); sets *dead when w_n != 0 and p_n = 0 (the
// score is then 0).  The product is rounded on its own (never fused into a following add), so
// that a serial and a lane-parallel evaluation give bit-identical scores.
template <typename IntT>
__device__ __forceinline__ float order_log_term(int n, IntT cn, IntT tn, int zeros_seen,
                                                const ScoreParams& sp, float w, bool* dead) {
  const float num = float(cn);
  const float den = float(tn < 1 ? IntT(1) : tn);
  float p;
  if (sp.smoothing == TB_SMOOTH_FLOOR) {
    p = (cn == 0) ? sp.param / den : num / den;
  } else if (sp.smoothing == TB_SMOOTH_ADD_K) {
    p = (n >= 2) ? (num + sp.param) / (den + sp.param) : num / den;
  } else if (sp.smoothing == TB_SMOOTH_EXP) {
    p = (cn == 0) ? 1.0f / (ldexpf(1.0f, zeros_seen) * den) : num / den;
  } else {
    p = num / den;
  }
  if (w == 0.0f) return 0.0f;
  if (!(p > 0.0f)) {
    *dead = true;
    return 0.0f;
  }
  return __fmul_rn(w, logf(p));
}

// BP * exp(sum_n w_n log p_n) from integer statistics.
template <typename IntT>
__device__ __forceinline__ float bleu_from_stats(const IntT* clipped, const IntT* total, IntT c,
                                                 IntT r, const ScoreParams& sp) {
  if (c == 0 || clipped[0] == 0) return 0.0f;
  float logsum = 0.0f;
  int zeros_seen = 0;
  bool dead = false;
#pragma unroll
  for (int n = 1; n <= 8; ++n) {
    if (n > sp.N) break;
    zeros_seen += (clipped[n - 1] == 0) ? 1 : 0;
    logsum = __fadd_rn(logsum, order_log_term<IntT>(n, clipped[n - 1], total[n - 1], zeros_seen,
                                                    sp, sp.w[n - 1], &dead));
  }
  if (dead) return 0.0f;
  const float bp = (c > r) ? 1.0f : expf(1.0f - float(r) / float(c));
  return bp * expf(logsum);
}

// The same score, bit for bit, computed by one wavefront: lane n < N holds the statistics of
// order n + 1, the four logarithms run side by side and so do the two exponentials.  All 64
// lanes must be active; the result is valid in every lane.
__device__ __forceinline__ float bleu_from_stats_wave(int cn, int tn, int c, int r,
                                                      const ScoreParams& sp) {
  const int lane = threadIdx.x & (kWave - 1);
  const bool order_lane = lane < sp.N;
  const unsigned long long zero_mask = __builtin_amdgcn_ballot_w64(order_lane && cn == 0);
  const int zeros_seen = __popcll(zero_mask & ((2ull << lane) - 1ull));  // orders 1..lane+1
  float w = sp.w[0];
#pragma unroll
  for (int n = 1; n < 8; ++n) w = (lane == n) ? sp.w[n] : w;
  bool dead = false;
  float t = 0.0f;
  if (order_lane) t = order_log_term<int>(lane + 1, cn, tn, zeros_seen, sp, w, &dead);
  const bool any_dead = __builtin_amdgcn_ballot_w64(dead) != 0ull;
  const int first_clipped = lane_value(cn, 0);
  float logsum = 0.0f;
#pragma unroll
  for (int n = 0; n < 8; ++n)
    logsum = __fadd_rn(logsum, __int_as_float(lane_value(__float_as_int(t), n)));
  const float x = lane == 0 ? logsum : 1.0f - float(r) / float(c);
  const float y = expf(x);
  const float e0 = __int_as_float(lane_value(__float_as_int(y), 0));
  const float e1 = __int_as_float(lane_value(__float_as_int(y), 1));
  if (c == 0 || first_clipped == 0 || any_dead) return 0.0f;
  return ((c > r) ? 1.0f : e1) * e0;
}

// Store score v as element i of `out`: fp32, or bfloat16 = the upper half of the fp32 pattern
// after rounding to nearest, ties to even (Section 6 names lower-precision scores as a direction;
// all arithmetic stays fp32, only the stored value is narrowed).  A NaN stays a quiet NaN.
__device__ __forceinline__ void store_score(void* out, int64_t i, float v, int out_bf16) {
  if (out_bf16) {
    const uint32_t u = __float_as_uint(v);
    const uint32_t rounded = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    const bool is_nan = (u & 0x7FFFFFFFu) > 0x7F800000u;
    static_cast<uint16_t*>(out)[i] = uint16_t(is_nan ? ((u >> 16) | 0x40u) : rounded);
  } else {
    static_cast<float*>(out)[i] = v;
  }
}

}  // namespace tb
