// Score assembly from the integer statistics (paper Section 3.4): per-sentence scores, and the
// corpus variant that sums numerators, denominators and lengths over the batch first.
#include "tb_kernels.h"
#include "tb_score.h"

namespace tb {

struct FinalArgs {
  Problem pb;
  StatPtrs st;
  ScoreParams sp;
  void* out;  // fp32 or bfloat16 scores (sp.out_bf16)
  const int32_t* overflow;  // [B] or null: groups whose dictionary overflowed score NaN
};

// One lane per sentence.
__global__ __launch_bounds__(256) void sentence_score_kernel(FinalArgs a) {
  const Problem& pb = a.pb;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= pb.B) return;
  const int c = clamped_len(pb.cand_len[i], pb.cand_stride, pb.status);
  const RefRows rr = ref_rows(pb, i, true);
  const int r = closest_ref_len(c, pb.ref_len + rr.row0, rr.used, pb.ref_stride, pb.status);
  a.st.closest[i] = r;
  int cl[8], to[8];
#pragma unroll
  for (int n = 0; n < 8; ++n) {
    cl[n] = (n < pb.N) ? a.st.clipped[int64_t(i) * pb.N + n] : 0;
    to[n] = (n < pb.N) ? a.st.total[int64_t(i) * pb.N + n] : 0;
  }
  // a group whose statistics are not trustworthy must not pass for a reward
  const bool spoilt = a.overflow && a.overflow[i] != 0;
  store_score(a.out, i, spoilt ? __int_as_float(0x7FC00000) : bleu_from_stats<int>(cl, to, c, r, a.sp),
              a.sp.out_bf16);
}

__device__ __forceinline__ long long wave_sum64(long long v) {
#pragma unroll
  for (int d = kWave / 2; d > 0; d >>= 1) {
    int lo = __shfl_down(int(uint32_t(uint64_t(v))), d, kWave);
    int hi = __shfl_down(int(uint32_t(uint64_t(v) >> 32)), d, kWave);
    v += (long long)((uint64_t(uint32_t(hi)) << 32) | uint32_t(lo));
  }
  return v;
}

// A single workgroup strides over the batch, reduces the 2N+2 integer sums with wavefront
// shuffles and LDS, and lane 0 forms the corpus score.
__global__ __launch_bounds__(1024) void corpus_kernel(FinalArgs a, int write_score) {
  __shared__ long long part[16][18];
  const Problem& pb = a.pb;
  long long acc[18];  // clipped_1..8, total_1..8, candidate lengths, closest reference lengths
#pragma unroll
  for (int k = 0; k < 18; ++k) acc[k] = 0;
  for (int i = threadIdx.x; i < pb.B; i += blockDim.x) {
    const int c = clamped_len(pb.cand_len[i], pb.cand_stride, pb.status);
    const RefRows rr = ref_rows(pb, i, true);
    const int r = closest_ref_len(c, pb.ref_len + rr.row0, rr.used, pb.ref_stride, pb.status);
    a.st.closest[i] = r;
#pragma unroll
    for (int n = 0; n < 8; ++n) {
      if (n < pb.N) {
        acc[n] += a.st.clipped[int64_t(i) * pb.N + n];
        acc[8 + n] += a.st.total[int64_t(i) * pb.N + n];
      }
    }
    acc[16] += c;
    acc[17] += r;
    if (a.overflow && a.overflow[i] != 0) acc[0] = (long long)(1) << 62;  // poisons the sums
  }
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
#pragma unroll
  for (int k = 0; k < 18; ++k) {
    const long long s = wave_sum64(acc[k]);
    if (lane == 0) part[wave][k] = s;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    const int nwaves = blockDim.x / kWave;
    long long tot[18];
    for (int k = 0; k < 18; ++k) {
      tot[k] = 0;
      for (int w = 0; w < nwaves; ++w) tot[k] += part[w][k];
    }
    for (int n = 0; n < pb.N; ++n) {
      a.st.corpus[n] = tot[n];
      a.st.corpus[pb.N + n] = tot[8 + n];
    }
    a.st.corpus[2 * pb.N] = tot[16];
    a.st.corpus[2 * pb.N + 1] = tot[17];
    const bool spoilt = tot[0] >= ((long long)(1) << 61);  // some group's dictionary overflowed
    if (write_score)
      store_score(a.out, 0,
                  spoilt ? __int_as_float(0x7FC00000)
                         : bleu_from_stats<long long>(tot, tot + 8, tot[16], tot[17], a.sp),
                  a.sp.out_bf16);
  }
}

// ROUGE-N from the overlap counts of the GLOBAL path, one lane per candidate: precision, recall
// and F against every reference in use; the best reference is the first one with the largest
// overlap / (candidate n-grams + beta^2 * reference n-grams), to which F is proportional (the
// same single-precision quotient as the fused kernel forms: both paths choose alike).
struct RougeFinalArgs {
  Problem pb;
  ScoreParams sp;
  const int32_t* overlap;   // [B, R] from the count pass
  void* prf;                // [B, 3]
  int32_t* overlap_out;     // [B, R] caller's array, or null (then `overlap` is the caller's)
  int32_t* best;            // [B] or null
  float beta2;
};

__global__ __launch_bounds__(256) void rouge_score_kernel(RougeFinalArgs a) {
  const Problem& pb = a.pb;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= pb.B) return;
  const int N = pb.N, R = pb.R;
  const RefRows rr = ref_rows(pb, i, true);
  const int used = rr.used;
  const int c = clamped_len(pb.cand_len[i], pb.cand_stride, pb.status);
  const float ct = float(max(c - N + 1, 0));
  int best_j = 0;
  float best_key = -1.0f, best_rt = 0.0f;
  int best_ov = 0;
  for (int j = 0; j < R; ++j) {
    const int ov = j < used ? a.overlap[int64_t(i) * R + j] : 0;
    if (a.overlap_out) a.overlap_out[int64_t(i) * R + j] = ov;
    if (j >= used) continue;
    const int len = clamped_len(pb.ref_len[rr.row0 + j], pb.ref_stride, pb.status);
    const float rt = float(max(len - N + 1, 0));
    const float key = ov > 0 ? float(ov) / __fmaf_rn(a.beta2, rt, ct) : 0.0f;
    if (key > best_key) {
      best_key = key;
      best_j = j;
      best_rt = rt;
      best_ov = ov;
    }
  }
  const float p = ct > 0.0f ? float(best_ov) / ct : 0.0f;
  const float r = best_rt > 0.0f ? float(best_ov) / best_rt : 0.0f;
  const float f = (p + r > 0.0f) ? (1.0f + a.beta2) * p * r / (r + a.beta2 * p) : 0.0f;
  store_score(a.prf, int64_t(i) * 3 + 0, p, a.sp.out_bf16);
  store_score(a.prf, int64_t(i) * 3 + 1, r, a.sp.out_bf16);
  store_score(a.prf, int64_t(i) * 3 + 2, f, a.sp.out_bf16);
  if (a.best) a.best[i] = best_j;
}

hipError_t launch_rouge_finalize(const Problem& pb, const ScoreParams& sp, const int32_t* overlap,
                                 const RougeOut& out, hipStream_t s) {
  RougeFinalArgs a;
  a.pb = pb;
  a.sp = sp;
  a.overlap = overlap;
  a.prf = out.prf;
  a.overlap_out = (out.overlap && out.overlap != overlap) ? out.overlap : nullptr;
  a.best = out.best;
  a.beta2 = out.beta2;
  hipLaunchKernelGGL(rouge_score_kernel, dim3((pb.B + 255) / 256), dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_finalize(const Problem& pb, const StatPtrs& st, const ScoreParams& sp,
                           bool sentence_scores, bool corpus_sums, bool corpus_score,
                           void* out_bleu, hipStream_t s, const int32_t* overflow) {
  FinalArgs a;
  a.pb = pb;
  a.st = st;
  a.sp = sp;
  a.out = out_bleu;
  a.overflow = overflow;
  if (sentence_scores) {
    const int blocks = (pb.B + 255) / 256;
    hipLaunchKernelGGL(sentence_score_kernel, dim3(blocks), dim3(256), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (corpus_sums || corpus_score) {
    hipLaunchKernelGGL(corpus_kernel, dim3(1), dim3(1024), 0, s, a, corpus_score ? 1 : 0);
    return hipGetLastError();
  }
  return hipSuccess;
}

}  // namespace tb
