// CPU oracle for batched per-sentence / corpus token-ID BLEU (and ROUGE-N on the same counts).
//
// TEST INFRASTRUCTURE ONLY.  This file is the plain, slow definition that the HIP path is
// checked against.  It shares no code with the GPU library and must never be called from the
// product path: only tests, the smoke check and the benchmark's CPU-baseline leg use it.
//
// What it computes is the textbook definition that the paper's vectorised method reproduces
// exactly (Section 4.1 states agreement with a per-sentence dictionary count to < 1e-6):
//   * n-grams of order n are the length-n windows lying wholly inside a sequence's true length
//     ("valid n-grams", Section 3.2 step 1);
//   * a dictionary (here an ordered map keyed by the window's token list) gives each distinct
//     n-gram its count in the candidate and in every reference (Section 3.3 steps 1-2);
//   * the reference count used for clipping is the maximum over the references, and the clipped
//     count is the minimum of candidate count and that maximum (Section 3.3 step 3);
//   * numerators are sums of clipped counts, denominators the number of candidate n-grams
//     (Section 3.4), and the score is BP * exp(sum_n w_n log p_n) (Section 2.1, the BLEU equation);
//   * the corpus variant sums numerators, denominators and lengths over the batch first
//     (Section 3.4, second paragraph).
// No key packing, no hashing, no blocking: everything is fp64 and std::map.
//
// Where the paper is silent the readings are (each is also listed in the design notes):
//   BP          1 if c > r, exp(1 - r/c) if 0 < c <= r, 0 if c == 0   (Papineni et al. 2002)
//   r           the reference length closest to c; ties go to the shorter reference
//   zero 1-gram score 0 in every smoothing mode (checked before smoothing)
//   den_n       max(total_n, 1) when forming p_n; the reported total stays max(c-n+1, 0)
//   none        any p_n == 0 with w_n > 0 gives score 0
//   floor       clipped_n == 0  ->  p_n = eps / den_n            (Chen & Cherry 2014, method 1)
//   add-k       n >= 2: p_n = (clipped_n + k) / (den_n + k); n = 1 unsmoothed   (method 2)
//   exp         scanning n = 1..N, the z-th zero numerator gets p_n = 1 / (2^z den_n) (method 3)
//   weights     used as given; w_n == 0 drops order n from the sum
// Agreement of these readings with NLTK itself is "parity unpinned" (NLTK is not available);
// everything else is pinned by the closed forms and brute force in tests/.

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <map>
#include <thread>
#include <vector>

namespace {

using Gram = std::vector<int32_t>;
using Counter = std::map<Gram, int32_t>;

enum Smoothing { kNone = 0, kFloor = 1, kAddK = 2, kExp = 3 };

// Count the valid windows of order n of one sequence.
Counter count_ngrams(const int32_t* seq, int len, int n) {
  Counter c;
  for (int p = 0; p + n <= len; ++p) c[Gram(seq + p, seq + p + n)] += 1;
  return c;
}

// Reference length closest to c; the shorter one on ties.
int closest_ref_len(int c, const int32_t* ref_len, int R) {
  int best = ref_len[0];
  for (int j = 1; j < R; ++j) {
    int d = std::abs(ref_len[j] - c), db = std::abs(best - c);
    if (d < db || (d == db && ref_len[j] < best)) best = ref_len[j];
  }
  return best;
}

// BP * exp(sum w_n log p_n) from integer statistics (numerators, true totals, lengths).
double bleu_from_stats(const int64_t* clipped, const int64_t* total, int64_t c, int64_t r, int N,
                       const double* w, int smoothing, double param) {
  if (c == 0) return 0.0;
  if (clipped[0] == 0) return 0.0;
  double bp = (c > r) ? 1.0 : std::exp(1.0 - double(r) / double(c));
  double logsum = 0.0;
  int zeros_seen = 0;
  for (int n = 1; n <= N; ++n) {
    double num = double(clipped[n - 1]);
    double den = double(std::max<int64_t>(total[n - 1], 1));
    double p;
    switch (smoothing) {
      case kFloor:
        p = (clipped[n - 1] == 0) ? param / den : num / den;
        break;
      case kAddK:
        p = (n >= 2) ? (num + param) / (den + param) : num / den;
        break;
      case kExp:
        if (clipped[n - 1] == 0) {
          zeros_seen += 1;
          p = 1.0 / (std::ldexp(1.0, zeros_seen) * den);
        } else {
          p = num / den;
        }
        break;
      default:
        p = num / den;
    }
    if (w[n - 1] == 0.0) continue;
    if (p <= 0.0) return 0.0;
    logsum += w[n - 1] * std::log(p);
  }
  return bp * std::exp(logsum);
}

struct Args {
  const int32_t* cand; int64_t cand_stride; const int32_t* cand_len;
  const int32_t* refs; int64_t ref_stride; const int32_t* ref_len;
  int B, R, N; const double* w; int smoothing; double param;
  int32_t *clipped, *total, *closest, *group_distinct, *cand_distinct; double* bleu;
  const int32_t* ref_count;  // per candidate: how many of its R reference rows exist (null: R)
};

void score_sentence(const Args& a, int i) {
  const int32_t* cs = a.cand + int64_t(i) * a.cand_stride;
  int c = a.cand_len[i];
  // a candidate with fewer references simply has fewer: the definition over its own references
  const int Ri = a.ref_count ? a.ref_count[i] : a.R;
  int64_t clip64[8], tot64[8];
  for (int n = 1; n <= a.N; ++n) {
    Counter cc = count_ngrams(cs, c, n);
    Counter ref_max, group = cc;
    for (int j = 0; j < Ri; ++j) {
      const int32_t* rs = a.refs + (int64_t(i) * a.R + j) * a.ref_stride;
      Counter rc = count_ngrams(rs, a.ref_len[int64_t(i) * a.R + j], n);
      for (const auto& kv : rc) {
        int32_t& m = ref_max[kv.first];
        m = std::max(m, kv.second);
        group[kv.first] += 0;
      }
    }
    int64_t clipped = 0;
    for (const auto& kv : cc) {
      auto it = ref_max.find(kv.first);
      int32_t rm = (it == ref_max.end()) ? 0 : it->second;
      clipped += std::min(kv.second, rm);
    }
    int64_t total = std::max(c - n + 1, 0);
    clip64[n - 1] = clipped;
    tot64[n - 1] = total;
    int64_t o = int64_t(i) * a.N + (n - 1);
    a.clipped[o] = int32_t(clipped);
    a.total[o] = int32_t(total);
    if (a.group_distinct) a.group_distinct[o] = int32_t(group.size());
    if (a.cand_distinct) a.cand_distinct[o] = int32_t(cc.size());
  }
  int r = closest_ref_len(c, a.ref_len + int64_t(i) * a.R, Ri);
  a.closest[i] = r;
  a.bleu[i] = bleu_from_stats(clip64, tot64, c, r, a.N, a.w, a.smoothing, a.param);
}

}  // namespace

extern "C" {

// Per-sentence statistics and scores for a batch, plus the corpus-level score over the batch.
//   cand [B, cand_stride], cand_len [B], refs [B, R, ref_stride], ref_len [B, R]: host int32.
//   weights [N] fp64.  smoothing 0 none / 1 floor / 2 add-k / 3 exp with parameter `param`.
//   threads: sentences are split statically over this many std::threads (1 = serial).
// Outputs (host, caller-allocated): clipped/total [B, N], closest [B], bleu [B] fp64,
//   optional group_distinct / cand_distinct [B, N] (distinct n-grams over candidate+references,
//   and over the candidate alone), corpus_stats [2N+2] = clipped_1..N, total_1..N, sum c, sum r,
//   corpus_bleu [1].  ref_count [B] (may be null): candidate i has only its first ref_count[i]
//   reference rows, 1 <= ref_count[i] <= R.  Returns 0, or 1 on invalid arguments.
int oracle_bleu(const int32_t* cand, int64_t cand_stride, const int32_t* cand_len,
                const int32_t* refs, int64_t ref_stride, const int32_t* ref_len, int B, int R,
                int N, const double* weights, int smoothing, double param, int threads,
                int32_t* clipped, int32_t* total, int32_t* closest, int32_t* group_distinct,
                int32_t* cand_distinct, double* bleu, int64_t* corpus_stats,
                double* corpus_bleu, const int32_t* ref_count) {
  if (B < 0 || R < 1 || N < 1 || N > 8 || smoothing < 0 || smoothing > 3) return 1;
  if (ref_count)
    for (int i = 0; i < B; ++i)
      if (ref_count[i] < 1 || ref_count[i] > R) return 1;
  Args a{cand, cand_stride, cand_len, refs, ref_stride, ref_len, B, R, N, weights, smoothing,
         param, clipped, total, closest, group_distinct, cand_distinct, bleu, ref_count};
  int T = std::max(1, std::min(threads, std::max(B, 1)));
  if (T == 1) {
    for (int i = 0; i < B; ++i) score_sentence(a, i);
  } else {
    std::vector<std::thread> pool;
    for (int t = 0; t < T; ++t) {
      int lo = int(int64_t(B) * t / T), hi = int(int64_t(B) * (t + 1) / T);
      pool.emplace_back([&a, lo, hi] { for (int i = lo; i < hi; ++i) score_sentence(a, i); });
    }
    for (auto& th : pool) th.join();
  }
  if (corpus_stats || corpus_bleu) {
    int64_t cs[18] = {0};
    for (int i = 0; i < B; ++i) {
      for (int n = 0; n < N; ++n) {
        cs[n] += clipped[int64_t(i) * N + n];
        cs[N + n] += total[int64_t(i) * N + n];
      }
      cs[2 * N] += cand_len[i];
      cs[2 * N + 1] += closest[i];
    }
    if (corpus_stats) std::copy(cs, cs + 2 * N + 2, corpus_stats);
    if (corpus_bleu)
      *corpus_bleu = bleu_from_stats(cs, cs + N, cs[2 * N], cs[2 * N + 1], N, weights, smoothing,
                                     param);
  }
  return 0;
}

// Score from already-aggregated integer statistics (exposed so tests can pin the scalar part).
double oracle_bleu_from_stats(const int64_t* clipped, const int64_t* total, int64_t c, int64_t r,
                              int N, const double* weights, int smoothing, double param) {
  return bleu_from_stats(clipped, total, c, r, N, weights, smoothing, param);
}

// Per-distinct-n-gram counts of one sentence group for one order, in lexicographic key order.
// Fills up to `cap` rows of: gram tokens [cap, n], cand_count [cap], ref_max [cap].
// Returns the number of distinct n-grams over candidate + references (may exceed cap).
int oracle_group_counts(const int32_t* cand, int cand_len, const int32_t* refs,
                        int64_t ref_stride, const int32_t* ref_len, int R, int n, int cap,
                        int32_t* grams, int32_t* cand_count, int32_t* ref_max_out) {
  Counter cc = count_ngrams(cand, cand_len, n);
  std::map<Gram, std::pair<int32_t, int32_t>> all;
  for (const auto& kv : cc) all[kv.first].first = kv.second;
  for (int j = 0; j < R; ++j) {
    Counter rc = count_ngrams(refs + int64_t(j) * ref_stride, ref_len[j], n);
    for (const auto& kv : rc) {
      auto& e = all[kv.first];
      e.second = std::max(e.second, kv.second);
    }
  }
  int k = 0;
  for (const auto& kv : all) {
    if (k < cap) {
      std::copy(kv.first.begin(), kv.first.end(), grams + int64_t(k) * n);
      cand_count[k] = kv.second.first;
      ref_max_out[k] = kv.second.second;
    }
    ++k;
  }
  return k;
}

// ROUGE-N overlap counts of every candidate against each of its references, on the same counting
// definition (the paper names ROUGE as the first metric its counting method extends to, Section 6
// "Future Work"; the metric itself is Lin 2004): for one order n,
//   overlap[i][j] = sum over distinct n-grams g of min(count in candidate i, count in reference j).
// Precision, recall, F and the choice of the best reference are formed from these integers by the
// Python wrapper in exact rational arithmetic (oracle.rouge_n).
// ref_count as in oracle_bleu: entries of references beyond it stay 0.
// Returns 0, or 1 on invalid arguments.
int oracle_rouge_overlap(const int32_t* cand, int64_t cand_stride, const int32_t* cand_len,
                         const int32_t* refs, int64_t ref_stride, const int32_t* ref_len, int B,
                         int R, int n, const int32_t* ref_count, int32_t* overlap) {
  if (B < 0 || R < 1 || n < 1 || n > 8) return 1;
  for (int i = 0; i < B; ++i) {
    const int Ri = ref_count ? ref_count[i] : R;
    if (Ri < 1 || Ri > R) return 1;
    Counter cc = count_ngrams(cand + int64_t(i) * cand_stride, cand_len[i], n);
    for (int j = 0; j < R; ++j) overlap[int64_t(i) * R + j] = 0;
    for (int j = 0; j < Ri; ++j) {
      Counter rc = count_ngrams(refs + (int64_t(i) * R + j) * ref_stride,
                                ref_len[int64_t(i) * R + j], n);
      int64_t ov = 0;
      for (const auto& kv : cc) {
        auto it = rc.find(kv.first);
        if (it != rc.end()) ov += std::min(kv.second, it->second);
      }
      overlap[int64_t(i) * R + j] = int32_t(ov);
    }
  }
  return 0;
}

}  // extern "C"
