// FUSED path: the whole per-sentence pipeline in one kernel, one workgroup per sentence group.
//
// Tokens of the candidate and its references are read from HBM once and staged in LDS; for each
// order n the workgroup
//   1. extends every position's packed key by one token (n-gram extraction, Section 3.1),
//   2. inserts the candidate's keys into an LDS open-addressing table (the dictionary of Section
//      3.2, restricted to the candidate: an n-gram that the candidate lacks cannot contribute to
//      min(candidate count, reference count)),
//   3. looks every reference n-gram up and bumps that reference's 16-bit counter of the slot
//      (the slot index is the compact id; one counter field per sequence keeps the sequences'
//      counts apart, which is what the offset of Section 3.3 step 1 achieves),
//   4. sweeps the slots: maximum over the reference fields, minimum with the candidate field,
//      summed (Section 3.3 step 3),
// and finally lane 0 forms the brevity penalty, smoothing and geometric mean (Section 3.4).
// HBM traffic is the tokens in and one score (plus optional integer statistics) out.
#include "tb_kernels.h"
#include "tb_score.h"

namespace tb {

constexpr int kMaxFusedSeqs = kWave;  // candidate + references handled by one lane each

struct FusedArgs {
  Problem pb;
  StatPtrs st;
  ScoreParams sp;
  float* out;          // per-sentence scores, or null
  int table_slots;     // power of two
  int table_shift;     // 32 - log2(table_slots)
  int words;           // 32-bit counter words per slot: ceil((R + 1) / 2)
  uint32_t off_cnt, off_tok;
};

bool plan_fused(int64_t cand_stride, int64_t ref_stride, int R, int N, int bits,
                FusedPlan* plan) {
  (void)N;
  if (R + 1 > kMaxFusedSeqs) return false;
  if (cand_stride > 65535 || ref_stride > 65535) return false;  // 16-bit counter fields
  const int64_t cap = cand_stride + int64_t(R) * ref_stride;
  if (cap > 12 * 1024) return false;
  int t = 256;
  while (t < 1024 && cap > 4 * t) t *= 2;
  plan->threads = t;
  const int need = int((cap + t - 1) / t);
  plan->items = need <= 2 ? 2 : need <= 4 ? 4 : need <= 6 ? 6 : need <= 8 ? 8 : 12;
  int slots = 256, lg = 8;
  while (int64_t(slots) * 3 < cand_stride * 4) {
    slots <<= 1;
    ++lg;
  }
  plan->table_slots = slots;
  // a key is (slot of the (n-1)-gram prefix) * 2^bits + last token
  plan->key_bytes = (lg + bits <= 31) ? 4 : 8;
  plan->words = (R + 2) / 2;
  size_t off = size_t(slots) * plan->key_bytes;
  plan->off_cnt = off;
  off += size_t(slots) * plan->words * 4;
  off = (off + 15) & ~size_t(15);
  plan->off_tok = off;
  off += size_t(cap) * 4;
  plan->lds_bytes = off;
  return off + 1024 <= size_t(kLdsBudget);
}

template <typename KeyT> struct KeyTraits;
template <> struct KeyTraits<uint32_t> {
  using Word = unsigned int;
  static constexpr Word kEmpty = 0xFFFFFFFFu;
  // One 32-bit multiply; the top bits of the product pick the slot, lower bits the probe step.
  static __device__ __forceinline__ uint32_t hash(Word k) { return k * 0x9E3779B1u; }
};
template <> struct KeyTraits<uint64_t> {
  using Word = unsigned long long;
  static constexpr Word kEmpty = ~0ull;
  static __device__ __forceinline__ uint32_t hash(Word k) {
    const uint32_t lo = uint32_t(k), hi = uint32_t(k >> 32);
    return (lo ^ ((hi << 15) | (hi >> 17))) * 0x9E3779B1u;
  }
};

// One workgroup per sentence group.  Each thread owns up to ITEMS token positions of the group's
// sequences (candidate first, then the references, back to back).
//
// Keys are hierarchical: the order-n key of a position is (slot that its (n-1)-gram prefix
// occupied in the order-(n-1) table) * 2^bits + the n-th token.  Two positions carry the same
// order-n key exactly when their n-grams are equal, because by induction a slot of the previous
// table stands for one distinct (n-1)-gram of the candidate.  The key therefore never needs more
// than log2(slots) + bits bits whatever n is, and a reference position whose prefix was not
// found in the candidate's table is dropped from all higher orders: no candidate n-gram can
// extend a prefix the candidate does not contain.
template <int ITEMS, typename KeyT>
__global__ __launch_bounds__(1024, (ITEMS <= 6 ? 8 : 4)) void fused_kernel(FusedArgs a) {
  using Traits = KeyTraits<KeyT>;
  using Word = typename Traits::Word;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int red[16][4];
  __shared__ int s_len[kMaxFusedSeqs];
  const Problem& pb = a.pb;
  const int nt = blockDim.x, tid = threadIdx.x;
  const int lane = tid & (kWave - 1), wave = tid / kWave;
  const int g = blockIdx.x;
  const int R = pb.R, N = pb.N, T = a.table_slots, W = a.words;
  Word* table = reinterpret_cast<Word*>(smem);
  uint32_t* cnt = reinterpret_cast<uint32_t*>(smem + a.off_cnt);
  int32_t* tok = reinterpret_cast<int32_t*>(smem + a.off_tok);
  const uint32_t mask = uint32_t(T) - 1u;
#ifdef TB_PHASE_CLOCKS
  long long ts[14];
  int nts = 0;
  ts[nts++] = clock64();
#endif

  // lane j of every wavefront: length of sequence j and the inclusive prefix of lengths
  int my_len = 0;
  if (lane <= R) {
    my_len = (lane == 0)
        ? clamped_len(pb.cand_len[g], pb.cand_stride, wave == 0 ? pb.status : nullptr)
        : clamped_len(pb.ref_len[int64_t(g) * R + lane - 1], pb.ref_stride,
                      wave == 0 ? pb.status : nullptr);
  }
  const int incl = wave_inclusive_scan(my_len);
  if (wave == 0 && lane <= R) s_len[lane] = my_len;
  const int total_tokens = min(lane_value(incl, R), ITEMS * nt);

  // clear the table and the counters once (afterwards each order resets the slots it created)
  for (int s = tid; s < T; s += nt) table[s] = Traits::kEmpty;
  for (int s = tid; s < T * W; s += nt) cnt[s] = 0;

  // which sequence each of this thread's token positions belongs to (boundaries are scalars)
  uint32_t info[ITEMS];  // tokens left in the sequence from this position (<= 255) | field << 8
  uint32_t cur[ITEMS];   // order 1: the token; later: slot of the position's current n-gram
  {
    int begin[ITEMS], end[ITEMS];
    const int e0 = lane_value(incl, 0);
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      info[i] = 0;
      begin[i] = 0;
      end[i] = e0;
    }
    for (int m = 1; m <= R; ++m) {
      const int bm = lane_value(incl, m - 1), em = lane_value(incl, m);
#pragma unroll
      for (int i = 0; i < ITEMS; ++i) {
        const bool ge = tid + i * nt >= bm;
        info[i] = ge ? uint32_t(m) : info[i];
        begin[i] = ge ? bm : begin[i];
        end[i] = ge ? em : end[i];
      }
    }
    // stage tokens in LDS
    const int32_t* cand_row = pb.cand + int64_t(g) * pb.cand_stride;
    const int32_t* ref_rows = pb.refs + int64_t(g) * R * pb.ref_stride;
    bool bad = false;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      const int k = tid + i * nt;
      const uint32_t j = info[i];
      cur[i] = 0;
      info[i] = 0;
      if (k < total_tokens) {
        const int p = k - begin[i];
        const int32_t t =
            (j == 0) ? cand_row[p] : ref_rows[int64_t(j - 1) * pb.ref_stride + p];
        tok[k] = t;
        bad |= (uint32_t(t) >= uint32_t(pb.vocab));
        cur[i] = uint32_t(t);
        info[i] = uint32_t(min(end[i] - k, 255)) | (j << 8);
      }
    }
    if (bad && pb.status) atomicOr(pb.status, TB_DEV_TOKEN_RANGE);
  }
  __syncthreads();
#ifdef TB_PHASE_CLOCKS
  ts[nts++] = clock64();
#endif

  int part[4] = {0, 0, 0, 0};  // per order: clipped sum (low 16 bits) | distinct count (high 16)
  const int bits = pb.bits;
#pragma unroll
  for (int n = 1; n <= 4; ++n) {
    if (n > N) break;
    if (n >= 2) __syncthreads();  // the previous order's slots have all been reset

    // candidate n-grams: claim or find the slot, count in field 0
    uint32_t win = 0;  // bit i: this thread's item i created its slot
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      if (int(info[i] & 0xFFu) >= n && (info[i] >> 8) == 0) {
        Word key = cur[i];
        if (n >= 2) key = (key << bits) | Word(uint32_t(tok[tid + i * nt + n - 1]));
        const uint32_t h = Traits::hash(key);
        const uint32_t step = (h >> 3) | 1u;
        uint32_t s = h >> a.table_shift;
        for (int guard = T; guard > 0; --guard) {  // T probes visit every slot
          const Word old = atomicCAS(&table[s], Traits::kEmpty, key);
          if (old == Traits::kEmpty) win |= 1u << i;
          if (old == Traits::kEmpty || old == key) break;
          s = (s + step) & mask;
        }
        atomicAdd(&cnt[__umul24(s, uint32_t(W))], 1u);
        cur[i] = s;
      }
    }
    __syncthreads();
#ifdef TB_PHASE_CLOCKS
    ts[nts++] = clock64();
#endif

    // reference n-grams: look up; count in the reference's own 16-bit field, or retire the
    // position when the candidate has no such n-gram
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      const uint32_t f = info[i] >> 8;
      if (int(info[i] & 0xFFu) >= n && f != 0) {
        Word key = cur[i];
        if (n >= 2) key = (key << bits) | Word(uint32_t(tok[tid + i * nt + n - 1]));
        const uint32_t h = Traits::hash(key);
        const uint32_t step = (h >> 3) | 1u;
        uint32_t s = h >> a.table_shift;
        bool found = false;
        for (int guard = T; guard > 0; --guard) {
          const Word w = table[s];
          found = (w == key);
          if (found || w == Traits::kEmpty) break;
          s = (s + step) & mask;
        }
        if (found) {
          atomicAdd(&cnt[__umul24(s, uint32_t(W)) + (f >> 1)], (f & 1u) ? 0x10000u : 1u);
          cur[i] = s;
        } else {
          info[i] = 0;
        }
      }
    }
    __syncthreads();
#ifdef TB_PHASE_CLOCKS
    ts[nts++] = clock64();
#endif

    // the thread that created a slot clips it (max over reference fields, min with the
    // candidate field) and resets it for the next order
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      if (win & (1u << i)) {
        const uint32_t base = __umul24(cur[i], uint32_t(W));
        const uint32_t w0 = cnt[base];
        uint32_t m = w0 >> 16;
        cnt[base] = 0;
        for (int w = 1; w < W; ++w) {
          const uint32_t x = cnt[base + w];
          m = max(m, max(x & 0xFFFFu, x >> 16));
          cnt[base + w] = 0;
        }
        part[n - 1] += int(min(w0 & 0xFFFFu, m)) + 0x10000;
        table[cur[i]] = Traits::kEmpty;
      }
    }
#ifdef TB_PHASE_CLOCKS
    ts[nts++] = clock64();
#endif
  }

  // reduce the packed per-thread partial sums of all orders
#pragma unroll
  for (int n = 0; n < 4; ++n) {
    const int p = wave_sum(part[n]);
    if (lane == 0) red[wave][n] = p;
  }
  __syncthreads();
  if (wave == 0) {
    const int nwaves = nt / kWave;
    int sums[4];
#pragma unroll
    for (int n = 0; n < 4; ++n) sums[n] = wave_sum(lane < nwaves ? red[lane][n] : 0);
    if (lane == 0) {
      int clipped[4] = {0, 0, 0, 0}, total[4] = {0, 0, 0, 0};
      const int c = s_len[0];
#pragma unroll
      for (int n = 0; n < 4; ++n) {
        if (n < N) {
          clipped[n] = sums[n] & 0xFFFF;
          total[n] = max(c - n, 0);
          a.st.clipped[int64_t(g) * N + n] = clipped[n];
          a.st.total[int64_t(g) * N + n] = total[n];
          a.st.distinct[int64_t(g) * N + n] = int(uint32_t(sums[n]) >> 16);
        }
      }
      int best = s_len[1], bd = abs(best - c);
      for (int j = 2; j <= R; ++j) {
        const int l = s_len[j], d = abs(l - c);
        if (d < bd || (d == bd && l < best)) {
          best = l;
          bd = d;
        }
      }
      a.st.closest[g] = best;
      if (a.out) a.out[g] = bleu_from_stats<int>(clipped, total, c, best, a.sp);
#ifdef TB_PHASE_CLOCKS
      for (int q = 0; q < 4; ++q) {
        a.st.clipped[int64_t(g) * N + q] = int(ts[2 + 3 * q] - ts[1 + 3 * q]);
        a.st.total[int64_t(g) * N + q] = int(ts[3 + 3 * q] - ts[2 + 3 * q]);
        a.st.distinct[int64_t(g) * N + q] = int(ts[4 + 3 * q] - ts[3 + 3 * q]);
      }
      a.st.closest[g] = int(ts[1] - ts[0]);
      a.out[g] = float(clock64() - ts[0]);
#endif
    }
  }
}

template <int ITEMS, typename KeyT>
hipError_t launch_fused_items(const FusedArgs& a, int blocks, int threads, size_t lds,
                              hipStream_t s) {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(fused_kernel<ITEMS, KeyT>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, int(lds));
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((fused_kernel<ITEMS, KeyT>), dim3(blocks), dim3(threads), lds, s, a);
  return hipGetLastError();
}

template <typename KeyT>
hipError_t launch_fused_key(const FusedArgs& a, const FusedPlan& plan, int blocks,
                            hipStream_t s) {
  switch (plan.items) {
    case 2: return launch_fused_items<2, KeyT>(a, blocks, plan.threads, plan.lds_bytes, s);
    case 4: return launch_fused_items<4, KeyT>(a, blocks, plan.threads, plan.lds_bytes, s);
    case 6: return launch_fused_items<6, KeyT>(a, blocks, plan.threads, plan.lds_bytes, s);
    case 8: return launch_fused_items<8, KeyT>(a, blocks, plan.threads, plan.lds_bytes, s);
    case 12: return launch_fused_items<12, KeyT>(a, blocks, plan.threads, plan.lds_bytes, s);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_fused(const Problem& pb, const FusedPlan& plan, const StatPtrs& st,
                        const ScoreParams& sp, float* out_bleu_or_null, hipStream_t s) {
  FusedArgs a;
  a.pb = pb;
  a.st = st;
  a.sp = sp;
  a.out = out_bleu_or_null;
  a.table_slots = plan.table_slots;
  int lg = 0;
  while ((1 << lg) < plan.table_slots) ++lg;
  a.table_shift = 32 - lg;
  a.words = plan.words;
  a.off_cnt = uint32_t(plan.off_cnt);
  a.off_tok = uint32_t(plan.off_tok);
  return plan.key_bytes == 4 ? launch_fused_key<uint32_t>(a, plan, pb.B, s)
                             : launch_fused_key<uint64_t>(a, plan, pb.B, s);
}

}  // namespace tb
