// FUSED path: the whole per-sentence pipeline in one kernel, one workgroup per sentence group.
//
// Tokens of the candidate and its references are read from HBM once and staged in LDS; then, for
// each order n, the workgroup
//   1. inserts the candidate's n-grams into an LDS open-addressing table (the dictionary of
//      Section 3.2, restricted to the candidate: an n-gram that the candidate lacks cannot
//      contribute to min(candidate count, reference count)); the id of a distinct n-gram is the
//      candidate position whose insertion created its entry,
//   2. looks the reference n-grams up and bumps the 16-bit counter field that belongs to
//      (id, reference) -- one field per sequence keeps the sequences' counts apart, which is what
//      the offset of Section 3.3 step 1 achieves,
//   3. lets the thread that created an entry take the maximum over the reference fields and the
//      minimum with the candidate field (Section 3.3 step 3) and sum it,
// and finally wavefront 0 forms the brevity penalty, smoothing and geometric mean (Section 3.4),
// one order per lane.  HBM traffic is the tokens in and one score (plus optional integer
// statistics) out.  The same kernel, instantiated with ROUGE = true, scores ROUGE-N instead.
#include "tb_kernels.h"
#include "tb_score.h"

// Phase time stamps for tuning builds only (-DTB_STAMPS), as in the hierarchical kernels.
#ifdef TB_STAMPS
__device__ unsigned long long tb_fused_stamps[8192 * 32];
#define TB_FSTAMP(i) \
  do { if (threadIdx.x == 0 && blockIdx.x < 8192) tb_fused_stamps[blockIdx.x * 32 + (i)] = wall_clock64(); } while (0)
extern "C" int tb_debug_stamps_fused(unsigned long long* host, int count) {
  return int(hipMemcpyFromSymbol(host, HIP_SYMBOL(tb_fused_stamps), size_t(count) * 8));
}
#else
#define TB_FSTAMP(i) do {} while (0)
#endif

namespace tb {

constexpr int kMaxFusedSeqs = kWave;  // candidate + references handled by one lane each
constexpr uint32_t kEmptySlot = 0xFFFFFFFFu;
constexpr size_t kLdsForTwoWorkgroups = 78 * 1024;  // per workgroup, so that two share a CU

struct FusedArgs {
  Problem pb;
  StatPtrs st;
  ScoreParams sp;
  void* out;            // per-sentence scores (fp32 or bfloat16: sp.out_bf16), or null
  // ROUGE-N mode (fused_kernel<.., true>): order N = pb.N only
  void* rouge_prf;      // [B, 3] precision, recall, F of the best reference (same type)
  int32_t* rouge_overlap;  // [B, R] or null
  int32_t* rouge_best;  // [B] or null
  float beta2;          // beta squared
  int table_slots;      // power of two
  int table_shift;      // 32 - log2(table_slots)
  int words;            // 32-bit counter words per id: ceil((R + 1) / 2)
  int list_per_wave;    // work-list entries reserved for each wavefront
  int progress_priority;  // 1: wavefronts of a workgroup that is behind get the higher priority
  uint32_t off_ids, off_cnt, off_cstate, off_tok, off_list;
};

static size_t fused_layout(int slots, int64_t cand_stride, int64_t cap, int list_total, int words,
                           int tok_bytes, FusedPlan* plan) {
  size_t off = size_t(slots) * 4;
  plan->off_ids = off;
  off += size_t(slots) * 2;
  plan->off_cnt = off;
  off += (size_t(cand_stride) * words * 4 + 15) & ~size_t(15);  // cleared in 16-byte stores
  plan->off_cstate = off;
  off += size_t(cand_stride) * 4;
  plan->off_tok = off;
  off += (size_t(cap + 4) * tok_bytes + 3) & ~size_t(3);
  plan->off_list = off;
  off += size_t(list_total) * 4;
  return off;
}

bool plan_fused(int64_t cand_stride, int64_t ref_stride, int R, int N, int bits,
                FusedPlan* plan) {
  (void)N;
  if (R + 1 > kMaxFusedSeqs) return false;
  const int64_t cap = cand_stride + int64_t(R) * ref_stride;
  // list entries pack position (14 bits), id (12 bits) and sequence index (6 bits)
  if (cap > 12 * 1024 || cand_stride > 4096 || ref_stride > 65535) return false;
  // key = id * 2^bits + token, id < cand_stride, must stay below the all-ones empty marker
  if (bits > 31 || (uint64_t(cand_stride) << bits) > 0xFFFFFFFFull) return false;
  int t = 256;
  while (t < 1024 && cap > 4 * t) t *= 2;
  plan->threads = t;
  const int need = int((cap + t - 1) / t);
  plan->items = need <= 2 ? 2 : need <= 4 ? 4 : need <= 6 ? 6 : need <= 8 ? 8 : 12;
  plan->words = (R + 2) / 2;
  plan->tok_bytes = bits <= 16 ? 2 : 4;
  const int nwaves = t / kWave;
  const int64_t list_cap = int64_t(R) * ref_stride;
  plan->list_per_wave = int((list_cap + nwaves - 1) / nwaves);
  plan->list_per_wave = (plan->list_per_wave + kWave - 1) / kWave * kWave;
  const int list_total = plan->list_per_wave * nwaves;
  int base = 256;
  while (int64_t(base) * 3 < cand_stride * 4) base <<= 1;
  // the emptier the table the fewer probes; take the largest of 4x, 2x, 1x the minimum size
  // that still lets two workgroups share a compute unit, else the minimum size
  plan->table_slots = base;
  plan->lds_bytes =
      fused_layout(base, cand_stride, cap, list_total, plan->words, plan->tok_bytes, plan);
  for (int mult = 4; mult >= 2; mult >>= 1) {
    FusedPlan trial = *plan;
    const size_t bytes = fused_layout(base * mult, cand_stride, cap, list_total, plan->words,
                                      plan->tok_bytes, &trial);
    if (bytes + 1024 <= kLdsForTwoWorkgroups && base * mult <= 65536) {
      *plan = trial;
      plan->table_slots = base * mult;
      plan->lds_bytes = bytes;
      break;
    }
  }
  return plan->lds_bytes + 1024 <= size_t(kLdsBudget);
}

// The candidate's dictionary of one order: an open-addressing table of 32-bit keys with double
// hashing.  One 32-bit multiply hashes the key: the top bits of the product pick the slot, lower
// bits the (odd) probe step, so a probe sequence reaches every slot of the power-of-two table.
// A probe loop ends at the key or at an empty slot and needs no round limit: the odd step visits
// every slot of the power-of-two table, which is at most 3/4 full (only candidate n-grams are
// inserted, at most cand_stride of them) and written by this workgroup alone after clearing it.
// The loops have a single exit (one condition, no break):
// that halves the instructions the compiler emits per probe round.  (Measured on this hardware:
// plain divergent loops beat
// variants that keep all lanes in lock step until the slowest is done, and probing slot pairs
// or 4-slot buckets with wider LDS reads did not pay either.)
struct ProbeTable {
  uint32_t* slots;
  uint32_t mask;  // slots - 1
  int shift;      // 32 - log2(slots)

  static constexpr uint32_t kNotFound = 0xFFFFFFFFu;

  // Slot of `key`, or kNotFound.  Lanes with active == false return kNotFound.
  __device__ __forceinline__ uint32_t find(uint32_t key, bool active) const {
    uint32_t found = kNotFound;
    if (active) {
      const uint32_t h = key * 0x9E3779B1u;
      const uint32_t step = (h >> 3) | 1u;
      uint32_t s = h >> shift;
      uint32_t e = slots[s];
      while (int(e != key) & int(e != kEmptySlot)) {
        s = (s + step) & mask;
        e = slots[s];
      }
      found = (e == key) ? s : kNotFound;
    }
    return found;
  }

  // Claim-or-find for active lanes.  Returns the slot; *won is set where this call created
  // the entry.
  __device__ __forceinline__ uint32_t insert(uint32_t key, bool active, bool* won) const {
    uint32_t slot = 0;
    bool created = false;
    if (active) {
      const uint32_t h = key * 0x9E3779B1u;
      const uint32_t step = (h >> 3) | 1u;
      uint32_t s = h >> shift;
      uint32_t old = atomicCAS(&slots[s], kEmptySlot, key);
      while (int(old != kEmptySlot) & int(old != key)) {
        s = (s + step) & mask;
        old = atomicCAS(&slots[s], kEmptySlot, key);
      }
      created = old == kEmptySlot;
      slot = s;
    }
    *won = created;
    return slot;
  }
};

// One workgroup per sentence group.
//
// Keys are hierarchical: the order-n key of a position is (id of its (n-1)-gram prefix) * 2^bits
// + the n-th token, where the id of a distinct candidate n-gram is the candidate position that
// created its table entry (order-0 ids are 0).  By induction two positions carry the same
// order-n key exactly when their n-grams are equal, so the key never needs more than
// log2(cand_stride) + bits bits whatever n is, and one 32-bit LDS compare-and-swap claims a slot.
//
// A reference position whose n-gram is not in the candidate's table cannot match at any higher
// order either (a candidate n-gram extends only prefixes the candidate contains), so it is
// dropped.  Each wavefront owns a slice of the reference positions and keeps the survivors --
// position, id, sequence index packed in one word -- compacted in its own LDS work list, so the
// next order runs over full wavefronts; reading and appending stay inside the wavefront and
// need neither atomics nor extra barriers.
// SITEMS: token positions per thread (workgroup size * SITEMS >= tokens of a group).
// The scalar-register cap matters for occupancy: two 1024-thread workgroups per compute unit are
// eight wavefronts per SIMD, and on this hardware a kernel that allocates more than 80 scalar
// registers gets only seven (measured: the same kernel at 96 runs one workgroup per compute
// unit and takes 34 us instead of 25 us at the headline shape).
// ROUGE: the same pipeline scores ROUGE-N for n = N instead of BLEU: at the last order the
// creator of an entry adds min(candidate count, reference j's count) to an overlap sum per
// reference, and the tail turns the sums into precision, recall and F.
template <typename TokT, int SITEMS, bool ROUGE>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_num_sgpr(80)))
void fused_kernel(FusedArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int s_part[8];              // per order: clipped sum (low 16) | distinct count (high 16)
  __shared__ int s_end[kMaxFusedSeqs];   // end of each sequence in back-to-back token indices
  __shared__ int s_overlap[ROUGE ? kMaxFusedSeqs : 1];  // ROUGE: overlap with each reference
  const Problem& pb = a.pb;
  const int nt = blockDim.x, tid = threadIdx.x;
  const int lane = tid & (kWave - 1), nwaves = nt / kWave;
  // the wavefront's index as a scalar: loop bounds derived from it stay in scalar registers
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int g = blockIdx.x;
  const int R = pb.R, N = pb.N, T = a.table_slots;
  const uint32_t W = uint32_t(a.words);
  uint32_t* table = reinterpret_cast<uint32_t*>(smem);
  uint16_t* ids = reinterpret_cast<uint16_t*>(smem + a.off_ids);
  uint32_t* cnt = reinterpret_cast<uint32_t*>(smem + a.off_cnt);
  uint32_t* cstate = reinterpret_cast<uint32_t*>(smem + a.off_cstate);
  TokT* tok = reinterpret_cast<TokT*>(smem + a.off_tok);
  uint32_t* my_list = reinterpret_cast<uint32_t*>(smem + a.off_list) + wave * a.list_per_wave;
  const ProbeTable dict{table, uint32_t(T) - 1u, a.table_shift};
  const int bits = pb.bits;
  TB_FSTAMP(0);
  if (a.progress_priority) __builtin_amdgcn_s_setprio(3);  // staging: as the first order, below

  // lane j of every wavefront: length of sequence j and the inclusive prefix of lengths
  // (a reference beyond the candidate's reference count has length 0 and no say in the closest
  // reference length)
  const RefRows rr = ref_rows(pb, g, tid == 0);
  const int used = rr.used;
  int my_len = 0;
  if (lane <= used) {
    my_len = (lane == 0)
        ? clamped_len(pb.cand_len[g], pb.cand_stride, wave == 0 ? pb.status : nullptr)
        : clamped_len(pb.ref_len[rr.row0 + lane - 1], pb.ref_stride,
                      wave == 0 ? pb.status : nullptr);
  }
  const int incl = wave_inclusive_scan(my_len);
  if (wave == 0 && lane <= R) {
    s_end[lane] = incl;
  }
  if (tid < 8) s_part[tid] = 0;
  if (ROUGE && tid < kMaxFusedSeqs) s_overlap[tid] = 0;
  const int total_tokens = min(lane_value(incl, R), SITEMS * nt);
  const int cand_len = lane_value(my_len, 0);

  {
    // 16-byte stores (table and counters start on 16-byte boundaries and the counters' area is
    // a whole number of them)
    uint4* t4 = reinterpret_cast<uint4*>(table);
    for (int q = tid; q < T / 4; q += nt)
      t4[q] = make_uint4(kEmptySlot, kEmptySlot, kEmptySlot, kEmptySlot);
    uint4* c4 = reinterpret_cast<uint4*>(cnt);
    for (int q = tid; q < (cand_len * int(W) + 3) / 4; q += nt) c4[q] = make_uint4(0u, 0u, 0u, 0u);
    for (int s = tid; s < cand_len; s += nt) cstate[s] = 0;
  }

  // stage the tokens back to back: candidate, reference 0, reference 1, ...  All of a thread's
  // loads are issued before the first one is consumed (one round trip to memory, not one per
  // position).
  {
    // sequence of each position and where it begins: the 64 positions of a wavefront usually
    // lie in one sequence, which one ballot over the lanes holding the sequence ends finds
    int seq[SITEMS], begin[SITEMS];
    {
      const int ends = (lane <= R) ? incl : 0x7FFFFFFF;
      const int wave_first = __builtin_amdgcn_readfirstlane(tid - lane);
#pragma unroll
      for (int i = 0; i < SITEMS; ++i) {
        const int k0 = wave_first + i * nt;
        const int f0 = min(int(__popcll(__builtin_amdgcn_ballot_w64(ends <= k0))), R);
        int sq = f0, bg = f0 > 0 ? __builtin_amdgcn_readlane(incl, max(f0 - 1, 0)) : 0;
        if (k0 + kWave > __builtin_amdgcn_readlane(incl, f0)) {  // uniform: the block straddles
          const int f1 =
              min(int(__popcll(__builtin_amdgcn_ballot_w64(ends <= k0 + kWave - 1))), R);
          for (int q = f0; q < f1; ++q) {
            const int e = __builtin_amdgcn_readlane(incl, q);
            const bool ge = k0 + lane >= e;
            sq = ge ? q + 1 : sq;
            bg = ge ? e : bg;
          }
        }
        seq[i] = sq;
        begin[i] = bg;
      }
    }
    const int64_t cand_row = int64_t(g) * pb.cand_stride;
    const int64_t ref_rows = rr.row0 * pb.ref_stride;
    int32_t t[SITEMS];
#pragma unroll
    for (int i = 0; i < SITEMS; ++i) {
      const int k = tid + i * nt;
      t[i] = 0;
      if (k < total_tokens) {
        const int p = k - begin[i];
        t[i] = (seq[i] == 0)
            ? load_token(pb.cand, cand_row + p, pb.tok64)
            : load_token(pb.refs, ref_rows + int64_t(seq[i] - 1) * pb.ref_stride + p, pb.tok64);
      }
    }
    bool bad = false;
#pragma unroll
    for (int i = 0; i < SITEMS; ++i) {
      const int k = tid + i * nt;
      if (k < total_tokens) {
        // a token outside the vocabulary is reported and staged as 0, so that every key formed
        // from the staged tokens stays below the empty-slot marker
        const bool outside = uint32_t(t[i]) >= uint32_t(pb.vocab);
        tok[k] = TokT(outside ? 0 : t[i]);
        bad |= outside;
      }
    }
    if (bad && pb.status) atomicOr(pb.status, TB_DEV_TOKEN_RANGE);
  }
  // this wavefront's slice of the reference positions (order 1 reads it directly), and the
  // range of sequences the slice touches
  const int nref = total_tokens - cand_len;
  const int slice = min((nref + nwaves - 1) / nwaves, a.list_per_wave);
  const int slice_begin = cand_len + wave * slice;
  int todo = max(min(slice, total_tokens - slice_begin), 0);  // entries in this wave's list
  int f_lo = 0, f_hi = 0;
  for (int m = 1; m <= R; ++m) {
    const int bm = lane_value(incl, m - 1);
    f_lo += (slice_begin >= bm) ? 1 : 0;
    f_hi += (slice_begin + todo - 1 >= bm) ? 1 : 0;
  }
  __syncthreads();
  TB_FSTAMP(1);

#pragma unroll 1
  for (int n = 1; n <= N; ++n) {
    // Two workgroups share a compute unit, and its arbiter serves the older wavefronts first:
    // left alone, the workgroup dispatched first finishes early and the other one then runs
    // alone on a half-empty unit.  A workgroup that is behind (a lower order) therefore gets
    // the higher priority, which keeps the two within an order of each other.  (Only for
    // batches of at most two rounds of workgroups: with more, fresh workgroups at the highest
    // priority would hold up the nearly finished ones whose slots the next round waits for.)
    if (a.progress_priority) {
      switch (n) {
        case 1: __builtin_amdgcn_s_setprio(3); break;
        case 2: __builtin_amdgcn_s_setprio(2); break;
        case 3: __builtin_amdgcn_s_setprio(1); break;
        default: __builtin_amdgcn_s_setprio(0); break;
      }
    }
    if (n >= 2) __syncthreads();  // every slot of the previous order has been emptied

    // ---- A: candidate n-grams claim or find their entry
    for (int k = tid; k + n <= cand_len; k += nt) {
      const uint32_t pid = (cstate[k] >> 16) & 0xFFFu;
      const uint32_t key = (pid << bits) | uint32_t(tok[k + n - 1]);
      bool won;
      const uint32_t s = dict.insert(key, true, &won);
      if (won) ids[s] = uint16_t(k);
      cstate[k] = s | (won ? 0x80000000u : 0u);
    }
    __syncthreads();
    TB_FSTAMP(2 + (n - 1) * 3);

    // ---- B: candidate counts (field 0 of the entry's id) ...
    for (int k = tid; k + n <= cand_len; k += nt) {
      const uint32_t st = cstate[k];
      const uint32_t id = ids[st & 0xFFFFu];
      atomicAdd(&cnt[__umul24(id, W)], 1u);
      cstate[k] = (st & 0x8000FFFFu) | (id << 16);
    }
    // ... and this wavefront's reference positions: look up, count in the reference's field,
    // keep the ones that can still match at the next order
    int kept = 0;
    for (int e0 = 0; e0 < todo; e0 += kWave) {
      const int e = e0 + lane;
      const bool active = e < todo;
      uint32_t q, pid, f;
      if (n == 1) {
        q = uint32_t(min(slice_begin + e, total_tokens - 1));
        pid = 0;
        f = uint32_t(f_lo);
        for (int m = f_lo + 1; m <= f_hi; ++m)
          f += (q >= uint32_t(lane_value(incl, m - 1))) ? 1u : 0u;
      } else {
        const uint32_t ent = my_list[active ? e : 0];
        q = ent & 0x3FFFu;
        pid = (ent >> 14) & 0xFFFu;
        f = ent >> 26;
      }
      const uint32_t key = (pid << bits) | uint32_t(tok[q + uint32_t(n) - 1]);
      const uint32_t s = dict.find(key, active);
      uint32_t next = 0xFFFFFFFFu;
      if (s != ProbeTable::kNotFound) {
        const uint32_t id = ids[s];
        atomicAdd(&cnt[__umul24(id, W) + (f >> 1)], (f & 1u) ? 0x10000u : 1u);
        const bool more = n < N && uint32_t(s_end[f]) >= q + uint32_t(n) + 1u;
        next = more ? (q | (id << 14) | (f << 26)) : next;
      }
      // in-place compaction: the write cursor never passes the entries still to be read
      const unsigned long long m = __builtin_amdgcn_ballot_w64(next != 0xFFFFFFFFu);
      const uint32_t rank =
          __builtin_amdgcn_mbcnt_hi(uint32_t(m >> 32), __builtin_amdgcn_mbcnt_lo(uint32_t(m), 0u));
      if (next != 0xFFFFFFFFu) my_list[kept + int(rank)] = next;
      kept += int(__builtin_popcountll(m));
    }
    todo = kept;
    __syncthreads();
    TB_FSTAMP(3 + (n - 1) * 3);

    // ---- C: the position that created an entry clips it (max over the reference fields, min
    // with the candidate field), zeroes its counters and empties its slot
    int part = 0;
    for (int k = tid; k + n <= cand_len; k += nt) {
      const uint32_t st = cstate[k];
      if (st >> 31) {
        const uint32_t base = __umul24(uint32_t(k), W);
        const uint32_t w0 = cnt[base];
        const uint32_t cc = w0 & 0xFFFFu;  // candidate count; reference j is field j + 1
        uint32_t mx = w0 >> 16;
        cnt[base] = 0;
        if (ROUGE && n == N && min(cc, mx)) atomicAdd(&s_overlap[0], int(min(cc, mx)));
        for (uint32_t w = 1; w < W; ++w) {
          const uint32_t x = cnt[base + w];
          mx = max(mx, max(x & 0xFFFFu, x >> 16));
          cnt[base + w] = 0;
          if (ROUGE && n == N) {  // per reference: min(candidate count, its own count)
            const uint32_t m_lo = min(cc, x & 0xFFFFu), m_hi = min(cc, x >> 16);
            if (m_lo) atomicAdd(&s_overlap[2 * w - 1], int(m_lo));
            if (m_hi) atomicAdd(&s_overlap[2 * w], int(m_hi));
          }
        }
        part += int(min(cc, mx)) + 0x10000;
        table[st & 0xFFFFu] = kEmptySlot;
      }
    }
    part = wave_sum(part);
    if (lane == 0 && part != 0) atomicAdd(&s_part[n - 1], part);
    TB_FSTAMP(4 + (n - 1) * 3);
  }
  __syncthreads();
  TB_FSTAMP(2 + N * 3);

  // wavefront 0: lane n < N owns order n + 1 (statistics out, one logarithm each)
  if (wave == 0) {
    const int c = cand_len;
    const int sum = (lane < N) ? s_part[lane & 7] : 0;
    const int cn = sum & 0xFFFF;
    const int tn = max(c - lane, 0);
    if (lane < N) {
      a.st.clipped[int64_t(g) * N + lane] = cn;
      a.st.total[int64_t(g) * N + lane] = tn;
      a.st.distinct[int64_t(g) * N + lane] = int(uint32_t(sum) >> 16);
    }
    // closest reference length, the shorter one on ties (lane j holds the length of sequence j)
    int best = lane_value(my_len, 1), bd = abs(best - c);
    for (int j = 2; j <= used; ++j) {
      const int l = lane_value(my_len, j), d = abs(l - c);
      if (d < bd || (d == bd && l < best)) {
        best = l;
        bd = d;
      }
    }
    if (!ROUGE) {
      const float score = bleu_from_stats_wave(cn, tn, c, best, a.sp);
      if (lane == 0) {
        a.st.closest[g] = best;
        if (a.out) store_score(a.out, g, score, a.sp.out_bf16);
      }
    } else {
      // lane j = 1..used: reference j - 1.  F is proportional to overlap / (cand + beta^2 ref)
      // n-grams; the best reference is the first one with the largest such quotient.
      const bool ref_lane = lane >= 1 && lane <= used;
      const int ov = ref_lane ? s_overlap[(lane - 1) & (kMaxFusedSeqs - 1)] : 0;
      const float ct = float(max(c - N + 1, 0)), rt = float(max(my_len - N + 1, 0));
      const float key = (ref_lane && ov > 0) ? float(ov) / __fmaf_rn(a.beta2, rt, ct) : 0.0f;
      if (a.rouge_overlap && lane >= 1 && lane <= R)
        a.rouge_overlap[int64_t(g) * R + lane - 1] = ov;
      int best_j = 1;
      float best_key = __int_as_float(lane_value(__float_as_int(key), 1));
      for (int j = 2; j <= used; ++j) {
        const float kj = __int_as_float(lane_value(__float_as_int(key), j));
        if (kj > best_key) {
          best_key = kj;
          best_j = j;
        }
      }
      const float p = ct > 0.0f ? float(ov) / ct : 0.0f;
      const float r = rt > 0.0f ? float(ov) / rt : 0.0f;
      const float f = (p + r > 0.0f) ? (1.0f + a.beta2) * p * r / (r + a.beta2 * p) : 0.0f;
      if (lane == best_j) {
        store_score(a.rouge_prf, int64_t(g) * 3 + 0, p, a.sp.out_bf16);
        store_score(a.rouge_prf, int64_t(g) * 3 + 1, r, a.sp.out_bf16);
        store_score(a.rouge_prf, int64_t(g) * 3 + 2, f, a.sp.out_bf16);
        if (a.rouge_best) a.rouge_best[g] = best_j - 1;
      }
    }
  }
}

template <typename TokT, int SITEMS, bool ROUGE>
hipError_t launch_fused_mode(const FusedArgs& a, const FusedPlan& plan, int blocks,
                             hipStream_t s) {
  hipError_t e = grant_dynamic_lds(
      reinterpret_cast<const void*>(fused_kernel<TokT, SITEMS, ROUGE>), plan.lds_bytes);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((fused_kernel<TokT, SITEMS, ROUGE>), dim3(blocks), dim3(plan.threads),
                     plan.lds_bytes, s, a);
  return hipGetLastError();
}
template <typename TokT, int SITEMS>
hipError_t launch_fused_items(const FusedArgs& a, const FusedPlan& plan, int blocks,
                              hipStream_t s) {
  return a.rouge_prf ? launch_fused_mode<TokT, SITEMS, true>(a, plan, blocks, s)
                     : launch_fused_mode<TokT, SITEMS, false>(a, plan, blocks, s);
}

template <typename TokT>
hipError_t launch_fused_tok(const FusedArgs& a, const FusedPlan& plan, int blocks,
                            hipStream_t s) {
  switch (plan.items) {
    case 2: return launch_fused_items<TokT, 2>(a, plan, blocks, s);
    case 4: return launch_fused_items<TokT, 4>(a, plan, blocks, s);
    case 6: return launch_fused_items<TokT, 6>(a, plan, blocks, s);
    case 8: return launch_fused_items<TokT, 8>(a, plan, blocks, s);
    case 12: return launch_fused_items<TokT, 12>(a, plan, blocks, s);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_fused(const Problem& pb, const FusedPlan& plan, const StatPtrs& st,
                        const ScoreParams& sp, void* out_bleu_or_null, hipStream_t s,
                        const RougeOut* rouge) {
  FusedArgs a;
  a.pb = pb;
  a.st = st;
  a.sp = sp;
  a.out = out_bleu_or_null;
  a.rouge_prf = rouge ? rouge->prf : nullptr;
  a.rouge_overlap = rouge ? rouge->overlap : nullptr;
  a.rouge_best = rouge ? rouge->best : nullptr;
  a.beta2 = rouge ? rouge->beta2 : 1.0f;
  a.table_slots = plan.table_slots;
  int lg = 0;
  while ((1 << lg) < plan.table_slots) ++lg;
  a.table_shift = 32 - lg;
  a.words = plan.words;
  a.list_per_wave = plan.list_per_wave;
  {
    // workgroups a compute unit holds at once (2048 threads, 160 KB of LDS), times 256 units
    const int by_threads = 2048 / plan.threads;
    const int by_lds = int(size_t(kLdsBudget) / (plan.lds_bytes + 512));
    const int resident = 256 * (by_threads < by_lds ? by_threads : (by_lds < 1 ? 1 : by_lds));
    a.progress_priority = pb.B <= 2 * resident ? 1 : 0;
  }
  a.off_ids = uint32_t(plan.off_ids);
  a.off_cnt = uint32_t(plan.off_cnt);
  a.off_cstate = uint32_t(plan.off_cstate);
  a.off_tok = uint32_t(plan.off_tok);
  a.off_list = uint32_t(plan.off_list);
  return plan.tok_bytes == 2 ? launch_fused_tok<uint16_t>(a, plan, pb.B, s)
                             : launch_fused_tok<int32_t>(a, plan, pb.B, s);
}

}  // namespace tb
