// GLOBAL path, dictionary and count/clip passes for groups that fit one LDS table, built on
// hierarchical keys.
//
// Dictionary (Section 3.2 step 2): one workgroup per sentence group walks the orders n = 1..N.
// Two n-grams of one order are equal exactly when their (n-1)-gram prefixes are equal and their
// last tokens are equal, and the order below has already numbered the prefixes; so the key that
// goes into the hash table is (id of the prefix, last token) -- at most log2(group_cap) + bits
// bits, a 32-bit word whatever n and the vocabulary are -- and every order, also one whose packed
// keys take 16 bytes, uses 4-byte table entries, one 32-bit LDS compare-and-swap per probe and a
// table at most 3/8 full for the usual shapes.  The last token of an n-gram is the low `bits`
// bits of its packed key, so the pass still reads the key array the pack pass wrote for every
// order (the low dword of each key: the memory system moves the same cache lines), and writes
// one offset id per n-gram.  The comparison is exact: no fingerprints, no lossy hashing.
// Ids are dense, and the n-grams that occur in the candidate get the lowest ones (their
// insertions run first): ids below cand_distinct[g][n] are exactly the candidate's n-grams.
//
// Count/clip (Section 3.3 steps 2-3): an n-gram the candidate lacks cannot contribute to
// min(candidate count, reference count), so counters exist only for the ids below
// cand_distinct: one 16-bit field per sequence of the group, for every order at once (a few tens
// of KB of LDS).  One workgroup per group streams the ids of all its orders with every load in
// flight from the start, bumps a field per occurrence (references skip ids at or above
// cand_distinct), and sweeps the few thousand entries once: maximum over the reference fields,
// minimum with the candidate field, sum.  Three barriers per workgroup.
#include <cstdio>
#include <cstdlib>
#include <type_traits>

#include "tb_group_index.h"
#include "tb_kernels.h"
#include "tb_score.h"

// Phase time stamps for tuning builds only (-DTB_STAMPS): thread 0 of every workgroup records the
// 100 MHz wall clock at phase boundaries; tb_debug_stamps copies them to the host.
#ifdef TB_STAMPS
__device__ unsigned long long tb_stamps[8192 * 32];
#define TB_STAMP(i) \
  do { const unsigned wg_ = blockIdx.y * gridDim.x + blockIdx.x; \
       if (threadIdx.x == 0 && wg_ < 8192) tb_stamps[wg_ * 32 + (i)] = wall_clock64(); } while (0)
extern "C" int tb_debug_stamps(unsigned long long* host, int count) {
  return int(hipMemcpyFromSymbol(host, HIP_SYMBOL(tb_stamps), size_t(count) * 8));
}
#else
#define TB_STAMP(i) do {} while (0)
#endif

namespace tb {

namespace {

constexpr int kHierMaxSeqs = 63;        // candidate + references, one lane each (lane 63 spare)
constexpr size_t kHierLdsPerWorkgroup = 72 * 1024;  // so that two workgroups share a CU

int ceil_log2_int(int64_t v) {
  int b = 0;
  while ((int64_t(1) << b) < v) ++b;
  return b;
}

struct HierDictArgs {
  Problem pb;
  GlobalWs ws;
  int32_t* distinct;       // [B, N] dictionary sizes
  int32_t* cand_distinct;  // [B, N] ids below this belong to n-grams the candidate contains
  int table_slots;         // power of two, > group_cap
  int table_shift;         // 32 - log2(table_slots)
};

// Sequence (0 = candidate) of token index k = k0 + lane, and one past the sequence's last token
// index.  `incl`: lane j holds the end of sequence j in the group's back-to-back token numbering
// (lanes beyond R repeat the total).  k0 is wave-uniform: the 64 positions of a wavefront
// usually lie inside one sequence, which one ballot finds; a block that straddles sequences
// walks the few ends inside it.  All 64 lanes must be active.
__device__ __forceinline__ void find_sequence(int k0, int lane, int incl, int R, int* seq,
                                              int* end) {
  const int ends = (lane <= R) ? incl : 0x7FFFFFFF;
  const int f0 = min(int(__popcll(__builtin_amdgcn_ballot_w64(ends <= k0))), R);
  int s = f0, e = __builtin_amdgcn_readlane(incl, f0);
  if (k0 + kWave > e) {  // uniform
    const int f_hi = min(int(__popcll(__builtin_amdgcn_ballot_w64(ends <= k0 + kWave - 1))), R);
    for (int q = f0; q < f_hi; ++q) {
      const bool ge = k0 + lane >= __builtin_amdgcn_readlane(incl, q);
      s = ge ? q + 1 : s;
      e = ge ? __builtin_amdgcn_readlane(incl, q + 1) : e;
    }
  }
  *seq = s;
  *end = e;
}

// Claim-or-find in the open-addressing table (double hashing; the plan keeps every key below the
// all-ones empty marker).  Single-exit probe loop.
__device__ __forceinline__ uint32_t hier_insert(uint32_t* table, uint32_t key, uint32_t mask,
                                                int shift, bool* won) {
  const uint32_t h = key * 0x9E3779B1u;
  const uint32_t step = (h >> 3) | 1u;
  uint32_t s = h >> shift;
  uint32_t old = atomicCAS(&table[s], kEmpty, key);
  // No round limit is needed: the odd step visits every slot of the power-of-two table, the
  // table has more slots than the group has n-grams (so an empty slot or the key itself is met
  // within table_slots probes), and only this workgroup writes the table after clearing it.
  while (int(old != kEmpty) & int(old != key)) {
    s = (s + step) & mask;
    old = atomicCAS(&table[s], kEmpty, key);
  }
  *won = old == kEmpty;
  return s;
}

// ITEMS: token positions per thread (threads * ITEMS >= tokens of a group).  Item i of thread t
// is the position k = t + i * threads of the group's tokens laid back to back (candidate,
// reference 0, ...), i.e. the n-gram that STARTS there, for every order it is valid for; its slot
// in the order-n arrays is k minus the n-gram starts lost by the sequences before it.
// (The scalar-register cap keeps two 1024-thread workgroups on a compute unit: eight wavefronts
// per SIMD need at most 80 scalar registers each on this hardware.)
template <int ITEMS>
__global__ __launch_bounds__(1024, (ITEMS <= 6 ? 8 : 4)) __attribute__((amdgpu_num_sgpr(80)))
void hier_dictionary_kernel(HierDictArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int s_delta[8 * kWave];  // [n-1][s]: order-1 slot minus order-n slot inside sequence s
  __shared__ int s_next[2];           // ids handed out to candidate-made / reference-made entries
  const Problem& pb = a.pb;
  const int nt = blockDim.x, tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int g = blockIdx.x;
  const int R = pb.R, N = pb.N, bits = pb.bits;
  uint32_t* table = reinterpret_cast<uint32_t*>(smem);
  const int T = a.table_slots;
  const uint32_t mask = uint32_t(T) - 1u;
  const int shift = a.table_shift;
  const uint32_t tokmask = (bits >= 32) ? 0xFFFFFFFFu : ((1u << bits) - 1u);
  const int clear_rows = __builtin_amdgcn_readfirstlane(T / (4 * nt));  // exact: see plan_hier
  const int64_t gslot = int64_t(g) * pb.group_cap;
  const uint32_t gbase = uint32_t(gslot);

  TB_STAMP(0);
  if (tid == 0 && a.ws.arrivals) a.ws.arrivals[g] = 0;  // counted up by the count kernel
  // lane j: stored length of sequence j (requested first, clamped once the key requests below
  // are out: a wavefront's loads return in order, so the lengths arrive first)
  const RefRows rr = ref_rows(pb, g);
  const int used = rr.used;
  // (two separate values, selected after the key requests are out: an if / else over one
  // variable makes the compiler wait for the vector load where the branches join)
  const int raw_cand = uniform_load(pb.cand_len, g);
  int raw_ref = 0;
  if (lane >= 1 && lane <= ref_rows_readable(pb, rr)) raw_ref = pb.ref_len[rr.row0 + lane - 1];
  // Low dwords of the order-1 keys, requested before the lengths are known: at order 1 the slot
  // of a position is the position itself (slots past the group's tokens hold stale bytes that
  // are never used).
  uint32_t prev[ITEMS], lo[ITEMS], lo_next[ITEMS];
  {
    const uint32_t kbytes = a.ws.wide[0] ? 16u : 8u;
    const unsigned char* kb = static_cast<const unsigned char*>(a.ws.keys[0]) + gslot * kbytes;
    const int last = int(pb.group_cap) - 1;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i)
      lo[i] = *reinterpret_cast<const uint32_t*>(kb + uint32_t(min(tid + i * nt, last)) * kbytes);
  }
  // clamped lengths (0 beyond the references in use) and their inclusive prefix; lanes beyond R
  // hold the group's token count
  const int cs = __builtin_amdgcn_readfirstlane(int(min(pb.cand_stride, int64_t(1) << 30)));
  const int rs = __builtin_amdgcn_readfirstlane(int(min(pb.ref_stride, int64_t(1) << 30)));
  const int raw_len = lane == 0 ? raw_cand : raw_ref;
  const int my_len = (lane <= used) ? min(max(raw_len, 0), lane == 0 ? cs : rs) : 0;
  const int incl = wave_inclusive_scan(my_len);
  const int total = min(lane_value(incl, R), ITEMS * nt);
  const int cand_len = min(lane_value(incl, 0), total);
  if (wave == 0) {
    for (int n = 1; n <= N; ++n) {
      const int lost = min(my_len, n - 1);  // n-gram starts sequence `lane` loses at order n
      s_delta[(n - 1) * kWave + lane] = wave_inclusive_scan(lost) - lost;
    }
  }
  // per item: sequence index and the number of orders the position is a valid start for
  int seq[ITEMS], nmax[ITEMS];
  {
    const int wave_first = __builtin_amdgcn_readfirstlane(tid - lane);
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      const int k0 = wave_first + i * nt;
      int end;
      find_sequence(k0, lane, incl, R, &seq[i], &end);
      nmax[i] = (k0 + lane < total) ? min(end - (k0 + lane), N) : 0;
    }
  }
  __syncthreads();  // s_delta is read from here on
  TB_STAMP(1);

  // low dword of the order-n key of item i (unconditional, clamped loads: see the narrow kernel)
  // (n = N + 1 is allowed and requests slot 0 of order N in every lane, one cache line: the
  // request stays unconditional, because a load under a branch makes the compiler wait for ALL
  // outstanding loads at the next use of an older one.)
  auto request_keys = [&](int n, uint32_t (&dst)[ITEMS]) {
    const int na = min(n, N);  // the array read
    const uint32_t kbytes = a.ws.wide[na - 1] ? 16u : 8u;
    const unsigned char* kb =
        static_cast<const unsigned char*>(a.ws.keys[na - 1]) + gslot * kbytes;
    const int* d = &s_delta[(na - 1) * kWave];
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      const int slot = tid + i * nt - d[seq[i]];
      dst[i] = *reinterpret_cast<const uint32_t*>(
          kb + uint32_t((nmax[i] >= n) ? slot : 0) * kbytes);
    }
  };

#pragma unroll
  for (int i = 0; i < ITEMS; ++i) prev[i] = 0u, lo_next[i] = 0u;

  // One order: `cur` holds its key dwords (requested one order earlier), the next order's are
  // requested into `nxt` first.  The caller alternates two register sets, so no copy (which
  // would have to wait for the id stores issued just before it) sits between the orders.
  auto run_order = [&](int n, uint32_t (&cur)[ITEMS], uint32_t (&nxt)[ITEMS]) {
#ifndef TB_NO_PRIO
    // Two workgroups share a compute unit, and its arbiter serves the older wavefronts first:
    // left alone, the workgroup dispatched first finishes early and the other one then runs
    // alone on a half-empty unit.  A workgroup that is behind (a lower order) therefore gets
    // the higher priority, which keeps the two within an order of each other.
    switch (n) {
      case 1: __builtin_amdgcn_s_setprio(3); break;
      case 2: __builtin_amdgcn_s_setprio(2); break;
      case 3: __builtin_amdgcn_s_setprio(1); break;
      default: __builtin_amdgcn_s_setprio(0); break;
    }
#endif
    request_keys(n + 1, nxt);
    {
      // (the table is a whole number of 16-byte rows of the workgroup: no lane is masked)
      uint4* t4 = reinterpret_cast<uint4*>(table) + tid;
      for (int r = 0; r < clear_rows; ++r) t4[r * nt] = make_uint4(kEmpty, kEmpty, kEmpty, kEmpty);
      if (tid < 2) s_next[tid] = 0;
    }
    __syncthreads();
    TB_STAMP(2 + (n - 1) * 5);

    uint32_t slot[ITEMS];
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) slot[i] = 0;
    uint32_t made_c = 0, made_r = 0;  // bit i: item i created its entry (candidate / reference position)
    // candidate positions first: their entries get the lowest ids
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      if (i * nt >= cand_len) break;  // uniform
      if (seq[i] == 0 && nmax[i] >= n) {
        bool won;
        slot[i] = hier_insert(table, (prev[i] << bits) | (cur[i] & tokmask), mask, shift, &won);
        made_c |= (won ? 1u : 0u) << i;
      }
    }
    uint32_t id_c = reserve_ids(__popc(made_c), &s_next[0]);
    __syncthreads();  // every candidate n-gram is in the table and numbered
    TB_STAMP(3 + (n - 1) * 5);
    const uint32_t uc = uint32_t(s_next[0]);
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      if ((i + 1) * nt <= cand_len) continue;  // uniform: candidate positions only
      if (seq[i] != 0 && nmax[i] >= n) {
        bool won;
        slot[i] = hier_insert(table, (prev[i] << bits) | (cur[i] & tokmask), mask, shift, &won);
        made_r |= (won ? 1u : 0u) << i;
      }
    }
    uint32_t id_r = uc + reserve_ids(__popc(made_r), &s_next[1]);
    __syncthreads();  // nobody compares keys any more: entries may now hold ids
    TB_STAMP(4 + (n - 1) * 5);
    {
      // a thread's created entries in item order: first those made by candidate positions
      const uint32_t made = made_c | made_r;
      const int from_cand = __popc(made_c);
      id_r -= uint32_t(from_cand);
      int j = 0;
#pragma unroll
      for (int i = 0; i < ITEMS; ++i) {
        if ((made >> i) & 1u) {
          table[slot[i]] = (j < from_cand ? id_c : id_r) + uint32_t(j);
          ++j;
        }
      }
    }
    __syncthreads();
    TB_STAMP(5 + (n - 1) * 5);
    {
      uint32_t* ginv = a.ws.inv[n - 1] + gslot;
      const int* d = &s_delta[(n - 1) * kWave];
#pragma unroll
      for (int i = 0; i < ITEMS; ++i) {
        if (nmax[i] >= n) {
          const uint32_t id = table[slot[i]];
          prev[i] = id;
          ginv[tid + i * nt - d[seq[i]]] = gbase + id;
        }
      }
    }
    if (tid == 0) {
      a.distinct[int64_t(g) * N + n - 1] = int(uc) + s_next[1];
      a.cand_distinct[int64_t(g) * N + n - 1] = int(uc);
    }
    __syncthreads();  // ids and counters read: the table may be cleared
    TB_STAMP(6 + (n - 1) * 5);
  };
#pragma unroll 1
  for (int n = 1; n <= N; n += 2) {
    run_order(n, lo, lo_next);
    if (n == N) break;
    run_order(n + 1, lo_next, lo);
  }
}

// ------------------------------------------------------------------------- count + clip

struct HierCountArgs {
  Problem pb;
  GlobalWs ws;
  StatPtrs st;
  const int32_t* cand_distinct;  // [B, N] written by the dictionary pass
  int words;       // 32-bit words of 16-bit fields per entry: ceil((R + 1) / 2)
  int order_words; // LDS words per order: cand_stride * words
  int split;       // workgroups per group; workgroup r takes the orders r + 1, r + 1 + split, ...
  // ROUGE-N (rouge_overlap != null): one workgroup per group counts order N only and, in its
  // sweep, sums min(candidate count, reference j's count) per reference into rouge_overlap[B, R]
  int32_t* rouge_overlap;
  // BLEU, whole calls (score_out != null): the last workgroup of a group to finish scores the
  // sentence from the group's statistics (Section 3.4); ws.arrivals counts the finished ones
  ScoreParams sp;
  void* score_out;
};

// Four consecutive offset ids, loaded with one 16-byte request.  A group's first slot is only
// 4-byte aligned (group_cap is arbitrary), which global memory instructions accept.
struct __attribute__((packed, aligned(4))) IdQuad {
  uint32_t v[4];
};

// ROWS: 16-byte requests per thread and order; a wavefront's request covers 256 consecutive
// slots (lane l: slots 4l .. 4l + 3 of the block), rows are 4 * threads slots apart.
// OPW: orders per workgroup (1 or 2; orders beyond N idle).
// The scalar work per block (its first sequence, the bounds, the branches) is shared by 256
// n-grams; a block inside one sequence runs four predicated atomics with a scalar field word and
// addend, a block that straddles sequences finds each slot's sequence per lane.
// SCORE: the whole-call variant that also scores the sentence (a.score_out; see HierCountArgs).
template <int ROWS, int OPW, bool SCORE>
__global__ __launch_bounds__(1024) void hier_count_kernel(HierCountArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int s_clipped[8];
  __shared__ int s_overlap[kWave];  // ROUGE-N: overlap with each reference
  const Problem& pb = a.pb;
  const int nt = blockDim.x, tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const bool rouge = a.rouge_overlap != nullptr;  // then split == 1, OPW == 1, order N only
  const int g = blockIdx.x;  // grid: (groups, workgroups per group)
  const int R = pb.R, N = pb.N;
  const int first_order = rouge ? N : int(blockIdx.y) + 1;
  const uint32_t W = uint32_t(a.words);
  const int cap = int(pb.group_cap);
  uint32_t* cnt = reinterpret_cast<uint32_t*>(smem);
  const int64_t gslot = int64_t(g) * pb.group_cap;
  const uint32_t gbase = uint32_t(gslot);

  TB_STAMP(0);
#ifndef TB_NO_PRIO
  // the workgroup that is behind gets the higher priority (see the dictionary kernel)
  __builtin_amdgcn_s_setprio(3);
#endif
  GroupIndex gi(pb, g, GroupIndex::WaveOnly{});  // the loads of the lengths go out first
  int uc[OPW];
#pragma unroll
  for (int o = 0; o < OPW; ++o)
    uc[o] = uniform_load(a.cand_distinct,
                         int64_t(g) * N + min(first_order + o * a.split, N) - 1);
  // counters of all orders: cleared while the lengths are on their way
  {
    uint4* c4 = reinterpret_cast<uint4*>(cnt);
    const int quads = (OPW * a.order_words + 3) / 4;
    for (int q = tid; q < quads; q += nt) c4[q] = make_uint4(0u, 0u, 0u, 0u);
    if (tid < 8) s_clipped[tid] = 0;
    if (tid < kWave) s_overlap[tid] = 0;
  }
  // Ids of every order of this workgroup, all requested before any is used, and only as far as
  // the order's n-gram count reaches (blocks beyond re-read its last ids, a cache hit; the id
  // arrays end with 16 spare bytes, so a request that starts at a group's last slot stays inside
  // the workspace): ragged batches move the ids that exist, nothing else.
  IdQuad id[OPW][ROWS];
  int count[OPW], ccnt[OPW], seq_end[OPW];
#pragma unroll
  for (int o = 0; o < OPW; ++o) {
    const int n = min(first_order + o * a.split, N);
    gi.set_order(n);
    count[o] = min(gi.start(R + 1), cap);
    ccnt[o] = gi.start(1);
    seq_end[o] = (lane <= R) ? gi.end_in_lane() : 0x7FFFFFFF;
    const uint32_t* ginv = a.ws.inv[n - 1] + gslot;
    const uint32_t last = uint32_t(max(count[o] - 1, 0));
#pragma unroll
    for (int i = 0; i < ROWS; ++i)
      id[o][i] = *reinterpret_cast<const IdQuad*>(
          reinterpret_cast<const unsigned char*>(ginv) + 4u * min(uint32_t(4 * (tid + i * nt)), last));
  }
  TB_STAMP(1);
  __syncthreads();
  TB_STAMP(2);

  const int wave_first = 4 * __builtin_amdgcn_readfirstlane(tid - lane);  // row 0 block of the wave
#pragma unroll
  for (int o = 0; o < OPW; ++o) {
    if (first_order + o * a.split > N) break;  // uniform
#ifndef TB_NO_PRIO
    if (2 * o < OPW)
      __builtin_amdgcn_s_setprio(2);
    else
      __builtin_amdgcn_s_setprio(1);
#endif
    // ids at or above u_c belong to n-grams the candidate lacks.  Candidate slots always hold
    // ids below it; the clamps only matter for a workspace the dictionary pass never filled,
    // where they keep every LDS access inside the order's counters.
    const uint32_t u_c = uint32_t(min(max(uc[o], 0), int(pb.cand_stride)));
    const uint32_t u_last = max(u_c, 1u) - 1u;
    uint32_t* ocnt = cnt + o * a.order_words;
#pragma unroll
    for (int i = 0; i < ROWS; ++i) {
      const int k0 = wave_first + 4 * i * nt;  // first slot of the wavefront's block
      if (k0 >= count[o]) break;               // uniform per wavefront
      const int f0 = __popcll(__builtin_amdgcn_ballot_w64(seq_end[o] <= k0));
      const int f0_end = __builtin_amdgcn_readlane(seq_end[o], f0);
      if (k0 + 4 * kWave <= f0_end) {  // the whole block lies in sequence f0
        if (f0 == 0) {
#pragma unroll
          for (int j = 0; j < 4; ++j)
            atomicAdd(&ocnt[__umul24(min(id[o][i].v[j] - gbase, u_last), W)], 1u);
        } else {
          const uint32_t word = uint32_t(f0 >> 1), addend = (f0 & 1) ? 0x10000u : 1u;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const uint32_t u = id[o][i].v[j] - gbase;
            if (u < u_c) atomicAdd(&ocnt[__umul24(u, W) + word], addend);
          }
        }
      } else {  // the block straddles sequences, or the end of the group: sequence per slot
        const int f_hi =
            __popcll(__builtin_amdgcn_ballot_w64(seq_end[o] <= k0 + 4 * kWave - 1));
        const int k = k0 + 4 * lane;
        int f[4] = {f0, f0, f0, f0};
        for (int q = f0; q < f_hi; ++q) {
          const int e = __builtin_amdgcn_readlane(seq_end[o], q);
#pragma unroll
          for (int j = 0; j < 4; ++j) f[j] += (k + j >= e) ? 1 : 0;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const uint32_t u = id[o][i].v[j] - gbase;
          if (k + j < count[o] && u < u_c)
            atomicAdd(&ocnt[__umul24(u, W) + uint32_t(f[j] >> 1)], (f[j] & 1) ? 0x10000u : 1u);
        }
      }
    }
  }
  TB_STAMP(3);
#ifndef TB_NO_PRIO
  __builtin_amdgcn_s_setprio(0);
#endif
  __syncthreads();
  TB_STAMP(4);

  // One sweep over the candidates' entries of every order.  A clipped sum never exceeds the
  // order's n-gram count (at most 65 535), so two orders share one 32-bit accumulator and one
  // wavefront reduction.
  uint32_t part[(OPW + 1) / 2];
#pragma unroll
  for (int o = 0; o < (OPW + 1) / 2; ++o) part[o] = 0;
#pragma unroll
  for (int o = 0; o < OPW; ++o) {
    if (first_order + o * a.split > N) break;
    const int u_c = min(max(uc[o], 0), int(pb.cand_stride));
    const uint32_t* ocnt = cnt + o * a.order_words;
    uint32_t sum = 0;
    auto sweep = [&](auto words) {  // words: compile-time W for the usual few references, or 0
      constexpr int kW = decltype(words)::value;
      for (int u = tid; u < u_c; u += nt) {
        const uint32_t* e = &ocnt[__umul24(uint32_t(u), W)];
        const uint32_t w0 = e[0];
        uint32_t m = w0 >> 16;
        if (kW > 0) {
#pragma unroll
          for (int q = 1; q < kW; ++q) m = max(m, max(e[q] & 0xFFFFu, e[q] >> 16));
        } else {
          for (uint32_t q = 1; q < W; ++q) m = max(m, max(e[q] & 0xFFFFu, e[q] >> 16));
        }
        sum += min(w0 & 0xFFFFu, m);
        if (rouge) {  // uniform; field j + 1 is reference j
          const uint32_t cc = w0 & 0xFFFFu;
          for (int j = 0; j < R; ++j) {
            const uint32_t w = e[(j + 1) >> 1];
            const uint32_t both = min(cc, ((j + 1) & 1) ? (w >> 16) : (w & 0xFFFFu));
            if (both) atomicAdd(&s_overlap[j], int(both));
          }
        }
      }
    };
    switch (W) {  // uniform
      case 1: sweep(std::integral_constant<int, 1>{}); break;
      case 2: sweep(std::integral_constant<int, 2>{}); break;
      case 3: sweep(std::integral_constant<int, 3>{}); break;
      default: sweep(std::integral_constant<int, 0>{}); break;
    }
    part[o / 2] += sum << (16 * (o & 1));
  }
#pragma unroll
  for (int o = 0; o < (OPW + 1) / 2; ++o) {
    const uint32_t sum = uint32_t(wave_sum(int(part[o])));
    if (lane == 0 && sum) {
      if (sum & 0xFFFFu) atomicAdd(&s_clipped[2 * o], int(sum & 0xFFFFu));
      if (sum >> 16) atomicAdd(&s_clipped[2 * o + 1], int(sum >> 16));
    }
  }
  __syncthreads();
  TB_STAMP(5);

  if (wave == 0) {
    // lane o < OPW: statistics of this workgroup's o-th order
    int cn = 0, tn = 0;
#pragma unroll
    for (int o = 0; o < OPW; ++o) {
      cn = (lane == o) ? s_clipped[o] : cn;
      tn = (lane == o) ? ccnt[o] : tn;
    }
    const int n = first_order + lane * a.split;
    if (!SCORE) {
      if (lane < OPW && n <= N) {
        a.st.clipped[int64_t(g) * N + n - 1] = cn;
        a.st.total[int64_t(g) * N + n - 1] = tn;
      }
    } else if (lane < OPW && n <= N) {
      // (stored with device-scope atomics: they are carried out where every compute unit of the
      // device sees them, which a plain store is only after a write-back of the whole L2)
      const int o1 = __hip_atomic_exchange(&a.st.clipped[int64_t(g) * N + n - 1], cn,
                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const int o2 = __hip_atomic_exchange(&a.st.total[int64_t(g) * N + n - 1], tn,
                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      // (the old values are asked for so that the atomics answer, which they do once done)
      asm volatile("" ::"v"(o1), "v"(o2) : "memory");
    }
    if (rouge && lane < R) a.rouge_overlap[int64_t(g) * R + lane] = s_overlap[lane];

    if (SCORE) {
      // An atomic returns once it has been carried out: after the wait every statistic of this
      // workgroup is in place, and only then does the workgroup announce its arrival.  The
      // workgroup whose arrival completes the group reads the others' statistics with
      // device-scope loads.  (No fence: a release fence writes back the whole L2.)
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      int arrived = 0;
      if (lane == 0)
        arrived = __hip_atomic_fetch_add(&a.ws.arrivals[g], 1, __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT);
      arrived = lane_value(arrived, 0);
      if (arrived == int(gridDim.y) - 1) {  // uniform
        const int my_len = gi.length_in_lane(), used = gi.refs_in_use();
        const int c = lane_value(my_len, 0);
        (void)ref_rows(pb, g, lane == 0);  // reports a reference count out of range
        // closest reference length, the shorter one on ties (lane j: length of sequence j)
        int best = 0;
        if (used >= 1) {
          best = lane_value(my_len, 1);
          int bd = abs(best - c);
          for (int j = 2; j <= used; ++j) {
            const int l = lane_value(my_len, j), d = abs(l - c);
            if (d < bd || (d == bd && l < best)) {
              best = l;
              bd = d;
            }
          }
        }
        // lane n < N: the statistics of order n + 1
        const int64_t stat = int64_t(g) * N + min(lane, N - 1);
        const int cn_read = __hip_atomic_load(&a.st.clipped[stat], __ATOMIC_RELAXED,
                                              __HIP_MEMORY_SCOPE_AGENT);
        const int tn_read = __hip_atomic_load(&a.st.total[stat], __ATOMIC_RELAXED,
                                              __HIP_MEMORY_SCOPE_AGENT);
        const int cn_all = lane < N ? cn_read : 0, tn_all = lane < N ? tn_read : 0;
        const float score = bleu_from_stats_wave(cn_all, tn_all, c, best, a.sp);
        if (lane == 0) {
          a.st.closest[g] = best;
          store_score(a.score_out, g, score, a.sp.out_bf16);
        }
      }
    }
  }
}

template <typename Kernel, typename ArgT>
hipError_t launch_lds(Kernel kernel, const ArgT& a, int64_t blocks, int threads, size_t lds,
                      hipStream_t s) {
  if (blocks <= 0 || blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
  hipError_t e = grant_dynamic_lds(reinterpret_cast<const void*>(kernel), lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kernel, dim3(uint32_t(blocks)), dim3(threads), lds, s, a);
  return hipGetLastError();
}

template <int ITEMS>
hipError_t launch_dict_items(const HierDictArgs& a, const HierPlan& plan, hipStream_t s) {
  return launch_lds(hier_dictionary_kernel<ITEMS>, a, a.pb.B, plan.threads, plan.dict_lds, s);
}

template <int ROWS, int OPW, bool SCORE>
hipError_t launch_count_variant(const HierCountArgs& a, int threads, hipStream_t s) {
  const size_t lds = size_t(OPW) * a.order_words * 4;
  hipError_t e = grant_dynamic_lds(
      reinterpret_cast<const void*>(hier_count_kernel<ROWS, OPW, SCORE>), lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((hier_count_kernel<ROWS, OPW, SCORE>),
                     dim3(uint32_t(a.pb.B), uint32_t(a.split)), dim3(threads), lds, s, a);
  return hipGetLastError();
}
template <int ROWS, int OPW>
hipError_t launch_count_shape(const HierCountArgs& a, int threads, hipStream_t s) {
  return a.score_out ? launch_count_variant<ROWS, OPW, true>(a, threads, s)
                     : launch_count_variant<ROWS, OPW, false>(a, threads, s);
}

hipError_t launch_count_rows(const HierCountArgs& a, int threads, int rows, int opw,
                             hipStream_t s) {
  switch (opw * 100 + rows) {
    case 101: return launch_count_shape<1, 1>(a, threads, s);
    case 102: return launch_count_shape<2, 1>(a, threads, s);
    case 103: return launch_count_shape<3, 1>(a, threads, s);
    case 104: return launch_count_shape<4, 1>(a, threads, s);
    case 106: return launch_count_shape<6, 1>(a, threads, s);
    case 201: return launch_count_shape<1, 2>(a, threads, s);
    case 202: return launch_count_shape<2, 2>(a, threads, s);
    case 203: return launch_count_shape<3, 2>(a, threads, s);
    case 204: return launch_count_shape<4, 2>(a, threads, s);
    case 206: return launch_count_shape<6, 2>(a, threads, s);
    default: return hipErrorInvalidValue;
  }
}

// Launch shape of the count/clip kernel: workgroup size, 16-byte requests per thread and order,
// orders per workgroup.
struct CountShape {
  int threads, rows, opw;
};

int rows_for(int64_t group_cap, int threads) {
  const int need = int((group_cap + 4 * threads - 1) / (4 * threads));
  for (int r : {1, 2, 3, 4, 6})
    if (r >= need) return r;
  return 0;
}

CountShape count_shape(const Problem& pb, const HierPlan& plan) {
  CountShape c{plan.count_threads, plan.count_rows, 1};
  // two orders per workgroup when single orders would make more workgroups than the GPU digests
  // well (measured: 16 384 workgroups of 128 threads lose to 8192 with two orders each)
  if (int64_t(pb.B) * pb.N > 8192 && plan.count_pairs_fit) c.opw = 2;
#ifdef TB_STAMPS
  if (const char* e = getenv("TB_COUNT_SHAPE")) {  // tuning builds: "threads,opw"
    int t = 0, o = 0;
    if (sscanf(e, "%d,%d", &t, &o) == 2 && rows_for(pb.group_cap, t) > 0) {
      c.threads = t;
      c.rows = rows_for(pb.group_cap, t);
      c.opw = o;
    }
  }
#endif
  return c;
}

}  // namespace

bool plan_hier(int64_t group_cap, int64_t cand_stride, int64_t ref_stride, int R, int N, int bits,
               HierPlan* plan) {
  if (R + 1 > kHierMaxSeqs || group_cap < 4 || group_cap > 12 * 1024) return false;
  if (cand_stride > 65535 || ref_stride > 65535) return false;  // 16-bit counter fields
  // key = id * 2^bits + token, id < group_cap, must stay below the all-ones empty marker
  if (bits > 31 || (uint64_t(group_cap) << bits) > 0xFFFFFFFFull) return false;
  int t = 256;
  while (t < 1024 && group_cap > 4 * t) t *= 2;
  plan->threads = t;
  const int need = int((group_cap + t - 1) / t);
  plan->items = need <= 2 ? 2 : need <= 4 ? 4 : need <= 6 ? 6 : need <= 8 ? 8 : 12;
  int slots = 1024;
  while (slots < 2 * group_cap && slots < 16384) slots <<= 1;
  while (slots < 4 * t) slots <<= 1;  // the kernel clears whole 16-byte rows of the workgroup
  plan->table_slots = slots;  // > group_cap: 12 288 < 16 384
  plan->dict_lds = size_t(slots) * 4;
  plan->words = (R + 2) / 2;
  const size_t per_order = size_t(cand_stride) * plan->words * 4;
  if (per_order > kHierLdsPerWorkgroup) return false;
  plan->count_pairs_fit = 2 * per_order <= kHierLdsPerWorkgroup / 2;
  // count/clip: 16-byte id requests, ROWS per thread and order; measured best with small
  // workgroups that take four to six requests per thread
  plan->count_threads = 1024;
  for (int nt = 128; nt <= 1024; nt *= 2) {
    const int rows = rows_for(group_cap, nt);
    if (rows >= 1) {
      plan->count_threads = nt;
      plan->count_rows = rows;
      break;
    }
  }
  return true;
}

hipError_t launch_hier_dictionary(const Problem& pb, const GlobalWs& ws, const HierPlan& plan,
                                  const StatPtrs& st, int32_t* cand_distinct, hipStream_t s) {
  HierDictArgs a;
  a.pb = pb;
  a.ws = ws;
  a.distinct = st.distinct;
  a.cand_distinct = cand_distinct;
  a.table_slots = plan.table_slots;
  a.table_shift = 32 - ceil_log2_int(plan.table_slots);
  HierPlan shape = plan;
  auto items_for = [&](int t) {
    const int need = int((pb.group_cap + t - 1) / t);
    return need <= 2 ? 2 : need <= 4 ? 4 : need <= 6 ? 6 : need <= 8 ? 8 : need <= 12 ? 12 : 0;
  };
  // A batch of many rounds of workgroups runs best on small workgroups with up to eight
  // positions per thread (the per-wavefront work of every phase is shared by more n-grams);
  // otherwise the plan's wider workgroups finish a group sooner.
  if (pb.B >= 2048) {
    for (int t = 256; t < plan.threads; t *= 2) {
      const int items = items_for(t);
      if (items >= 2 && items <= 8 && plan.table_slots % (4 * t) == 0) {
        shape.threads = t;
        shape.items = items;
        break;
      }
    }
  }
#ifdef TB_STAMPS
  if (const char* e = getenv("TB_DICT_THREADS")) {  // tuning builds
    const int t = atoi(e);
    if ((t == 256 || t == 512 || t == 1024) && items_for(t) && plan.table_slots % (4 * t) == 0) {
      shape.threads = t;
      shape.items = items_for(t);
    }
  }
#endif
  switch (shape.items) {
    case 2: return launch_dict_items<2>(a, shape, s);
    case 4: return launch_dict_items<4>(a, shape, s);
    case 6: return launch_dict_items<6>(a, shape, s);
    case 8: return launch_dict_items<8>(a, shape, s);
    case 12: return launch_dict_items<12>(a, shape, s);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_hier_count_clip(const Problem& pb, const GlobalWs& ws, const HierPlan& plan,
                                  const StatPtrs& st, const int32_t* cand_distinct,
                                  hipStream_t s, int32_t* rouge_overlap, const ScoreTail* tail) {
  HierCountArgs a;
  a.pb = pb;
  a.ws = ws;
  a.st = st;
  a.score_out = nullptr;
  if (tail && !rouge_overlap) {
    if (!ws.arrivals) return hipErrorInvalidValue;
    a.sp = tail->sp;
    a.score_out = tail->out;
  } else {
    a.sp = ScoreParams{};
  }
  a.cand_distinct = cand_distinct;
  a.words = plan.words;
  a.order_words = int(pb.cand_stride) * plan.words;
  const CountShape shape = count_shape(pb, plan);
  a.rouge_overlap = rouge_overlap;
  if (rouge_overlap) {  // order N only
    a.split = 1;
    return launch_count_rows(a, shape.threads, shape.rows, 1, s);
  }
  a.split = (pb.N + shape.opw - 1) / shape.opw;
  return launch_count_rows(a, shape.threads, shape.rows, shape.opw, s);
}

}  // namespace tb
