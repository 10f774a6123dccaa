// GLOBAL path for sentence groups of 12 289 .. 2 097 152 n-gram slots: too many for one LDS hash
// table, few enough that the table can be split.  The dictionary and count/clip passes
// (paper Sections 3.2-3.3) run with P workgroups per (group, order); workgroup p owns the
// n-grams whose key hashes into partition p and keeps its share of the dictionary (or of the
// counters) in LDS, where random access is cheap -- the same kernels with the table in HBM are
// several times slower per n-gram.  A scatter kernel first sorts each (group, order)'s slots by
// partition (one workgroup each: histogram, prefix sums, scatter), so every key is hashed once
// and the P workgroups read only their own members.
//
// Ids: partition p numbers its distinct n-grams 0, 1, ... and publishes them as p * id_cap + local,
// so ids stay unique inside the group without any exchange between workgroups; they are no
// longer dense, and the group's id range grows to id_stride = max(group_cap, P * id_cap).
// Keys are spread over the partitions by a multiplicative hash; a partition that receives more
// than id_cap distinct keys (possible only for keys built to collide) is reported through
// TB_DEV_TABLE_OVERFLOW instead of being scored wrongly in silence.
//
// Orders whose packed n-grams need 16 bytes get an 8-byte key of their own here: (id of the
// (n-1)-gram that starts at the same position, last token).  Two n-grams are equal exactly when
// their (n-1)-gram prefixes are equal -- i.e. have the same id -- and their last tokens are equal,
// so this key identifies the n-gram as exactly as the packed one does; it needs the dictionary of
// order n - 1 to be complete, hence one launch per such order after the others.
#include <type_traits>

#include "tb_group_index.h"
#include "tb_kernels.h"

// Phase time stamps for tuning builds only (-DTB_STAMPS), as in the hierarchical kernels.
#ifdef TB_STAMPS
__device__ unsigned long long tb_part_stamps[8192 * 16];
#define TB_PSTAMP(i) \
  do { if (threadIdx.x == 0 && blockIdx.x < 8192) tb_part_stamps[blockIdx.x * 16 + (i)] = wall_clock64(); } while (0)
extern "C" int tb_debug_stamps_part(unsigned long long* host, int count) {
  return int(hipMemcpyFromSymbol(host, HIP_SYMBOL(tb_part_stamps), size_t(count) * 8));
}
#else
#define TB_PSTAMP(i) do {} while (0)
#endif

namespace tb {

namespace {

constexpr int kPartThreads = 1024;
constexpr int kPartSlots = 8192;     // 8-byte table entries: 64 KB of LDS
constexpr int kPartIdCap = 6144;     // distinct n-grams a partition may hold (3/4 of its slots)
constexpr int kPartTarget = 4096;    // P is chosen so that a partition expects at most this many slots
constexpr int kPartUnroll = 8;       // loads in flight per thread
constexpr int kMaxParts = 512;       // partitions per (group, order): groups of up to 2 097 152 slots
constexpr int kScatterChunk = 16384; // slots per workgroup of the chunked scatter
constexpr unsigned long long kFreeEntry = ~0ull;

struct PartArgs {
  Problem pb;
  GlobalWs ws;
  StatPtrs st;
  int32_t* part_distinct;  // [B, N, P] distinct n-grams per partition (dictionary -> count/clip)
  int32_t* part_start;     // [B, N, P + 1] where each partition's members start in member_slot
  uint32_t* member_slot;   // [N][B * group_cap] the slots of a (group, order), grouped by partition
  uint64_t* member_key;    // [N][B * group_cap] their 8-byte keys, in the same order
  uint32_t* member_id;     // [N][B * group_cap] their ids within the partition, same order
  int32_t* chunk_hist;     // [B, N, chunks, P] chunked scatter: per-chunk partition histograms
  int xcd_aware;           // block -> (group, order, partition): see role_of_block
  int with_count;          // the dictionary kernel also counts and clips its partition
  int ids_wanted;          // bit n: order n's ids must reach the id array (ws.inv)
  int refs_per_pass;       // count kernel: 0, or references per pass when they do not fit LDS
  int log2_parts;          // P = 1 << log2_parts, P >= 2
  int orders[8];           // dictionary: the orders of this launch, and how many
  int num_orders;
  int derived;             // dictionary: 1 if this launch's orders use (prefix id, last token) keys
  int from_tokens;         // dictionary: keys are built from the token rows (whole calls)
  int words;               // count/clip: 32-bit counter words per id
  int fields_per_word;     // 2: 16-bit counters (sequences of at most 65 535 tokens); 1: 32-bit
  int64_t id_stride;       // ids of group g lie in [g * id_stride, (g + 1) * id_stride)
  int32_t* rouge_overlap;  // count kernel, ROUGE-N: [B, R] sums of min(candidate count, reference
                           // j's count), zeroed by the launcher and added to per partition; or null
};

__device__ __forceinline__ uint32_t part_hash(uint64_t key) {
  const uint32_t lo = uint32_t(key), hi = uint32_t(key >> 32);
  return (lo ^ ((hi << 15) | (hi >> 17))) * 0x9E3779B1u;
}
// Partition of a key: the top bits of a second product, independent of the bits that pick the
// slot (top bits of h) and the probe step.
__device__ __forceinline__ int part_of(uint32_t h, int log2_parts) {
  return int((h * 0x85EBCA6Bu + 0x27D4EB2Fu) >> (32 - log2_parts));
}

// Workgroup -> (group, order, partition).  Workgroups are handed to the eight XCDs in turn
// (workgroup i runs on XCD i mod 8) and each XCD has its own L2, so the P workgroups of one
// (group, order) are given indices that are equal mod 8: the keys, member lists and ids they
// share then stay in that XCD's L2.  g < 0: no work (the grid is rounded up).
constexpr int kXcds = 8;
struct Role {
  int g, n, p;
};
// `orders` / `num_orders`: the orders this launch handles (null: all of 1..N).
__device__ __forceinline__ Role role_of_block(const PartArgs& a, const int* orders,
                                              int num_orders) {
  const int parts = 1 << a.log2_parts;
  const int xcd = a.xcd_aware ? int(blockIdx.x) % kXcds : 0;
  const int j = a.xcd_aware ? int(blockIdx.x) / kXcds : int(blockIdx.x);
  Role r;
  r.p = j & (parts - 1);
  // (32-bit: the grid, at least P times the number of pairs, fits an int)
  const uint32_t gn = uint32_t(j >> a.log2_parts) * uint32_t(a.xcd_aware ? kXcds : 1) + xcd;
  const uint32_t group = gn / uint32_t(num_orders);
  r.g = int64_t(gn) < int64_t(a.pb.B) * num_orders ? int(group) : -1;
  const int idx = int(gn - group * uint32_t(num_orders));
  r.n = orders ? orders[idx] : idx + 1;
  return r;
}
// Few (group, order)s: blocks in plain order, so that their partitions spread over all XCDs.
__host__ inline bool part_xcd_aware(const Problem& pb, int num_orders) {
  return int64_t(pb.B) * num_orders >= 8 * kXcds;
}
__host__ inline int64_t part_grid(const Problem& pb, const PartPlan& plan, int num_orders) {
  const int64_t gn = int64_t(pb.B) * num_orders;
  if (!part_xcd_aware(pb, num_orders)) return gn << plan.log2_parts;
  return (((gn + kXcds - 1) / kXcds * kXcds)) << plan.log2_parts;
}

__global__ __launch_bounds__(256) void zero_ints_kernel(int32_t* p, int64_t count) {
  const int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
  if (i < count) p[i] = 0;
}

// The 8-byte key of slot k of one (group, order): the n tokens packed `bits` apiece, or for an
// order whose packed n-grams would need 16 bytes (id of the (n-1)-gram at the same position, last
// token).  A whole call builds the keys from the token rows themselves (the n-gram extraction of
// Section 3.1 happens here, and the pack kernel does not run); the staged dictionary entry point
// is not given the tokens and reads the pack kernel's arrays.  Construct and call in wave-uniform
// control flow with all 64 lanes active; within a call the lanes' slots must not decrease with
// the lane number (consecutive slots, possibly clamped to the last one).
struct KeySource {
  const uint64_t* narrow_keys;  // the pack kernel's arrays (used unless from_tokens)
  const Key128* wide_keys;
  int from_tokens;
  const void* cand;  // token rows
  const void* refs;
  int64_t cand_first;  // element index of the candidate's first token
  int64_t ref_first;   // element index of the first token of the group's reference 0
  int64_t ref_stride;
  const uint32_t* prev_inv;
  uint32_t prev_base;
  uint32_t vocab;
  int32_t* status;
  int bits, R, derived, n, tok64;
  int end_lane;    // lane j: end of sequence j among the order's slots
  int shift_lane;  // lane j: how far sequence j's slots of order n - 1 lie behind those of order n
  int count;       // n-grams of this (group, order)
  mutable int bad; // a token outside the vocabulary was met (checked on the order-1 keys)

  __device__ __forceinline__ KeySource(const PartArgs& a, int g, int order) {
    const Problem& pb = a.pb;
    GroupIndex gi(pb, g, GroupIndex::WaveOnly{});
    derived = a.derived;
    n = order;
    shift_lane = 0;
    if (derived) {
      gi.set_order(n - 1);
      shift_lane = gi.end_in_lane();
    }
    gi.set_order(n);
    end_lane = gi.end_in_lane();
    {
      const int d = shift_lane - end_lane;  // lane j: start_{n-1}(j + 1) - start_n(j + 1)
      shift_lane = __shfl_up(d, 1, kWave);
      if ((threadIdx.x & (kWave - 1)) == 0) shift_lane = 0;
    }
    count = int(min(int64_t(gi.start(pb.R + 1)), pb.group_cap));
    from_tokens = a.from_tokens;
    narrow_keys = reinterpret_cast<const uint64_t*>(a.ws.keys[n - 1]) + int64_t(g) * pb.group_cap;
    wide_keys = reinterpret_cast<const Key128*>(a.ws.keys[n - 1]) + int64_t(g) * pb.group_cap;
    cand = pb.cand;
    refs = pb.refs;
    cand_first = int64_t(g) * pb.cand_stride;
    ref_stride = pb.ref_stride;
    ref_first = ref_rows(pb, g).row0 * pb.ref_stride;
    prev_inv = a.ws.inv[max(n - 2, 0)] + int64_t(g) * pb.group_cap;
    prev_base = uint32_t(int64_t(g) * a.id_stride);
    vocab = uint32_t(pb.vocab);
    status = pb.status;
    bits = pb.bits;
    R = pb.R;
    tok64 = pb.tok64;
    bad = 0;
  }

  // Calls f(T, W) with T = integral constant, the tokens a key is built from (1..8; 0: the key
  // is read from the pack kernel's arrays), and W = whether token ids are 64-bit: the loads of
  // get<T, W> then carry no branches, so a caller's batch of them is in flight together.
  template <typename F>
  __device__ __forceinline__ void dispatch(F&& f) const {
    if (!from_tokens) {
      f(std::integral_constant<int, 0>{}, std::false_type{});
      return;
    }
    const int t = derived ? 1 : n;
    if (tok64) {
      switch (t) {
        case 1: f(std::integral_constant<int, 1>{}, std::true_type{}); break;
        case 2: f(std::integral_constant<int, 2>{}, std::true_type{}); break;
        case 3: f(std::integral_constant<int, 3>{}, std::true_type{}); break;
        case 4: f(std::integral_constant<int, 4>{}, std::true_type{}); break;
        case 5: f(std::integral_constant<int, 5>{}, std::true_type{}); break;
        case 6: f(std::integral_constant<int, 6>{}, std::true_type{}); break;
        case 7: f(std::integral_constant<int, 7>{}, std::true_type{}); break;
        default: f(std::integral_constant<int, 8>{}, std::true_type{}); break;
      }
    } else {
      switch (t) {
        case 1: f(std::integral_constant<int, 1>{}, std::false_type{}); break;
        case 2: f(std::integral_constant<int, 2>{}, std::false_type{}); break;
        case 3: f(std::integral_constant<int, 3>{}, std::false_type{}); break;
        case 4: f(std::integral_constant<int, 4>{}, std::false_type{}); break;
        case 5: f(std::integral_constant<int, 5>{}, std::false_type{}); break;
        case 6: f(std::integral_constant<int, 6>{}, std::false_type{}); break;
        case 7: f(std::integral_constant<int, 7>{}, std::false_type{}); break;
        default: f(std::integral_constant<int, 8>{}, std::false_type{}); break;
      }
    }
  }

  // 0 <= k < count.  T, W: as handed out by dispatch().
  template <int T, bool W>
  __device__ __forceinline__ uint64_t get(int k) const {
    if (T == 0 && !derived) return narrow_keys[k];
    // the sequence slot k belongs to: usually the same for the whole wavefront, found by one
    // ballot over the sequence ends (row address and offsets then stay in scalar registers); a
    // wavefront that straddles sequences walks the ends inside
    const int lane = threadIdx.x & (kWave - 1);
    const int k_lo = __builtin_amdgcn_readfirstlane(k);
    const int k_hi = __builtin_amdgcn_readlane(k, kWave - 1);
    const int ends = lane <= R ? end_lane : 0x7FFFFFFF;
    const int f0 = min(int(__popcll(__builtin_amdgcn_ballot_w64(ends <= k_lo))), R);
    constexpr int kLoads = T == 0 ? 1 : T;
    uint32_t tok[kLoads];
    int shift;
    // tokens [from, from + T) of the n-gram (derived keys: its last token only)
    const int from = derived ? n - 1 : 0;
    if (k_hi < __builtin_amdgcn_readlane(end_lane, f0)) {  // uniform
      const int start = f0 > 0 ? __builtin_amdgcn_readlane(end_lane, max(f0 - 1, 0)) : 0;
      const void* base = f0 == 0 ? cand : refs;
      const int64_t row = f0 == 0 ? cand_first : ref_first + int64_t(f0 - 1) * ref_stride;
      shift = __builtin_amdgcn_readlane(shift_lane, f0);
      if (T != 0) {
#pragma unroll
        for (int i = 0; i < kLoads; ++i)
          tok[i] = uint32_t(load_token(base, row + (from - start + i) + k, W));
      }
    } else {
      const int f_hi = min(int(__popcll(__builtin_amdgcn_ballot_w64(ends <= k_hi))), R);
      int seq = f0;
      int start = f0 > 0 ? __builtin_amdgcn_readlane(end_lane, max(f0 - 1, 0)) : 0;
      shift = __builtin_amdgcn_readlane(shift_lane, f0);
      for (int q = f0; q < f_hi; ++q) {
        const int e = __builtin_amdgcn_readlane(end_lane, q);
        const bool ge = k >= e;
        seq = ge ? q + 1 : seq;
        start = ge ? e : start;
        shift = ge ? __builtin_amdgcn_readlane(shift_lane, q + 1) : shift;
      }
      const void* base = seq == 0 ? cand : refs;
      const int64_t first =
          (seq == 0 ? cand_first : ref_first + int64_t(seq - 1) * ref_stride) + (k - start);
      if (T != 0) {
#pragma unroll
        for (int i = 0; i < kLoads; ++i) tok[i] = uint32_t(load_token(base, first + from + i, W));
      }
    }
    if (derived) {
      const uint64_t last =
          T == 0 ? (wide_keys[k].lo & ((uint64_t(1) << bits) - 1u)) : uint64_t(tok[0]);
      const uint64_t prefix = prev_inv[k + shift] - prev_base;
      return (prefix << bits) | last;
    }
    uint64_t key = 0;
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
      if (T == 1) bad |= int(tok[i] >= vocab);
      key = (key << bits) | tok[i];
    }
    return key;
  }

  // Once per thread, after its last get(): reports a token outside the vocabulary.
  __device__ __forceinline__ void report() const {
    if (bad && status) atomicOr(status, TB_DEV_TOKEN_RANGE);
  }
};

__device__ __forceinline__ int partition_of_key(uint64_t key, int log2_parts) {
  // the all-ones key (the table's empty marker) lives in partition 0
  return key == kFreeEntry ? 0 : part_of(part_hash(key), log2_parts);
}

// Writes the slots [begin, end) of one (group, order), with their keys, behind the partitions'
// cursors (LDS, one per partition; advanced here).  The slots go through LDS in rounds of 4096,
// sorted by partition there, so that each partition's share of a round is one contiguous run of
// stores rather than one store per cache line.  Call from all threads of the workgroup.
constexpr int kRound = 4096, kRoundUnroll = kRound / kPartThreads;
struct ScatterLds {
  uint64_t key[kRound];
  uint32_t slot[kRound];  // slot number (below 2^22) | partition << 22
  int count[kMaxParts];   // of the round, per partition; zero between rounds
  int first[kMaxParts];   // where the partition's run starts in the round's sorted order
  int shift[kMaxParts];   // sorted position + shift = position in the partition's segment
  int scan_scratch[17];
};
__device__ __forceinline__ void scatter_range(const PartArgs& a, const KeySource& key_of,
                                              int begin, int end, int* cursor, ScatterLds& lds,
                                              uint32_t* members, uint64_t* member_keys) {
  const int nt = blockDim.x, tid = threadIdx.x;
  const int parts = 1 << a.log2_parts;
  const int last = max(key_of.count - 1, 0);
  if (tid < kMaxParts) lds.count[tid] = 0;
  __syncthreads();
  for (int base = begin; base < end; base += kRound) {
    uint64_t key[kRoundUnroll];
    int where[kRoundUnroll];  // rank within the partition's run | partition << 16
    key_of.dispatch([&](auto T, auto W) {
#pragma unroll
      for (int u = 0; u < kRoundUnroll; ++u)
        key[u] = key_of.template get<T(), W()>(min(base + u * nt + tid, end - 1));
    });
#pragma unroll
    for (int u = 0; u < kRoundUnroll; ++u) {
      const int q = partition_of_key(key[u], a.log2_parts);
      where[u] = q << 16;
      if (base + u * nt + tid < end) where[u] |= atomicAdd(&lds.count[q], 1);
    }
    __syncthreads();
    int total = 0;
    const int mine = tid < parts ? lds.count[tid] : 0;
    const int run = block_exclusive_scan(mine, lds.scan_scratch, &total);
    if (tid < parts) {
      lds.first[tid] = run;
      lds.shift[tid] = cursor[tid] - run;
      cursor[tid] += mine;
      lds.count[tid] = 0;
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kRoundUnroll; ++u) {
      const int k = base + u * nt + tid;
      if (k < end) {
        const int q = where[u] >> 16;
        const int pos = min(lds.first[q] + (where[u] & 0xFFFF), kRound - 1);
        lds.key[pos] = key[u];
        lds.slot[pos] = uint32_t(k) | (uint32_t(q) << 22);
      }
    }
    __syncthreads();
    const int in_round = min(kRound, end - base);
    for (int i = tid; i < in_round; i += nt) {
      const uint32_t v = lds.slot[i];
      const int at = min(max(lds.shift[v >> 22] + i, 0), last);  // (clamped: see the callers)
      members[at] = v & 0x3FFFFFu;
      member_keys[at] = lds.key[i];
    }
    __syncthreads();
  }
}

// One workgroup per (group, order) of the launch sorts the order's slots by partition: a
// histogram over the keys' partitions, its prefix sums (published as part_start), then every slot
// is written to its partition's segment of member_slot.  Each key is hashed here and nowhere
// else; the P dictionary workgroups read only their own members.
__global__ __launch_bounds__(kPartThreads) void part_scatter_kernel(PartArgs a) {
  __shared__ int hist[kMaxParts], cursor[kMaxParts];
  const Problem& pb = a.pb;
  const int nt = blockDim.x, tid = threadIdx.x;
  const int g = int(blockIdx.x) / a.num_orders, n = a.orders[int(blockIdx.x) % a.num_orders];
  const int parts = 1 << a.log2_parts;
  const KeySource key_of(a, g, n);
  const int count = key_of.count;
  uint32_t* members = a.member_slot + (int64_t(n - 1) * pb.B + g) * pb.group_cap;
  uint64_t* member_keys = a.member_key + (int64_t(n - 1) * pb.B + g) * pb.group_cap;
  int32_t* start = a.part_start + (int64_t(g) * pb.N + n - 1) * (parts + 1);
  if (tid < kMaxParts) hist[tid] = 0;
  if (a.with_count && tid == 0) {  // the dictionary workgroups of this (group, order) add into these
    a.st.clipped[int64_t(g) * pb.N + n - 1] = 0;
    a.st.distinct[int64_t(g) * pb.N + n - 1] = 0;
  }
  // (order 1 is in the first launch of a call; the dictionary workgroups raise the flag later)
  if (n == 1 && tid == 0 && a.ws.overflow) a.ws.overflow[g] = 0;
  __syncthreads();
  for (int base = 0; base < count; base += kPartUnroll * nt) {
    uint64_t key[kPartUnroll];
    key_of.dispatch([&](auto T, auto W) {
#pragma unroll
      for (int u = 0; u < kPartUnroll; ++u)
        key[u] = key_of.template get<T(), W()>(min(base + u * nt + tid, count - 1));
    });
#pragma unroll
    for (int u = 0; u < kPartUnroll; ++u)
      if (base + u * nt + tid < count) atomicAdd(&hist[partition_of_key(key[u], a.log2_parts)], 1);
  }
  __syncthreads();
  if (tid == 0) {
    int run = 0;
    for (int q = 0; q < parts; ++q) {
      cursor[q] = run;
      start[q] = run;
      run += hist[q];
    }
    start[parts] = run;
  }
  __syncthreads();
  // (a partition's share of a wave's stores is a run of neighbouring addresses already)
  for (int base = 0; base < count; base += kPartUnroll * nt) {
    uint64_t key[kPartUnroll];
    key_of.dispatch([&](auto T, auto W) {
#pragma unroll
      for (int u = 0; u < kPartUnroll; ++u)
        key[u] = key_of.template get<T(), W()>(min(base + u * nt + tid, count - 1));
    });
#pragma unroll
    for (int u = 0; u < kPartUnroll; ++u) {
      const int k = base + u * nt + tid;
      if (k < count) {
        const int at = atomicAdd(&cursor[partition_of_key(key[u], a.log2_parts)], 1);
        members[at] = uint32_t(k);
        member_keys[at] = key[u];
      }
    }
  }
  key_of.report();
}

// The same for groups of at most 16 384 slots: every thread keeps its 16 keys in registers
// between the histogram and the scatter, so the keys are read once.
constexpr int kScatterRegItems = 16;
__global__ __launch_bounds__(kPartThreads, 8) void part_scatter_small_kernel(PartArgs a) {
  __shared__ int hist[kMaxParts], cursor[kMaxParts];
  const Problem& pb = a.pb;
  const int nt = blockDim.x, tid = threadIdx.x;
  const int g = int(blockIdx.x) / a.num_orders, n = a.orders[int(blockIdx.x) % a.num_orders];
  const int parts = 1 << a.log2_parts;
  const KeySource key_of(a, g, n);
  const int count = min(key_of.count, kScatterRegItems * nt);
  uint32_t* members = a.member_slot + (int64_t(n - 1) * pb.B + g) * pb.group_cap;
  uint64_t* member_keys = a.member_key + (int64_t(n - 1) * pb.B + g) * pb.group_cap;
  int32_t* start = a.part_start + (int64_t(g) * pb.N + n - 1) * (parts + 1);
  if (tid < kMaxParts) hist[tid] = 0;
  if (a.with_count && tid == 0) {  // see part_scatter_kernel
    a.st.clipped[int64_t(g) * pb.N + n - 1] = 0;
    a.st.distinct[int64_t(g) * pb.N + n - 1] = 0;
  }
  if (n == 1 && tid == 0 && a.ws.overflow) a.ws.overflow[g] = 0;
  __syncthreads();
  uint64_t key[kScatterRegItems];
#pragma unroll
  for (int i = 0; i < kScatterRegItems; ++i) key[i] = 0;
  if (count > 0)
    key_of.dispatch([&](auto T, auto W) {
#pragma unroll
      for (int i = 0; i < kScatterRegItems; ++i)
        key[i] = key_of.template get<T(), W()>(min(i * nt + tid, count - 1));
    });
#pragma unroll
  for (int i = 0; i < kScatterRegItems; ++i)
    if (i * nt + tid < count) atomicAdd(&hist[partition_of_key(key[i], a.log2_parts)], 1);
  __syncthreads();
  if (tid == 0) {
    int run = 0;
    for (int q = 0; q < parts; ++q) {
      cursor[q] = run;
      start[q] = run;
      run += hist[q];
    }
    start[parts] = run;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < kScatterRegItems; ++i) {
    const int k = i * nt + tid;
    if (k < count) {
      const int at = atomicAdd(&cursor[partition_of_key(key[i], a.log2_parts)], 1);
      members[at] = uint32_t(k);
      member_keys[at] = key[i];
    }
  }
  key_of.report();
}

// The same in two kernels with one workgroup per 16 384 slots, for batches of few, very long
// groups (one workgroup per (group, order) would leave most of the GPU idle): per-chunk
// histograms, then the scatter, in which every workgroup derives its own cursors (and chunk 0
// publishes part_start) from all the chunks' histograms of its (group, order).
__global__ __launch_bounds__(kPartThreads) void part_chunk_hist_kernel(PartArgs a, int chunks) {
  __shared__ int hist[kMaxParts];
  const Problem& pb = a.pb;
  const int nt = blockDim.x, tid = threadIdx.x;
  const int c = int(blockIdx.x) % chunks, gn = int(blockIdx.x) / chunks;
  const int g = gn / a.num_orders, n = a.orders[gn % a.num_orders];
  const int parts = 1 << a.log2_parts;
  const KeySource key_of(a, g, n);
  const int begin = min(c * kScatterChunk, key_of.count);
  const int end = min(begin + kScatterChunk, key_of.count);
  if (tid < kMaxParts) hist[tid] = 0;
  __syncthreads();
  for (int base = begin; base < end; base += kPartUnroll * nt) {
    uint64_t key[kPartUnroll];
    key_of.dispatch([&](auto T, auto W) {
#pragma unroll
      for (int u = 0; u < kPartUnroll; ++u)
        key[u] = key_of.template get<T(), W()>(min(base + u * nt + tid, end - 1));
    });
#pragma unroll
    for (int u = 0; u < kPartUnroll; ++u)
      if (base + u * nt + tid < end) atomicAdd(&hist[partition_of_key(key[u], a.log2_parts)], 1);
  }
  __syncthreads();
  int32_t* out = a.chunk_hist + ((int64_t(g) * pb.N + n - 1) * chunks + c) * parts;
  if (tid < parts) out[tid] = hist[tid];
  if (a.with_count && c == 0 && tid == 0) {  // see part_scatter_kernel
    a.st.clipped[int64_t(g) * pb.N + n - 1] = 0;
    a.st.distinct[int64_t(g) * pb.N + n - 1] = 0;
  }
  if (n == 1 && c == 0 && tid == 0 && a.ws.overflow) a.ws.overflow[g] = 0;
  key_of.report();
}

__global__ __launch_bounds__(kPartThreads) void part_chunk_scatter_kernel(PartArgs a,
                                                                         int chunks) {
  __shared__ int total[kMaxParts], before[kMaxParts], cursor[kMaxParts];
  __shared__ int scan_scratch[17];
  __shared__ ScatterLds lds;
  const Problem& pb = a.pb;
  const int nt = blockDim.x, tid = threadIdx.x;
  const int c = int(blockIdx.x) % chunks, gn = int(blockIdx.x) / chunks;
  const int g = gn / a.num_orders, n = a.orders[gn % a.num_orders];
  const int parts = 1 << a.log2_parts;
  const KeySource key_of(a, g, n);
  const int begin = min(c * kScatterChunk, key_of.count);
  const int end = min(begin + kScatterChunk, key_of.count);
  uint32_t* members = a.member_slot + (int64_t(n - 1) * pb.B + g) * pb.group_cap;
  uint64_t* member_keys = a.member_key + (int64_t(n - 1) * pb.B + g) * pb.group_cap;
  const int32_t* h = a.chunk_hist + (int64_t(g) * pb.N + n - 1) * chunks * parts;
  int32_t* start = a.part_start + (int64_t(g) * pb.N + n - 1) * (parts + 1);

  // partition q's segment starts at the sum of the smaller partitions' sizes; within it this
  // chunk writes behind the chunks before it
  if (tid < kMaxParts) total[tid] = before[tid] = 0;
  __syncthreads();
  for (int i = tid; i < chunks * parts; i += nt) {
    const int v = h[i], q = i & (parts - 1);
    atomicAdd(&total[q], v);
    if ((i >> a.log2_parts) < c) atomicAdd(&before[q], v);
  }
  __syncthreads();
  int all = 0;
  const int first = block_exclusive_scan(tid < parts ? total[tid] : 0, scan_scratch, &all);
  if (tid < parts) {
    cursor[tid] = first + before[tid];
    if (c == 0) start[tid] = first;
  }
  if (c == 0 && tid == 0) start[parts] = all;
  __syncthreads();

  scatter_range(a, key_of, begin, end, cursor, lds, members, member_keys);
  key_of.report();
}

// Counts a partition's members into one counter field per (id, sequence) -- `cnt`, LDS, U * W
// words, zeroed here -- and clips: returns this thread's share of the sum over the ids of
// min(candidate count, largest reference count).  member_ids[i] is member i's (id within the
// partition | index of its sequence << 16); with kFirstRoundInRegs, first_round[u] holds it for
// member u * nt + tid.  With kSeqFromSlot the words hold only the id (bit 31 is ignored) and the
// sequence is found from the member's slot number (member_slot[i], clamped to last_slot;
// seq_end: lane j holds the end of sequence j).  Contains barriers: call from all threads,
// after everyone's last use of what `cnt` overlays.
template <bool kFirstRoundInRegs, bool kSeqFromSlot = false>
__device__ __forceinline__ int count_clip_partition(uint32_t* cnt, int U, int W,
                                                    int fields_per_word, int R, int members,
                                                    const uint32_t* member_ids,
                                                    const uint32_t (&first_round)[kPartUnroll],
                                                    const uint32_t* member_slot = nullptr,
                                                    uint32_t last_slot = 0, int seq_end = 0,
                                                    int* overlap = nullptr) {
  // overlap (LDS, R ints, or null): ROUGE-N -- the sweep also adds, per reference j, the sum over
  // the ids of min(candidate count, reference j's count)
  const int nt = blockDim.x, tid = threadIdx.x;
  {
    uint4* c4 = reinterpret_cast<uint4*>(cnt);
    const int quads = (U * W + 3) / 4;
    for (int q = tid; q < quads; q += nt) c4[q] = make_uint4(0u, 0u, 0u, 0u);
  }
  __syncthreads();
  TB_PSTAMP(4);
  // A crowded partition (see the dictionary kernel) holds thousands of occurrences of one
  // n-gram: there the lanes of a wavefront that hold the same (id, sequence) as its first lane
  // add up in one atomic instead of queueing at one LDS address.
  auto tally = [&](auto crowded) {
    constexpr bool kCrowded = decltype(crowded)::value;
    for (int base = 0; base < members; base += kPartUnroll * nt) {
      uint32_t id[kPartUnroll];
#pragma unroll
      for (int u = 0; u < kPartUnroll; ++u)
        id[u] = (kFirstRoundInRegs && base == 0)
                    ? first_round[u]
                    : member_ids[min(base + u * nt + tid, members - 1)];
      uint32_t k[kSeqFromSlot ? kPartUnroll : 1];
      if (kSeqFromSlot) {
#pragma unroll
        for (int u = 0; u < kPartUnroll; ++u)
          k[kSeqFromSlot ? u : 0] =
              min(member_slot[min(base + u * nt + tid, members - 1)], last_slot);
      }
#pragma unroll
      for (int u = 0; u < kPartUnroll; ++u) {
        int f = 0;
        if (kSeqFromSlot) {
          for (int j = 0; j < R; ++j)
            f += (int(k[kSeqFromSlot ? u : 0]) >= __builtin_amdgcn_readlane(seq_end, j)) ? 1 : 0;
        } else {
          f = min(int((id[u] >> 16) & 0x7FFFu), R);  // (bit 31 may hold a dictionary flag)
        }
        const uint32_t word = (id[u] & 0xFFFFu) | (uint32_t(f) << 16);
        id[u] &= 0xFFFFu;
        bool mine = base + u * nt + tid < members && id[u] < uint32_t(U);
        uint32_t times = 1;
        if (kCrowded) {
          const unsigned long long live = __ballot(mine);
          if (live) {  // uniform over the wavefront
            const int leader = __ffsll(live) - 1;
            const uint32_t first = uint32_t(__builtin_amdgcn_readlane(int(word), leader));
            const unsigned long long same = __ballot(mine && word == first);
            times = word == first ? uint32_t(__popcll(same)) : 1u;  // the leader adds for all
            mine = mine && (word != first || int(tid & (kWave - 1)) == leader);
          }
        }
        if (mine) {
          if (fields_per_word == 2)
            atomicAdd(&cnt[__umul24(id[u], uint32_t(W)) + uint32_t(f >> 1)],
                      (f & 1) ? (times << 16) : times);
          else
            atomicAdd(&cnt[__umul24(id[u], uint32_t(W)) + uint32_t(f)], times);
        }
      }
    }
  };
  if (members > 2 * kPartTarget)
    tally(std::true_type{});
  else
    tally(std::false_type{});
  TB_PSTAMP(5);
  __syncthreads();
  TB_PSTAMP(6);
  int part = 0;
  for (int u = tid; u < U; u += nt) {
    const uint32_t* e = &cnt[__umul24(uint32_t(u), uint32_t(W))];
    const uint32_t w0 = e[0];
    if (fields_per_word == 2) {
      uint32_t m = w0 >> 16;
      for (int q = 1; q < W; ++q) {
        const uint32_t w = e[q];
        m = max(m, max(w & 0xFFFFu, w >> 16));
      }
      part += int(min(w0 & 0xFFFFu, m));
      if (overlap) {  // uniform; field j + 1 is reference j
        for (int j = 0; j < R; ++j) {
          const uint32_t w = e[(j + 1) >> 1];
          const uint32_t both = min(w0 & 0xFFFFu, ((j + 1) & 1) ? (w >> 16) : (w & 0xFFFFu));
          if (both) atomicAdd(&overlap[j], int(both));
        }
      }
    } else {  // word 0: candidate, word 1 + j: reference j
      uint32_t m = 0;
      for (int q = 1; q < W; ++q) m = max(m, e[q]);
      part += int(min(w0, m));
      if (overlap) {
        for (int j = 0; j < R; ++j) {
          const uint32_t both = min(w0, e[1 + j]);
          if (both) atomicAdd(&overlap[j], int(both));
        }
      }
    }
  }
  return part;
}

// The same when one counter field per sequence does not fit LDS: the references are taken
// `refs_per_pass` at a time.  Per id, W = kPassWords words: the candidate's count and the largest
// reference count so far (two 16-bit halves of word 0, or words 0 and 1 with 32-bit counters),
// then the fields of the pass's references.  Every pass walks the members, keeps those of its
// references (and, in the first, the candidate's), folds the fields' maximum into the running one
// and clears them.
constexpr int kPassWords = 6;
__device__ __forceinline__ int count_clip_partition_in_passes(uint32_t* cnt, int U,
                                                              int fields_per_word, int R,
                                                              int refs_per_pass, int members,
                                                              const uint32_t* member_ids,
                                                              int* overlap = nullptr) {
  const int nt = blockDim.x, tid = threadIdx.x;
  constexpr int W = kPassWords;
  const int first_word = fields_per_word == 2 ? 1 : 2;  // of the pass's reference fields
  {
    uint4* c4 = reinterpret_cast<uint4*>(cnt);
    const int quads = (U * W + 3) / 4;
    for (int q = tid; q < quads; q += nt) c4[q] = make_uint4(0u, 0u, 0u, 0u);
  }
  __syncthreads();
  for (int pass_first = 0; pass_first < R; pass_first += refs_per_pass) {  // first reference
    for (int base = 0; base < members; base += kPartUnroll * nt) {
      uint32_t id[kPartUnroll];
#pragma unroll
      for (int u = 0; u < kPartUnroll; ++u)
        id[u] = member_ids[min(base + u * nt + tid, members - 1)];
#pragma unroll
      for (int u = 0; u < kPartUnroll; ++u) {
        const int f = min(int(id[u] >> 16), R);  // 0: candidate, 1 + j: reference j
        id[u] &= 0xFFFFu;
        if (base + u * nt + tid >= members || id[u] >= uint32_t(U)) continue;
        uint32_t* e = &cnt[id[u] * uint32_t(W)];
        const int r = f - 1 - pass_first;  // reference within the pass
        if (f == 0) {
          if (pass_first == 0) atomicAdd(&e[0], 1u);
        } else if (r >= 0 && r < refs_per_pass) {
          if (fields_per_word == 2)
            atomicAdd(&e[first_word + (r >> 1)], (r & 1) ? 0x10000u : 1u);
          else
            atomicAdd(&e[first_word + r], 1u);
        }
      }
    }
    __syncthreads();
    for (int u = tid; u < U; u += nt) {
      uint32_t* e = &cnt[uint32_t(u) * uint32_t(W)];
      if (overlap) {  // ROUGE-N: the pass's references against the candidate's count
        const uint32_t cc = fields_per_word == 2 ? (e[0] & 0xFFFFu) : e[0];
        for (int r = 0; r < refs_per_pass && pass_first + r < R; ++r) {
          const uint32_t w = fields_per_word == 2 ? e[first_word + (r >> 1)] : e[first_word + r];
          const uint32_t c = fields_per_word == 2 ? ((r & 1) ? (w >> 16) : (w & 0xFFFFu)) : w;
          const uint32_t both = min(cc, c);
          if (both) atomicAdd(&overlap[pass_first + r], int(both));
        }
      }
      uint32_t m = 0;
      for (int q = first_word; q < W; ++q) {
        const uint32_t w = e[q];
        m = fields_per_word == 2 ? max(m, max(w & 0xFFFFu, w >> 16)) : max(m, w);
        e[q] = 0;
      }
      if (fields_per_word == 2) {
        const uint32_t w0 = e[0];
        e[0] = (w0 & 0xFFFFu) | (max(w0 >> 16, m) << 16);
      } else {
        e[1] = max(e[1], m);
      }
    }
    __syncthreads();
  }
  int part = 0;
  for (int u = tid; u < U; u += nt) {
    const uint32_t* e = &cnt[uint32_t(u) * uint32_t(W)];
    part += fields_per_word == 2 ? int(min(e[0] & 0xFFFFu, e[0] >> 16)) : int(min(e[0], e[1]));
  }
  return part;
}

// Dictionary of one partition of one (group, order): its members' keys are inserted into the LDS
// table and each occurrence's table entry is remembered; the entries are then numbered by the
// threads that created them; a second walk over the members turns the remembered entries into
// ids.
__global__ __launch_bounds__(kPartThreads, 8) void part_dictionary_kernel(PartArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int scan_scratch[18];
  int* next_id = &scan_scratch[17];
  const Problem& pb = a.pb;
  const int nt = blockDim.x, tid = threadIdx.x, lane = tid & (kWave - 1);
  TB_PSTAMP(0);
  const Role me = role_of_block(a, a.orders, a.num_orders);
  if (me.g < 0) return;  // uniform over the workgroup
  const int g = me.g, n = me.n, p = me.p;
  const int parts = 1 << a.log2_parts;
  constexpr int T = kPartSlots;
  constexpr uint32_t mask = uint32_t(T) - 1u;
  constexpr int shift = 32 - 13;  // log2(kPartSlots) = 13
  static_assert((1 << 13) == kPartSlots, "table_shift");
  unsigned long long* table = reinterpret_cast<unsigned long long*>(smem);
  uint32_t* ginv = a.ws.inv[n - 1] + int64_t(g) * pb.group_cap;
  // where the partition's members are: written by the scatter kernel, a launch earlier, and the
  // same for the whole workgroup -- read through the scalar cache, next to the lengths' loads
  const int64_t start_at = (int64_t(g) * pb.N + n - 1) * (parts + 1) + p;
  const int start_p = uniform_load(a.part_start, start_at);
  const int start_next = uniform_load(a.part_start, start_at + 1);
  GroupIndex gi(pb, g, GroupIndex::WaveOnly{});
  // (bounded by the arrays' extent, not by the lengths: the members' addresses then do not wait
  // for the lengths, whose loads are in flight)
  const int cap = int(min(pb.group_cap, int64_t(0x7FFFFFFF)));
  const int first = min(max(start_p, 0), cap);
  const int members_fetched = min(max(start_next - first, 0), cap - first);
  const int64_t list = (int64_t(n - 1) * pb.B + g) * pb.group_cap + first;
  const uint32_t* member = a.member_slot + list;
  const uint64_t* member_keys = a.member_key + list;
  // in the end: id within the partition | sequence within the group << 16; meanwhile the table
  // entries of the members beyond the first 8192 (those of the first 8192 stay in registers)
  uint32_t* member_ids = a.member_id + list;
  uint32_t parked0[kPartUnroll];
#pragma unroll
  for (int u = 0; u < kPartUnroll; ++u) parked0[u] = 0;
  // A whole call that needs this order's ids nowhere (no later order is derived from them) and
  // counts here can count by table entry: no ids, no second look into the table.
  const bool by_entry = a.with_count && !((a.ids_wanted >> n) & 1);

  // The first 4096 members' keys (and, to count by entry, their slots) -- all of them in a
  // partition of the expected size -- are requested before the table is cleared, so that the
  // clearing runs while they are on their way; those of the next 4096 after it.
  constexpr int kHalf = kPartUnroll / 2;
  uint64_t key0[kHalf];
  uint32_t slot0[kHalf];
#pragma unroll
  for (int u = 0; u < kHalf; ++u) key0[u] = 0, slot0[u] = 0;
  if (members_fetched > 0) {  // uniform
#pragma unroll
    for (int u = 0; u < kHalf; ++u)
      key0[u] = member_keys[min(u * nt + tid, members_fetched - 1)];
    if (by_entry) {
#pragma unroll
      for (int u = 0; u < kHalf; ++u) slot0[u] = member[min(u * nt + tid, members_fetched - 1)];
    }
  }
  gi.set_order(n);
  const int count = int(min(int64_t(gi.start(pb.R + 1)), pb.group_cap));
  const int seq_end = (lane <= pb.R) ? gi.end_in_lane() : 0x7FFFFFFF;
  const int members = min(members_fetched, max(count - first, 0));
  const uint32_t last_slot = uint32_t(max(count - 1, 0));
  // the sequence of a slot (how many sequences end at or before it), in bits 16 and up
  auto sequence_bits = [&](uint32_t slot) {
    int f = 0;
    for (int j = 0; j < pb.R; ++j)
      f += (int(min(slot, last_slot)) >= __builtin_amdgcn_readlane(seq_end, j)) ? 1 : 0;
    return uint32_t(f) << 16;
  };

  {  // T + 1 entries (entry T belongs to the all-ones key), 16 bytes per store
    uint4* t4 = reinterpret_cast<uint4*>(table);
    for (int s = tid; s < T / 2; s += nt) t4[s] = make_uint4(~0u, ~0u, ~0u, ~0u);
    if (tid == 0) table[T] = kFreeEntry;
    if (tid == 0) *next_id = 0;
  }
  __syncthreads();
  TB_PSTAMP(1);
  // Far more members than a partition expects means that some n-gram occurs thousands of times
  // (a frequent token in a long text): its occurrences would queue up at one LDS address.
  const bool crowded = members > 2 * kPartTarget;
  bool lost = false;  // a probe sequence ran through the whole table
  int created = 0;    // table entries that this thread's compare-and-swaps created ...
  uint32_t created0 = 0;  // ... bit u: among them the one of member u * nt + tid
  // Half a round: the members base + (u0 + u) * nt + tid, u < 4.  A member's table entry is
  // remembered (in registers for the first round of 8192, in member_ids beyond); counting by
  // entry, its sequence rides along in bits 16 and up (found from the member's slot number).
  auto insert_half = [&](auto peek, int base, auto first_u, const uint64_t (&key)[kHalf],
                         const uint32_t (&slot)[kHalf]) {
    constexpr bool kPeek = decltype(peek)::value;
    constexpr int u0 = decltype(first_u)::value;
    {
  #pragma unroll
      for (int v = 0; v < kHalf; ++v) {
        const int u = u0 + v;
        if (base + u * nt + tid >= members) continue;
        const uint32_t seq = by_entry ? sequence_bits(slot[v]) : 0u;
        if (key[v] == kFreeEntry) {
          const uint32_t made = atomicCAS(&table[T], kFreeEntry, 0ull) == kFreeEntry ? 1u : 0u;
          created += int(made);
          if (base == 0) {
            parked0[u] = uint32_t(T) | seq;
            created0 |= made << u;
          } else {
            member_ids[base + u * nt + tid] = uint32_t(T) | seq | (made << 31);
          }
          continue;
        }
        const uint32_t h = part_hash(key[v]);
        const uint32_t step = (h >> 3) | 1u;
        uint32_t s = h >> shift;
        // crowded partition: a plain read answers for a key that is already there, and only an
        // empty entry is worth an atomic
        unsigned long long old = kPeek ? table[s] : kFreeEntry;
        if (old == kFreeEntry) old = atomicCAS(&table[s], kFreeEntry, key[v]);
        int rounds = 0;
        while (int(old != kFreeEntry) & int(old != key[v]) & int(rounds < T)) {
          s = (s + step) & mask;
          old = kPeek ? table[s] : kFreeEntry;
          if (old == kFreeEntry) old = atomicCAS(&table[s], kFreeEntry, key[v]);
          ++rounds;
        }
        lost |= (old != kFreeEntry && old != key[v]);
        const uint32_t made = old == kFreeEntry ? 1u : 0u;
        created += int(made);
        if (base == 0) {
          parked0[u] = s | seq;
          created0 |= made << u;
        } else {
          member_ids[base + u * nt + tid] = s | seq | (made << 31);
        }
      }
    }
  };
  // the members [base + u0 * nt, base + (u0 + 4) * nt), loaded here
  auto load_and_insert_half = [&](auto peek, int base, auto first_u) {
    constexpr int u0 = decltype(first_u)::value;
    if (base + u0 * nt >= members) return;  // uniform
    uint64_t key[kHalf];
    uint32_t slot[kHalf];
#pragma unroll
    for (int v = 0; v < kHalf; ++v)
      key[v] = member_keys[min(base + (u0 + v) * nt + tid, members - 1)];
#pragma unroll
    for (int v = 0; v < kHalf; ++v)
      slot[v] = by_entry ? member[min(base + (u0 + v) * nt + tid, members - 1)] : 0u;
    insert_half(peek, base, first_u, key, slot);
  };
  auto insert_members = [&](auto peek) {
    using First = std::integral_constant<int, 0>;
    using Second = std::integral_constant<int, kHalf>;
    insert_half(peek, 0, First{}, key0, slot0);
    load_and_insert_half(peek, 0, Second{});
    for (int base = kPartUnroll * nt; base < members; base += kPartUnroll * nt) {
      load_and_insert_half(peek, base, First{});
      load_and_insert_half(peek, base, Second{});
    }
  };
  if (crowded)
    insert_members(std::true_type{});
  else
    insert_members(std::false_type{});
  if (by_entry) {
    TB_PSTAMP(2);
    const int distinct = block_sum(created, scan_scratch);  // (its barriers end the insertions)
    TB_PSTAMP(3);
    if (lost || distinct > kPartIdCap) {
      if (pb.status) atomicOr(pb.status, TB_DEV_TABLE_OVERFLOW);
      if (a.ws.overflow) a.ws.overflow[g] = 1;
    }
    if (tid == 0)
      a.part_distinct[(int64_t(g) * pb.N + n - 1) * (int64_t(1) << a.log2_parts) + p] = distinct;
    // (the members' words hold their table entries and sequences)
    const int part = count_clip_partition<true>(reinterpret_cast<uint32_t*>(smem), T + 1,
                                                a.words, a.fields_per_word, pb.R, members,
                                                member_ids, parked0);
    TB_PSTAMP(7);
    const int clipped = block_sum(part, scan_scratch);
    TB_PSTAMP(8);
    if (tid == 0) {
      const int64_t stat = int64_t(g) * pb.N + n - 1;
      if (clipped) atomicAdd(&a.st.clipped[stat], clipped);
      if (distinct) atomicAdd(&a.st.distinct[stat], distinct);
      if (p == 0) a.st.total[stat] = gi.start(1);
    }
    return;
  }

  // number the entries (any numbering that is dense and unique will do): the thread whose
  // compare-and-swap created an entry names it, from a block of ids its wavefront reserves
  uint32_t next = reserve_ids(created, next_id);
  __syncthreads();  // nobody compares keys any more: entries may now hold ids
#pragma unroll
  for (int u = 0; u < kPartUnroll; ++u)
    if ((created0 >> u) & 1u) table[min(parked0[u], uint32_t(T))] = uint64_t(next++);
  for (int base = kPartUnroll * nt; base < members; base += kPartUnroll * nt) {
#pragma unroll
    for (int u = 0; u < kPartUnroll; ++u) {
      const int i = base + u * nt + tid;
      if (i < members) {
        const uint32_t w = member_ids[i];
        if (w >> 31) table[min(w & 0x7FFFFFFFu, uint32_t(T))] = uint64_t(next++);
      }
    }
  }
  __syncthreads();
  const int distinct = *next_id;
  if (lost || distinct > kPartIdCap) {
    if (pb.status) atomicOr(pb.status, TB_DEV_TABLE_OVERFLOW);
    if (a.ws.overflow) a.ws.overflow[g] = 1;
  }

  const uint32_t id_base =
      uint32_t(int64_t(g) * a.id_stride) + uint32_t(p) * uint32_t(kPartIdCap);
  // a whole call needs the id array only where the next order's keys are derived from it
  const bool publish_ids = (a.ids_wanted >> n) & 1;
  for (int base = 0; base < members; base += kPartUnroll * nt) {
    uint32_t k[kPartUnroll], parked[kPartUnroll];
#pragma unroll
    for (int u = 0; u < kPartUnroll; ++u)
      k[u] = min(member[min(base + u * nt + tid, members - 1)], last_slot);
#pragma unroll
    for (int u = 0; u < kPartUnroll; ++u)
      parked[u] = base == 0
                      ? parked0[u]
                      : (member_ids[min(base + u * nt + tid, members - 1)] & 0x7FFFFFFFu);
#pragma unroll
    for (int u = 0; u < kPartUnroll; ++u) {
      int f = 0;  // the sequence of a slot: how many sequences end at or before it
      for (int j = 0; j < pb.R; ++j)
        f += (int(k[u]) >= __builtin_amdgcn_readlane(seq_end, j)) ? 1 : 0;
      if (base + u * nt + tid < members) {
        const uint32_t id = uint32_t(table[min(parked[u], uint32_t(T))]);
        const uint32_t packed = id | (uint32_t(f) << 16);
        if (publish_ids) ginv[k[u]] = id_base + id;
        // (when this kernel counts, only the members beyond the first 8192 are read again)
        if (!a.with_count || base != 0) member_ids[base + u * nt + tid] = packed;
        if (base == 0) parked0[u] = packed;
      }
    }
  }
  if (tid == 0)
    a.part_distinct[(int64_t(g) * pb.N + n - 1) * (int64_t(1) << a.log2_parts) + p] = distinct;
  if (!a.with_count) return;  // (then the count pass also forms the group's dictionary size)

  // the count pass's work for this partition, in the table's memory (the host checked that the
  // counter fields fit); the scatter kernel zeroed the group's statistics
  __syncthreads();
  const int part = count_clip_partition<true>(
      reinterpret_cast<uint32_t*>(smem), min(distinct, kPartIdCap), a.words, a.fields_per_word,
      pb.R, members, member_ids, parked0);
  const int clipped = block_sum(part, scan_scratch);
  if (tid == 0) {
    const int64_t stat = int64_t(g) * pb.N + n - 1;
    if (clipped) atomicAdd(&a.st.clipped[stat], clipped);
    if (distinct) atomicAdd(&a.st.distinct[stat], distinct);
    if (p == 0) a.st.total[stat] = gi.start(1);
  }
}

// Count and clip the ids of one partition of one (group, order): one 16-bit LDS field per
// (id, sequence) as in the LDS count kernel, filled from the partition's members; then
// a sweep over the partition's entries takes the maximum over the reference fields and the
// minimum with the candidate field.
__global__ __launch_bounds__(kPartThreads) void part_count_kernel(PartArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int red_scratch[17];
  __shared__ int s_overlap[kWave];  // ROUGE-N: this partition's overlap with each reference
  const Problem& pb = a.pb;
  const int tid = threadIdx.x;
  const Role me = role_of_block(a, a.orders, a.num_orders);
  if (me.g < 0) return;  // uniform over the workgroup
  const int g = me.g, n = me.n, p = me.p;
  const int W = a.words;
  int* overlap = a.rouge_overlap ? s_overlap : nullptr;  // (at most 62 references here)
  if (tid < kWave) s_overlap[tid] = 0;  // (the counting routines start with a barrier)
  uint32_t* cnt = reinterpret_cast<uint32_t*>(smem);
  const int U = min(
      max(a.part_distinct[(int64_t(g) * pb.N + n - 1) * (int64_t(1) << a.log2_parts) + p], 0),
      kPartIdCap);
  GroupIndex gi(pb, g, GroupIndex::WaveOnly{});
  gi.set_order(n);
  const int count = int(min(int64_t(gi.start(pb.R + 1)), pb.group_cap));
  const int ccnt = gi.start(1);

  // the partition's members are exactly the n-grams whose ids lie in this partition's id range;
  // the dictionary pass left each one's id within the partition and its sequence's index
  const int parts = 1 << a.log2_parts;
  const int32_t* start = a.part_start + (int64_t(g) * pb.N + n - 1) * (parts + 1);
  const int first = min(max(start[p], 0), count);
  const int members = min(max(start[p + 1] - first, 0), count - first);
  const uint32_t* member_ids =
      a.member_id + (int64_t(n - 1) * pb.B + g) * pb.group_cap + first;
  const uint32_t none[kPartUnroll] = {};
  const int part =
      a.refs_per_pass
          ? count_clip_partition_in_passes(cnt, U, a.fields_per_word, pb.R, a.refs_per_pass,
                                           members, member_ids, overlap)
          : count_clip_partition<false>(cnt, U, W, a.fields_per_word, pb.R, members, member_ids,
                                        none, nullptr, 0, 0, overlap);
  const int clipped = block_sum(part, red_scratch);  // (two barriers: s_overlap is complete)
  if (overlap && tid < pb.R && s_overlap[tid])
    atomicAdd(&a.rouge_overlap[int64_t(g) * pb.R + tid], s_overlap[tid]);
  if (tid == 0) {
    if (clipped) atomicAdd(&a.st.clipped[int64_t(g) * pb.N + n - 1], clipped);
    if (p == 0) {
      a.st.total[int64_t(g) * pb.N + n - 1] = ccnt;
      const int32_t* sizes =
          a.part_distinct + (int64_t(g) * pb.N + n - 1) * (int64_t(1) << a.log2_parts);
      int group_distinct = 0;
      for (int q = 0; q < (1 << a.log2_parts); ++q) group_distinct += sizes[q];
      a.st.distinct[int64_t(g) * pb.N + n - 1] = group_distinct;
    }
  }
}

// The partitioned kernels' share of the workspace: int32 [B, N, P] dictionary sizes, int32
// [B, N, P + 1] segment starts, uint32 [N][B * group_cap] slots grouped by partition; each part
// rounded up to 256 bytes.
size_t round256(size_t x) { return (x + 255) & ~size_t(255); }
size_t sizes_bytes(int64_t B, int N, int log2_parts) {
  return round256(((size_t(B) * N) << log2_parts) * 4);
}
size_t starts_bytes(int64_t B, int N, int log2_parts) {
  return round256(size_t(B) * N * ((size_t(1) << log2_parts) + 1) * 4);
}

PartArgs make_args(const Problem& pb, const GlobalWs& ws, const PartPlan& plan,
                   const StatPtrs& st) {
  PartArgs a;
  a.pb = pb;
  a.ws = ws;
  a.st = st;
  unsigned char* base = static_cast<unsigned char*>(ws.tables);
  a.part_distinct = reinterpret_cast<int32_t*>(base);
  a.part_start = reinterpret_cast<int32_t*>(base + sizes_bytes(pb.B, pb.N, plan.log2_parts));
  a.member_slot = reinterpret_cast<uint32_t*>(base + sizes_bytes(pb.B, pb.N, plan.log2_parts) +
                                              starts_bytes(pb.B, pb.N, plan.log2_parts));
  const size_t slots4 = round256(size_t(pb.B) * size_t(pb.group_cap) * pb.N * 4);
  unsigned char* after_slots = reinterpret_cast<unsigned char*>(a.member_slot) + slots4;
  a.member_id = reinterpret_cast<uint32_t*>(after_slots);
  a.member_key = reinterpret_cast<uint64_t*>(after_slots + slots4);
  a.chunk_hist = reinterpret_cast<int32_t*>(after_slots + 3 * slots4);
  a.rouge_overlap = nullptr;
  a.xcd_aware = 1;
  a.with_count = 0;
  a.ids_wanted = ~0;
  a.log2_parts = plan.log2_parts;
  a.words = plan.words;
  a.fields_per_word = plan.fields_per_word;
  a.refs_per_pass = plan.refs_per_pass;
  a.id_stride = plan.id_stride;
  for (int k = 0; k < 8; ++k) a.orders[k] = 0;
  a.num_orders = 0;
  a.derived = 0;
  a.from_tokens = 0;
  return a;
}

hipError_t zero_ints(int32_t* p, int64_t count, hipStream_t s) {
  const int64_t blocks = (count + 255) / 256;
  if (blocks <= 0 || blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
  hipLaunchKernelGGL(zero_ints_kernel, dim3(uint32_t(blocks)), dim3(256), 0, s, p, count);
  return hipGetLastError();
}

}  // namespace

size_t part_workspace_bytes(int64_t B, int N, int64_t group_cap, const PartPlan& plan) {
  const size_t chunks = size_t((group_cap + kScatterChunk - 1) / kScatterChunk);
  return sizes_bytes(B, N, plan.log2_parts) + starts_bytes(B, N, plan.log2_parts) +
         4 * round256(size_t(B) * size_t(group_cap) * N * 4) +  // slots, ids, 8-byte keys
         round256(((size_t(B) * N * chunks) << plan.log2_parts) * 4);
}

bool plan_part(int64_t group_cap, int64_t cand_stride, int64_t ref_stride, int R, int N,
               const int32_t* key_bytes, PartPlan* plan) {
  (void)key_bytes;  // orders with 16-byte keys are keyed by (prefix id, last token) instead
  if (R >= kWave - 1) return false;
  int lg = 1;
  while ((int64_t(kPartTarget) << lg) < group_cap) ++lg;
  if ((1 << lg) > kMaxParts) return false;
  plan->log2_parts = lg;
  plan->id_cap = kPartIdCap;
  // 16-bit counters while no sequence can hold an n-gram more than 65 535 times
  plan->fields_per_word = (cand_stride > 65535 || ref_stride > 65535) ? 1 : 2;
  plan->words = plan->fields_per_word == 2 ? (R + 2) / 2 : R + 1;
  plan->refs_per_pass = 0;
  if (plan->words > kPassWords) {  // several passes over the references: see the count kernel
    plan->words = kPassWords;
    plan->refs_per_pass = plan->fields_per_word == 2 ? 2 * (kPassWords - 1) : kPassWords - 2;
  }
  plan->id_stride = group_cap;
  if ((int64_t(kPartIdCap) << lg) > plan->id_stride) plan->id_stride = int64_t(kPartIdCap) << lg;
  plan->dict_lds = size_t(kPartSlots + 2) * 8;
  plan->count_lds = (size_t(kPartIdCap) * plan->words * 4 + 15) & ~size_t(15);
  plan->count_in_dictionary = plan->count_lds <= size_t(kPartSlots) * 8 ? 1 : 0;
  return plan->count_lds + 256 <= size_t(kLdsBudget);
}

hipError_t launch_part_dictionary(const Problem& pb, const GlobalWs& ws, const PartPlan& plan,
                                  const StatPtrs& st, bool whole_call, bool from_tokens,
                                  hipStream_t s) {
  const bool with_count = whole_call && plan.count_in_dictionary;
  hipError_t e =
      grant_dynamic_lds(reinterpret_cast<const void*>(part_dictionary_kernel), plan.dict_lds);
  if (e != hipSuccess) return e;
  // one launch for the orders with 8-byte packed keys, then one per order with 16-byte keys in
  // ascending order (each is keyed by the ids of the order below it)
  PartArgs a = make_args(pb, ws, plan, st);
  a.with_count = with_count ? 1 : 0;
  a.from_tokens = from_tokens ? 1 : 0;
  if (whole_call) {  // nobody reads the id array afterwards, except the derived keys
    a.ids_wanted = 0;
    for (int n = 1; n < pb.N; ++n)
      if (ws.wide[n]) a.ids_wanted |= 1 << n;  // order n + 1 is keyed by order n's ids
  }
  for (int n = 1; n <= pb.N; ++n)
    if (!ws.wide[n - 1]) a.orders[a.num_orders++] = n;
  for (int next_wide = 1; next_wide <= pb.N + 1; ++next_wide) {
    if (a.num_orders) {
      a.xcd_aware = part_xcd_aware(pb, a.num_orders) ? 1 : 0;
      const int64_t blocks = part_grid(pb, plan, a.num_orders);
      if (blocks <= 0 || blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
      const int64_t pairs = int64_t(pb.B) * a.num_orders;  // (group, order)s of this launch
      const int chunks = int((pb.group_cap + kScatterChunk - 1) / kScatterChunk);
      if (chunks > 1 && pairs < 256) {  // few long groups: one workgroup per 16 384 slots
        hipLaunchKernelGGL(part_chunk_hist_kernel, dim3(uint32_t(pairs * chunks)),
                           dim3(kPartThreads), 0, s, a, chunks);
        hipLaunchKernelGGL(part_chunk_scatter_kernel, dim3(uint32_t(pairs * chunks)),
                           dim3(kPartThreads), 0, s, a, chunks);
      } else if (pb.group_cap <= int64_t(kScatterRegItems) * kPartThreads) {
        hipLaunchKernelGGL(part_scatter_small_kernel, dim3(uint32_t(pairs)), dim3(kPartThreads),
                           0, s, a);
      } else {
        hipLaunchKernelGGL(part_scatter_kernel, dim3(uint32_t(pairs)), dim3(kPartThreads), 0, s,
                           a);
      }
      e = hipGetLastError();
      if (e != hipSuccess) return e;
      hipLaunchKernelGGL(part_dictionary_kernel, dim3(uint32_t(blocks)), dim3(kPartThreads),
                         plan.dict_lds, s, a);
      e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
    a.num_orders = 0;
    a.derived = 1;
    while (next_wide <= pb.N && !ws.wide[next_wide - 1]) ++next_wide;
    if (next_wide <= pb.N) a.orders[a.num_orders++] = next_wide;
  }
  return hipSuccess;
}

hipError_t launch_part_count_clip(const Problem& pb, const GlobalWs& ws, const PartPlan& plan,
                                  const StatPtrs& st, hipStream_t s, int32_t* rouge_overlap) {
  PartArgs a = make_args(pb, ws, plan, st);
  // every order, or for ROUGE-N the highest one only
  a.num_orders = rouge_overlap ? 1 : pb.N;
  for (int k = 0; k < 8; ++k) a.orders[k] = rouge_overlap ? pb.N : k + 1;
  a.rouge_overlap = rouge_overlap;
  a.xcd_aware = part_xcd_aware(pb, a.num_orders) ? 1 : 0;
  const int64_t blocks = part_grid(pb, plan, a.num_orders);
  if (blocks <= 0 || blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
  hipError_t e = zero_ints(st.clipped, int64_t(pb.B) * pb.N, s);
  if (e != hipSuccess) return e;
  if (rouge_overlap && (e = zero_ints(rouge_overlap, int64_t(pb.B) * pb.R, s)) != hipSuccess)
    return e;
  e = grant_dynamic_lds(reinterpret_cast<const void*>(part_count_kernel), plan.count_lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(part_count_kernel, dim3(uint32_t(blocks)), dim3(kPartThreads),
                     plan.count_lds, s, a);
  return hipGetLastError();
}

}  // namespace tb
