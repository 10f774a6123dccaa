// GLOBAL path kernels: pack -> dictionary -> count/clip, with keys and inverse indices in HBM.
//
// Mapping to the paper (Sections 3.1-3.3):
//   pack_kernel        n-gram extraction and the flattened list of valid n-grams, stored as
//                      packed integer keys instead of (total_ngrams, n) token rows;
//   dictionary_*       the compact dictionary + inverse indices (the role of torch.unique with
//                      return_inverse), built per sentence group in an LDS hash table;
//   count_clip_kernel  offset ids -> counts (the batched bincount), maximum over references,
//                      minimum with the candidate counts, summed per sentence and order.
// Clipping never compares n-grams of different sentence groups, so each group (a candidate and
// its references) gets its own dictionary; the group's offset g*group_cap keeps id ranges
// disjoint exactly like the paper's i*num_unique offset, with an a-priori bound in place of the
// data-dependent num_unique so that no size ever travels back to the host.
//
// Key / id arrays are group-compact: group g owns slots [g*group_cap, (g+1)*group_cap) and its
// valid n-grams of one order are stored back to back (candidate first, then each reference), so
// the dictionary and count kernels read one contiguous range per workgroup.
#include "tb_group_index.h"
#include "tb_kernels.h"

namespace tb {

// ---------------------------------------------------------------------------------- pack

constexpr int kPackThreads = 256;
constexpr int kPackTile = 1024;  // n-gram start positions per workgroup

struct PackArgs {
  Problem pb;
  GlobalWs ws;
  int cand_chunks, ref_chunks;
};

__device__ __forceinline__ void store_key(void* base, int wide, int64_t slot, uint64_t lo,
                                          uint64_t hi) {
  if (wide) {
    Key128 k;
    k.lo = lo;
    k.hi = hi;
    reinterpret_cast<Key128*>(base)[slot] = k;
  } else {
    reinterpret_cast<uint64_t*>(base)[slot] = lo;
  }
}

__global__ __launch_bounds__(kPackThreads) void pack_kernel(PackArgs a) {
  __shared__ int32_t tok[kPackTile + 8];
  const Problem& pb = a.pb;
  const int per_group = a.cand_chunks + pb.R * a.ref_chunks;
  const int g = blockIdx.x / per_group;
  int rem = blockIdx.x % per_group;
  const void* rows;   // token array and first element of this sequence's row
  int64_t row;
  int len, chunk, j;
  if (rem < a.cand_chunks) {
    j = 0;
    chunk = rem;
    rows = pb.cand;
    row = int64_t(g) * pb.cand_stride;
    len = clamped_len(pb.cand_len[g], pb.cand_stride, pb.status);
  } else {
    rem -= a.cand_chunks;
    j = 1 + rem / a.ref_chunks;
    chunk = rem % a.ref_chunks;
    rows = pb.refs;
    const RefRows rr = ref_rows(pb, g);
    row = (rr.row0 + j - 1) * pb.ref_stride;
    len = j <= rr.used ? clamped_len(pb.ref_len[rr.row0 + j - 1], pb.ref_stride, pb.status)
                       : 0;  // reference not in use
  }
  const int p0 = chunk * kPackTile;
  if (p0 >= len) return;  // uniform over the workgroup
  // where this sequence's n-grams start inside the group's compact range, per order
  int base[8];
  {
    GroupIndex gi(pb, g);
#pragma unroll
    for (int n = 1; n <= 8; ++n) {
      base[n - 1] = 0;
      if (n <= pb.N) {
        gi.set_order(n);
        base[n - 1] = gi.start(j);
      }
    }
  }
  const int ntok = min(kPackTile + pb.N - 1, len - p0);
  bool bad = false;
  for (int i = threadIdx.x; i < ntok; i += kPackThreads) {
    const int32_t t = load_token(rows, row + p0 + i, pb.tok64);
    tok[i] = t;
    bad |= (uint32_t(t) >= uint32_t(pb.vocab));
  }
  if (bad && pb.status) atomicOr(pb.status, TB_DEV_TOKEN_RANGE);
  __syncthreads();
  const int bits = pb.bits;
  const int64_t gslot = int64_t(g) * pb.group_cap + p0;
#pragma unroll
  for (int k = 0; k < kPackTile / kPackThreads; ++k) {
    const int q = threadIdx.x + k * kPackThreads;
    if (q >= ntok) break;
    const int avail = ntok - q;  // tokens from this start that lie inside the row (capped)
    uint64_t lo = uint32_t(tok[q]), hi = 0;
    store_key(a.ws.keys[0], a.ws.wide[0], gslot + base[0] + q, lo, hi);
#pragma unroll
    for (int n = 2; n <= 8; ++n) {
      if (n > pb.N || n > avail) break;
      hi = (hi << bits) | (lo >> (64 - bits));
      lo = (lo << bits) | uint32_t(tok[q + n - 1]);
      store_key(a.ws.keys[n - 1], a.ws.wide[n - 1], gslot + base[n - 1] + q, lo, hi);
    }
  }
}

hipError_t launch_pack(const Problem& pb, const GlobalWs& ws, hipStream_t s) {
  PackArgs a;
  a.pb = pb;
  a.ws = ws;
  a.cand_chunks = int((pb.cand_stride + kPackTile - 1) / kPackTile);
  a.ref_chunks = int((pb.ref_stride + kPackTile - 1) / kPackTile);
  const int64_t blocks = int64_t(pb.B) * (a.cand_chunks + int64_t(pb.R) * a.ref_chunks);
  if (blocks <= 0 || blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
  hipLaunchKernelGGL(pack_kernel, dim3(uint32_t(blocks)), dim3(kPackThreads), 0, s, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------- dictionary

struct DictArgs {
  Problem pb;
  GlobalWs ws;
  int32_t* distinct;
  int table_slots;  // 8-byte entries (narrow) or 4-byte entries (wide); power of two
  int table_shift;  // 32 - log2(table_slots)
  uint32_t lds_table_off;
  int slot32_mask;  // bit n: the keys of order n fit 32 bits
  int orders[16];  // wide kernel: its orders; narrow kernel: pairs (orders[2p], orders[2p + 1])
  int num_orders;  // wide kernel
  int num_pairs;   // narrow kernel: workgroups per group
};

bool plan_dictionary(int64_t group_cap, const int32_t* key_bytes, int N, int bits,
                     DictPlan* plan) {
  if (group_cap < 1 || group_cap > 12 * 1024) return false;
  int t = 256;
  while (t < 1024 && group_cap > 4 * t) t *= 2;
  plan->threads = t;
  const int need = int((group_cap + t - 1) / t);
  plan->items = need <= 2 ? 2 : need <= 4 ? 4 : need <= 6 ? 6 : need <= 8 ? 8 : 12;
  plan->n_narrow = plan->n_wide = 0;
  plan->slot32_mask = 0;
  for (int n = 1; n <= N; ++n) {
    if (key_bytes[n - 1] == 16) {
      plan->wide_orders[plan->n_wide++] = n;
    } else {
      plan->narrow_orders[plan->n_narrow++] = n;
      if (n * bits <= 32) plan->slot32_mask |= 1 << n;
    }
  }
  int slots = 256;
  while (int64_t(slots) * 3 < group_cap * 4) slots <<= 1;
  plan->narrow_slots = plan->wide_slots = slots;
  plan->narrow_lds = size_t(slots + 1) * 8;
  // every 16-byte order within 64 + 18 bits and 13-bit positions: stage the low halves only
  plan->wide_compact = group_cap <= 8192 && N * bits <= 64 + 18;
  plan->wide_table_off = size_t(group_cap) * (plan->wide_compact ? 8 : 16);
  plan->wide_lds = plan->wide_table_off + size_t(slots) * 4;
  bool ok = true;
  if (plan->n_narrow) ok = ok && plan->narrow_lds + 256 <= size_t(kLdsBudget);
  if (plan->n_wide) ok = ok && plan->wide_lds + 256 <= size_t(kLdsBudget) && group_cap <= 65535;
  return ok;
}

// Keys of at most 64 bits.  The open-addressing table holds the keys themselves, as 4-byte
// entries when the order's keys fit 32 bits (twice the slots in the same LDS, cheaper atomics)
// and as 8-byte entries otherwise; an insertion is one LDS compare-and-swap per probe (double
// hashing).  All-ones is the empty marker, so the one key with that bit pattern owns the extra
// entry at index T.  The thread whose compare-and-swap created an entry gives it a dense id
// and, once every insertion is done, replaces the key in the table by that id.
// `key` holds this thread's keys of the order (already in registers), `count` the group's
// number of n-grams of the order.  Starts and ends with the table free for reuse.
template <int ITEMS, typename SlotT>
__device__ __forceinline__ void narrow_dictionary(const DictArgs& a, unsigned char* smem,
                                                  int* next_id, int g, int n,
                                                  const uint64_t (&key64)[ITEMS], int count) {
  constexpr bool kSmall = sizeof(SlotT) == 4;
  const SlotT kFree = ~SlotT(0);
  const Problem& pb = a.pb;
  const int nt = blockDim.x, tid = threadIdx.x;
  SlotT* table = reinterpret_cast<SlotT*>(smem);
  const int T = kSmall ? 2 * a.table_slots : a.table_slots;
  const int shift = kSmall ? a.table_shift - 1 : a.table_shift;
  const uint32_t mask = uint32_t(T) - 1u;
  uint32_t* ginv = a.ws.inv[n - 1] + int64_t(g) * pb.group_cap;

  for (int s = tid; s <= T; s += nt) table[s] = kFree;
  if (tid == 0) *next_id = 0;
  __syncthreads();

  uint32_t slot[ITEMS];
  uint32_t created = 0;  // bit i: this thread's item i created its table entry
#pragma unroll
  for (int i = 0; i < ITEMS; ++i) {
    const int k = tid + i * nt;
    slot[i] = 0;
    if (k < count) {
      const SlotT key = SlotT(key64[i]);
      if (key == kFree) {
        if (atomicCAS(&table[T], kFree, SlotT(0)) == kFree) created |= 1u << i;
        slot[i] = uint32_t(T);
      } else {
        uint32_t h;
        if (kSmall) {
          h = uint32_t(key) * 0x9E3779B1u;
        } else {
          const uint32_t lo = uint32_t(key), hi = uint32_t(uint64_t(key) >> 32);
          h = (lo ^ ((hi << 15) | (hi >> 17))) * 0x9E3779B1u;
        }
        const uint32_t step = (h >> 3) | 1u;
        uint32_t s = h >> shift;
        SlotT old = atomicCAS(&table[s], kFree, key);
        int rounds = 0;  // equal in all lanes still probing (scalar); T probes reach every slot
        while (int(old != kFree) & int(old != key) & int(rounds < T)) {
          s = (s + step) & mask;
          old = atomicCAS(&table[s], kFree, key);
          rounds = __builtin_amdgcn_readfirstlane(rounds) + 1;
        }
        if (old == kFree) created |= 1u << i;
        slot[i] = s;
      }
    }
  }
  uint32_t id = reserve_ids(__popc(created), next_id);
  __syncthreads();  // nobody compares keys any more: entries may now hold ids
#pragma unroll
  for (int i = 0; i < ITEMS; ++i)
    if ((created >> i) & 1u) table[slot[i]] = SlotT(id++);
  __syncthreads();

  const uint32_t gbase = uint32_t(int64_t(g) * pb.group_cap);
#pragma unroll
  for (int i = 0; i < ITEMS; ++i) {
    const int k = tid + i * nt;
    if (k < count) ginv[k] = gbase + uint32_t(table[slot[i]]);
  }
  if (tid == 0) a.distinct[int64_t(g) * pb.N + n - 1] = *next_id;
  __syncthreads();  // ids read, next_id read: table and counter are free again
}

// One workgroup builds the dictionaries of up to two orders of one group, one after the other
// in the same LDS.  The keys of both orders are requested together, so the second order never
// waits for memory; the host pairs a cheap order with an expensive one.
template <int ITEMS>
__global__ __launch_bounds__(1024) void dictionary_narrow_kernel(DictArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int next_id;
  const Problem& pb = a.pb;
  const int nt = blockDim.x, tid = threadIdx.x;
  const int g = blockIdx.x / a.num_pairs;
  const int pair = blockIdx.x % a.num_pairs;
  const int n0 = a.orders[2 * pair], n1 = a.orders[2 * pair + 1];  // n1 = 0: single order
  GroupIndex gi(pb, g);
  gi.set_order(n0);
  const int count0 = min(gi.start(pb.R + 1), ITEMS * nt);
  int count1 = 0;
  if (n1) {
    gi.set_order(n1);
    count1 = min(gi.start(pb.R + 1), ITEMS * nt);
  }
  uint64_t key0[ITEMS], key1[ITEMS];
  {
    const uint64_t* gkeys =
        reinterpret_cast<const uint64_t*>(a.ws.keys[n0 - 1]) + int64_t(g) * pb.group_cap;
    // unconditional loads (slots past the count re-read the last key, a cache hit): branches
    // around loads would make the compiler wait for earlier loads before issuing later ones
    const int last = max(count0 - 1, 0);
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) key0[i] = gkeys[min(tid + i * nt, last)];
  }
  {
    const uint64_t* gkeys =
        reinterpret_cast<const uint64_t*>(a.ws.keys[max(n1, 1) - 1]) + int64_t(g) * pb.group_cap;
    const int last = max(count1 - 1, 0);
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) key1[i] = gkeys[min(tid + i * nt, last)];
  }
  if ((a.slot32_mask >> n0) & 1)
    narrow_dictionary<ITEMS, uint32_t>(a, smem, &next_id, g, n0, key0, count0);
  else
    narrow_dictionary<ITEMS, unsigned long long>(a, smem, &next_id, g, n0, key0, count0);
  if (n1 == 0) return;
  if ((a.slot32_mask >> n1) & 1)
    narrow_dictionary<ITEMS, uint32_t>(a, smem, &next_id, g, n1, key1, count1);
  else
    narrow_dictionary<ITEMS, unsigned long long>(a, smem, &next_id, g, n1, key1, count1);
}

// 16-byte keys (n*bits > 64): no 128-bit LDS atomic exists, so the keys are staged in LDS and the
// table holds 32-bit words claimed with a compare-and-swap that name the position of the
// occurrence representing the n-gram.  Ids as in the narrow kernel.
//   COMPACT (keys of at most 64 + 18 bits, groups of at most 8192 n-grams): the word is the
//     key's bits above 64 next to a 13-bit position, and only the low 64 bits are staged, which
//     halves the LDS; a match compares those bits exactly and then the staged low halves.
//   otherwise: a 16-bit fingerprint next to a 16-bit position; a fingerprint match is confirmed
//     on the staged 128-bit keys.
template <int ITEMS, bool COMPACT>
__global__ __launch_bounds__(1024) void dictionary_wide_kernel(DictArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int next_id;
  const Problem& pb = a.pb;
  const int nt = blockDim.x, tid = threadIdx.x;
  const int g = blockIdx.x / a.num_orders;
  const int n = a.orders[blockIdx.x % a.num_orders];
  Key128* skeys = reinterpret_cast<Key128*>(smem);
  uint64_t* slow = reinterpret_cast<uint64_t*>(smem);  // COMPACT: low halves only
  uint32_t* table = reinterpret_cast<uint32_t*>(smem + a.lds_table_off);
  const int T = a.table_slots;
  const uint32_t mask = uint32_t(T) - 1u;
  const int count =
      min(min(GroupIndex(pb, g, n).start(pb.R + 1), ITEMS * nt), int(pb.group_cap));
  const Key128* gkeys =
      reinterpret_cast<const Key128*>(a.ws.keys[n - 1]) + int64_t(g) * pb.group_cap;
  uint32_t* ginv = a.ws.inv[n - 1] + int64_t(g) * pb.group_cap;

  Key128 key[ITEMS];
  const int last = max(count - 1, 0);  // unconditional loads, as in the narrow kernel
#pragma unroll
  for (int i = 0; i < ITEMS; ++i) key[i] = gkeys[min(tid + i * nt, last)];
  for (int s = tid; s < T; s += nt) table[s] = kEmpty;
  if (tid == 0) next_id = 0;
#pragma unroll
  for (int i = 0; i < ITEMS; ++i) {
    const int k = tid + i * nt;
    if (k < count) {
      if (COMPACT)
        slow[k] = key[i].lo;
      else
        skeys[k] = key[i];
    }
  }
  __syncthreads();

  uint32_t slot[ITEMS];
  uint32_t created = 0;
#pragma unroll
  for (int i = 0; i < ITEMS; ++i) {
    const int k = tid + i * nt;
    slot[i] = 0;
    if (k < count) {
      const uint32_t h = key_hash(key[i]);
      const uint32_t step = (h >> 8) | 1u;
      // COMPACT: the high bits are < 2^18, so the word never equals the empty marker
      const uint32_t tag = COMPACT ? uint32_t(key[i].hi) : h >> 16;
      const uint32_t mine = COMPACT ? (tag << 13) | uint32_t(k) : (tag << 16) | uint32_t(k);
      uint32_t s = h & mask;
      int rounds = 0;  // equal in all lanes still probing (scalar); T probes reach every slot
      bool won, more;
      do {
        uint32_t w = table[s];
        if (w == kEmpty) w = atomicCAS(&table[s], kEmpty, mine);
        won = w == kEmpty;  // this occurrence now represents its n-gram
        bool same = false;
        if (COMPACT) {
          if (!won && (w >> 13) == tag) same = slow[w & 0x1FFFu] == key[i].lo;
        } else {
          if (!won && (w >> 16) == tag) same = key_eq(skeys[w & 0xFFFFu], key[i]);
        }
        rounds = __builtin_amdgcn_readfirstlane(rounds) + 1;
        more = !won && !same && rounds < T;
        s = more ? (s + step) & mask : s;
      } while (more);
      if (won) created |= 1u << i;
      slot[i] = s;
    }
  }
  uint32_t id = reserve_ids(__popc(created), &next_id);
  __syncthreads();
#pragma unroll
  for (int i = 0; i < ITEMS; ++i)
    if ((created >> i) & 1u) table[slot[i]] = id++;
  __syncthreads();

  const uint32_t gbase = uint32_t(int64_t(g) * pb.group_cap);
#pragma unroll
  for (int i = 0; i < ITEMS; ++i) {
    const int k = tid + i * nt;
    if (k < count) ginv[k] = gbase + table[slot[i]];
  }
  if (tid == 0) a.distinct[int64_t(g) * pb.N + n - 1] = next_id;
}

template <template <int> class Launcher, typename... Args>
hipError_t dispatch_items(int items, Args&&... args) {
  switch (items) {
    case 2: return Launcher<2>::run(args...);
    case 4: return Launcher<4>::run(args...);
    case 6: return Launcher<6>::run(args...);
    case 8: return Launcher<8>::run(args...);
    case 12: return Launcher<12>::run(args...);
    default: return hipErrorInvalidValue;
  }
}

template <typename Kernel, typename ArgT>
hipError_t launch_with_lds(Kernel kernel, const ArgT& a, int64_t blocks, int threads, size_t lds,
                           hipStream_t s) {
  if (blocks <= 0 || blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
  hipError_t e = grant_dynamic_lds(reinterpret_cast<const void*>(kernel), lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kernel, dim3(uint32_t(blocks)), dim3(threads), lds, s, a);
  return hipGetLastError();
}

template <int ITEMS>
struct NarrowLauncher {
  static hipError_t run(const DictArgs& a, int64_t blocks, int threads, size_t lds,
                        hipStream_t s) {
    return launch_with_lds(dictionary_narrow_kernel<ITEMS>, a, blocks, threads, lds, s);
  }
};
template <int ITEMS>
struct WideLauncher {
  static hipError_t run(const DictArgs& a, int64_t blocks, int threads, size_t lds,
                        hipStream_t s) {
    return launch_with_lds(dictionary_wide_kernel<ITEMS, false>, a, blocks, threads, lds, s);
  }
};
template <int ITEMS>
struct CompactWideLauncher {
  static hipError_t run(const DictArgs& a, int64_t blocks, int threads, size_t lds,
                        hipStream_t s) {
    return launch_with_lds(dictionary_wide_kernel<ITEMS, true>, a, blocks, threads, lds, s);
  }
};

hipError_t launch_dictionary(const Problem& pb, const GlobalWs& ws, const DictPlan& plan,
                             int32_t* distinct, hipStream_t s) {
  DictArgs a;
  a.pb = pb;
  a.ws = ws;
  a.distinct = distinct;
  a.slot32_mask = 0;
  auto shift_of = [](int slots) {
    int lg = 0;
    while ((1 << lg) < slots) ++lg;
    return 32 - lg;
  };
  if (plan.n_narrow) {
    a.table_slots = plan.narrow_slots;
    a.table_shift = shift_of(plan.narrow_slots);
    a.lds_table_off = 0;
    a.slot32_mask = plan.slot32_mask;
    // Pairs of about equal cost (cost grows with the order): the cheapest with the most
    // expensive, e.g. four orders -> (1st, 4th) and (2nd, 3rd).  An odd number of orders would leave workgroups of unequal length, which
    // measured slower than one order per workgroup; a small batch keeps one order per workgroup
    // so that the GPU still fills.
    const int m = plan.n_narrow;
    const bool pairs = int64_t(pb.B) * m >= 1024 && m % 2 == 0;
    int np = 0;
    auto add = [&](int first, int second) {
      a.orders[2 * np] = plan.narrow_orders[first];
      a.orders[2 * np + 1] = second >= 0 ? plan.narrow_orders[second] : 0;
      ++np;
    };
    if (!pairs) {
      for (int k = 0; k < m; ++k) add(k, -1);
    } else {
      for (int k = 0; k < m / 2; ++k) add(k, m - 1 - k);
    }
    a.num_pairs = np;
    hipError_t e = dispatch_items<NarrowLauncher>(plan.items, a, int64_t(pb.B) * a.num_pairs,
                                                  plan.threads, plan.narrow_lds, s);
    if (e != hipSuccess) return e;
  }
  if (plan.n_wide) {
    a.table_slots = plan.wide_slots;
    a.table_shift = shift_of(plan.wide_slots);
    a.lds_table_off = uint32_t(plan.wide_table_off);
    a.num_orders = plan.n_wide;
    for (int k = 0; k < 8; ++k) a.orders[k] = plan.wide_orders[k];
    const int64_t blocks = int64_t(pb.B) * plan.n_wide;
    hipError_t e = plan.wide_compact
                       ? dispatch_items<CompactWideLauncher>(plan.items, a, blocks, plan.threads,
                                                             plan.wide_lds, s)
                       : dispatch_items<WideLauncher>(plan.items, a, blocks, plan.threads,
                                                      plan.wide_lds, s);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// ---------------------------------------------------------------------------- count + clip

struct CountArgs {
  Problem pb;
  GlobalWs ws;
  StatPtrs st;
  int words;  // count_fields_kernel: 32-bit words per dictionary entry
  int split;  // count_fields_kernel: workgroups per group; workgroup r of a group handles the
              // orders r + 1, r + 1 + split, ...
};

// Workgroups per group for a kernel that walks several orders: one when the groups alone fill
// the GPU, more when the batch is small.
static int order_split(int B, int N) {
  int split = 1;
  while (split < N && (int64_t(B) * split < 384 || 4 * split < N)) split *= 2;  // <= 4 orders each
  return split < N ? split : N;
}

bool plan_count(int64_t group_cap, int64_t cand_stride, int64_t ref_stride, int R,
                CountPlan* plan) {
  // every counter is a 16-bit field of an LDS word
  if (group_cap < 1 || group_cap > 12 * 1024 || ref_stride > 65535 || cand_stride > 65535)
    return false;
  int t = 256;
  while (t < 1024 && group_cap > 4 * t) t *= 2;
  plan->threads = t;
  const int need = int((group_cap + t - 1) / t);
  plan->items = need <= 2 ? 2 : need <= 4 ? 4 : need <= 6 ? 6 : need <= 8 ? 8 : 12;
  // one field per sequence when that fits (and the wave-wide sequence lookup applies), else
  // the two-references-at-a-time kernel
  plan->words = (R + 2) / 2;
  const size_t field_lds = (size_t(group_cap) * plan->words * 4 + 15) & ~size_t(15);
  plan->fields = R < kWave - 1 && field_lds + 256 <= size_t(kLdsBudget) / 2;
  plan->lds_bytes = plan->fields ? field_lds : size_t(group_cap) * 8;
  return plan->lds_bytes + 256 <= size_t(kLdsBudget);
}

// One workgroup per group walks the orders n = first, first + split, ... (at most four); the
// offset ids of the next order are requested while the current one is counted, so only the
// first order of a workgroup waits for memory.
// A dictionary entry owns `words` LDS words holding one 16-bit counter per sequence of the
// group (field 0: candidate, field 1 + j: reference j).  One LDS atomic add per n-gram
// occurrence.  The candidate occurrence whose add finds its field at zero is the first of its
// n-gram; after the barrier it alone clips the entry (maximum over the reference fields,
// minimum with the candidate field), so no sweep over the table is needed.
template <int ITEMS>
__global__ __launch_bounds__(1024) void count_fields_kernel(CountArgs a) {
  static_assert(ITEMS % 2 == 0, "items are processed in pairs");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int clipped_sum[4];
  const Problem& pb = a.pb;
  const int nt = blockDim.x, tid = threadIdx.x, lane = tid & (kWave - 1);
  const int g = blockIdx.x / a.split;
  const int first_order = blockIdx.x % a.split + 1;
  const int cap = int(pb.group_cap);
  const int W = a.words;
  uint32_t* cnt = reinterpret_cast<uint32_t*>(smem);
  const uint32_t gbase = uint32_t(int64_t(g) * pb.group_cap);

  // Slot layout: a wavefront owns blocks of 128 consecutive slots (block p of wavefront w starts
  // at 128 * w + p * 2 * nt); lane l holds the slots l and 64 + l of each block as items 2p and
  // 2p + 1.  The scalar work that finds a block's sequence is then shared by 128 n-grams.
  const int wave_block = __builtin_amdgcn_readfirstlane(2 * (tid - lane));
  auto block_start = [&](int p) { return wave_block + p * 2 * nt; };

  GroupIndex gi(pb, g, GroupIndex::WaveOnly{});  // the loads of the lengths go out first
  int U4[4], total4[4] = {0, 0, 0, 0};
  uint32_t id[4][ITEMS];
  // The id loads are unconditional (clamped slot, clamped order) so that the hardware's in-order
  // load counter lets an order start as soon as its own ids have arrived; the ids of order o + 1
  // are requested when order o starts, which spreads the memory traffic over the kernel.  The
  // first order's request goes out before the lengths have arrived and therefore covers the
  // group's whole slot range (slots past the count hold stale bytes that are never used); later
  // requests stop at the order's real n-gram count (slots beyond re-read its last id, a cache
  // hit).
  auto request_ids = [&](int o, int last_slot) {
    const int n = min(first_order + o * a.split, pb.N);
    const uint32_t* ginv = a.ws.inv[n - 1] + int64_t(g) * pb.group_cap;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i)
      id[o][i] = ginv[min(block_start(i >> 1) + (i & 1) * kWave + lane, last_slot)];
  };
  request_ids(0, cap - 1);
#pragma unroll
  for (int o = 0; o < 4; ++o)
    U4[o] = a.st.distinct[int64_t(g) * pb.N + min(first_order + o * a.split, pb.N) - 1];
  if (tid < 4) clipped_sum[tid] = 0;
  gi.set_order(first_order);

#pragma unroll
  for (int o = 0; o < 4; ++o) {
    const int n = first_order + o * a.split;
    if (n > pb.N) break;
    const int U = min(max(U4[o], 0), cap);
    // this order's slot ranges (the index already holds order n) ...
    const int count = min(gi.start(pb.R + 1), ITEMS * nt);
    const int ccnt = gi.start(1);
    const int seq_end = (lane <= pb.R) ? gi.end_in_lane() : 0x7FFFFFFF;
    // ... then the next order's, for its request
    if (o < 3) {
      const int next = min(n + a.split, pb.N);
      gi.set_order(next);
      request_ids(o + 1, max(min(gi.start(pb.R + 1), cap) - 1, 0));
    }
    if (o > 0) __syncthreads();  // the previous order's entries have been clipped
    {
      uint4* c4 = reinterpret_cast<uint4*>(cnt);
      const int quads = (U * W + 3) / 4;
      for (int q = tid; q < quads; q += nt) c4[q] = make_uint4(0u, 0u, 0u, 0u);
    }
    __syncthreads();

    // Sequence of a slot = number of sequences that end at or before it (seq_end: lane j holds
    // the end of sequence j).  A block's 128 slots usually lie inside one sequence, which one
    // ballot finds; then sequence, counter word and addend are scalars for both items.
    // Ids are clamped to the dictionary size instead of tested against it: every id the
    // dictionary pass wrote is below U, so the clamp only matters for a workspace that pass never
    // filled, where it keeps the LDS accesses inside the table.
    const uint32_t u_max = uint32_t(max(U, 1) - 1);
    uint32_t first = 0;  // bit i: item i is the first occurrence of its candidate n-gram
    // one n-gram whose sequence is known per lane
    auto count_one = [&](int i, uint32_t u, int f) {
      if (f <= pb.R) {
        uint32_t* word = &cnt[__umul24(u, uint32_t(W)) + uint32_t(f >> 1)];
        if (f == 0) {
          if ((atomicAdd(word, 1u) & 0xFFFFu) == 0u) first |= 1u << i;
        } else {
          atomicAdd(word, (f & 1) ? 0x10000u : 1u);
        }
      }
    };
#pragma unroll
    for (int p = 0; p < ITEMS / 2; ++p) {
      const int k0 = block_start(p);
      if (k0 >= count) break;
      const int f = __popcll(__builtin_amdgcn_ballot_w64(seq_end <= k0));  // <= R: k0 < count
      const int f_end = __builtin_amdgcn_readlane(seq_end, f);
      const uint32_t u0 = min(id[o][2 * p] - gbase, u_max);
      const uint32_t u1 = min(id[o][2 * p + 1] - gbase, u_max);
      if (k0 + 2 * kWave <= f_end) {  // the whole block is inside sequence f
        uint32_t* w0 = &cnt[__umul24(u0, uint32_t(W)) + uint32_t(f >> 1)];
        uint32_t* w1 = &cnt[__umul24(u1, uint32_t(W)) + uint32_t(f >> 1)];
        if (f == 0) {  // candidate slots: remember the first occurrence of each n-gram
          const uint32_t before0 = atomicAdd(w0, 1u), before1 = atomicAdd(w1, 1u);
          first |= ((before0 & 0xFFFFu) == 0u ? 1u : 0u) << (2 * p);
          first |= ((before1 & 0xFFFFu) == 0u ? 1u : 0u) << (2 * p + 1);
        } else {
          const uint32_t addend = (f & 1) ? 0x10000u : 1u;
          atomicAdd(w0, addend);
          atomicAdd(w1, addend);
        }
      } else {  // the block straddles sequences (or the end): sequence per lane and half
        const int f_hi = __popcll(__builtin_amdgcn_ballot_w64(seq_end <= k0 + 2 * kWave - 1));
        int fl0 = f, fl1 = f;
        for (int j = f; j < f_hi; ++j) {
          const int e = __builtin_amdgcn_readlane(seq_end, j);
          fl0 += (k0 + lane >= e);
          fl1 += (k0 + kWave + lane >= e);
        }
        count_one(2 * p, u0, fl0);
        count_one(2 * p + 1, u1, fl1);
      }
    }
    __syncthreads();

    int part = 0;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      // only candidate slots can be first occurrences
      if (block_start(i >> 1) + (i & 1) * kWave >= ccnt) break;
      if ((first >> i) & 1u) {
        const uint32_t* e = &cnt[__umul24(min(id[o][i] - gbase, u_max), uint32_t(W))];
        const uint32_t w0 = e[0];
        uint32_t m = w0 >> 16;
        // (the first words unrolled under a scalar test: the usual few references need no loop)
#pragma unroll
        for (int q = 1; q < 4; ++q) {
          if (q < W) {
            const uint32_t w = e[q];
            m = max(m, max(w & 0xFFFFu, w >> 16));
          }
        }
        for (int q = 4; q < W; ++q) {
          const uint32_t w = e[q];
          m = max(m, max(w & 0xFFFFu, w >> 16));
        }
        part += int(min(w0 & 0xFFFFu, m));
      }
    }
    part = wave_sum(part);
    if (lane == 0 && part) atomicAdd(&clipped_sum[o], part);
    total4[o] = ccnt;
  }
  __syncthreads();
  if (tid < 4) {
    const int n = first_order + tid * a.split;
    if (n <= pb.N) {
      a.st.clipped[int64_t(g) * pb.N + n - 1] = clipped_sum[tid];
      a.st.total[int64_t(g) * pb.N + n - 1] =
          tid == 0 ? total4[0] : tid == 1 ? total4[1] : tid == 2 ? total4[2] : total4[3];
    }
  }
}

// Fallback for groups whose per-sequence fields do not fit.  One workgroup per (group, order).
// All of the group's offset ids are fetched into registers in one round trip; LDS holds two
// words per dictionary entry:
//   acc[u] = candidate count (low 16 bits) | maximum reference count so far (high 16 bits)
//   cur[u] = counts of the two references being histogrammed (16 bits each)
// References are histogrammed two at a time with LDS atomic adds and folded into the maximum.
template <int ITEMS>
__global__ __launch_bounds__(1024) void count_clip_kernel(CountArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int red_scratch[17];
  const Problem& pb = a.pb;
  const int nt = blockDim.x, tid = threadIdx.x;
  const int g = blockIdx.x / pb.N;
  const int n = blockIdx.x % pb.N + 1;
  const int cap = int(pb.group_cap);
  uint32_t* acc = reinterpret_cast<uint32_t*>(smem);
  uint32_t* cur = acc + cap;
  const uint32_t* ginv = a.ws.inv[n - 1] + int64_t(g) * pb.group_cap;
  const uint32_t gbase = uint32_t(int64_t(g) * pb.group_cap);
  // The loads go out before the group's n-gram count is known (that needs the lengths, another
  // round trip to memory): every slot of the group's range exists, slots past the count hold
  // stale bytes that are never used.
  uint32_t id[ITEMS];
#pragma unroll
  for (int i = 0; i < ITEMS; ++i) {
    const int k = tid + i * nt;
    id[i] = (k < cap) ? ginv[k] : 0u;
  }
  const int U = min(max(a.st.distinct[int64_t(g) * pb.N + n - 1], 0), cap);
  const GroupIndex gi(pb, g, n);
  const int count = min(gi.start(pb.R + 1), ITEMS * nt);
#pragma unroll
  for (int i = 0; i < ITEMS; ++i) id[i] = (tid + i * nt < count) ? id[i] - gbase : 0xFFFFFFFFu;
  for (int u = tid; u < U; u += nt) {
    acc[u] = 0;
    cur[u] = 0;
  }
  __syncthreads();

  const int ccnt = gi.start(1);
#pragma unroll
  for (int i = 0; i < ITEMS; ++i) {
    const int k = tid + i * nt;
    if (k < ccnt && id[i] < uint32_t(U)) atomicAdd(&acc[id[i]], 1u);
  }
  int lo = ccnt;  // first slot of the reference pair being processed
  for (int j = 0; j < pb.R; j += 2) {
    const int mid = gi.start(j + 2);
    const int hi = (j + 1 < pb.R) ? gi.start(j + 3) : mid;
#pragma unroll
    for (int i = 0; i < ITEMS; ++i) {
      const int k = tid + i * nt;
      if (k >= lo && k < hi && id[i] < uint32_t(U))
        atomicAdd(&cur[id[i]], (k < mid) ? 1u : 0x10000u);
    }
    lo = hi;
    __syncthreads();
    if (j + 2 < pb.R) {
      for (int u = tid; u < U; u += nt) {
        const uint32_t w = cur[u];
        const uint32_t m = max(w & 0xFFFFu, w >> 16);
        const uint32_t x = acc[u];
        acc[u] = (x & 0xFFFFu) | (max(x >> 16, m) << 16);
        cur[u] = 0;
      }
      __syncthreads();
    }
  }
  int part = 0;
  for (int u = tid; u < U; u += nt) {
    const uint32_t w = cur[u], x = acc[u];
    const uint32_t m = max(max(w & 0xFFFFu, w >> 16), x >> 16);
    part += int(min(x & 0xFFFFu, m));
  }
  const int clipped = block_sum(part, red_scratch);
  if (tid == 0) {
    a.st.clipped[int64_t(g) * pb.N + n - 1] = clipped;
    a.st.total[int64_t(g) * pb.N + n - 1] = ccnt;
  }
}

template <int ITEMS>
struct FieldCountLauncher {
  static hipError_t run(const CountArgs& a, int64_t blocks, int threads, size_t lds,
                        hipStream_t s) {
    return launch_with_lds(count_fields_kernel<ITEMS>, a, blocks, threads, lds, s);
  }
};
template <int ITEMS>
struct CountLauncher {
  static hipError_t run(const CountArgs& a, int64_t blocks, int threads, size_t lds,
                        hipStream_t s) {
    return launch_with_lds(count_clip_kernel<ITEMS>, a, blocks, threads, lds, s);
  }
};

hipError_t launch_count_clip(const Problem& pb, const GlobalWs& ws, const CountPlan& plan,
                             const StatPtrs& st, hipStream_t s) {
  CountArgs a;
  a.pb = pb;
  a.ws = ws;
  a.st = st;
  a.words = plan.words;
  a.split = order_split(pb.B, pb.N);
  if (plan.fields)
    return dispatch_items<FieldCountLauncher>(plan.items, a, int64_t(pb.B) * a.split,
                                              plan.threads, plan.lds_bytes, s);
  return dispatch_items<CountLauncher>(plan.items, a, int64_t(pb.B) * pb.N, plan.threads,
                                       plan.lds_bytes, s);
}

}  // namespace tb
