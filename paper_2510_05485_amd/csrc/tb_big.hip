// GLOBAL path for sentence groups too large for the LDS plans: the same dictionary and count/clip
// algorithms (paper Sections 3.2-3.3) with the hash table and the counters kept in the workspace
// (HBM / L2) instead of LDS.  One workgroup per (group, order) walks its n-grams in strides.
// Slower than the LDS kernels -- every probe is a device-scope atomic -- but exact and without a
// size limit other than the workspace; it exists so that long sequences are scored rather than
// rejected.
#include "tb_kernels.h"

namespace tb {

namespace {

constexpr unsigned long long kEmptyEntry = ~0ull;

struct BigArgs {
  Problem pb;
  GlobalWs ws;
  StatPtrs st;
  unsigned long long* tables;  // [B * N] tables of `slots` + 8 entries
  int64_t slots;               // power of two >= 2 * group_cap
  int table_shift;             // 32 - log2(slots) (slots <= 2^31)
  int32_t* rouge_overlap;      // count kernel, ROUGE-N: [B, R] (then order N only), or null
};

__device__ __forceinline__ int big_seq_len(const Problem& pb, int g, int j) {
  if (j == 0) return clamped_len(pb.cand_len[g], pb.cand_stride, nullptr);
  const RefRows rr = ref_rows(pb, g);
  if (j > rr.used) return 0;  // reference not in use
  return clamped_len(pb.ref_len[rr.row0 + j - 1], pb.ref_stride, nullptr);
}
// First compact slot of sequence j for order n (j = R + 1: the group's n-gram count).
__device__ __forceinline__ int64_t big_seq_start(const Problem& pb, int g, int n, int j) {
  int64_t s = 0;
  for (int jj = 0; jj < j; ++jj) s += max(big_seq_len(pb, g, jj) - n + 1, 0);
  return s;
}

__device__ __forceinline__ unsigned long long entry_load(const unsigned long long* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t word_load(const uint32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ uint32_t big_hash(uint64_t k) {
  const uint32_t lo = uint32_t(k), hi = uint32_t(k >> 32);
  return (lo ^ ((hi << 15) | (hi >> 17))) * 0x9E3779B1u;
}
__device__ __forceinline__ uint32_t big_hash(const Key128& k) {
  return big_hash(k.lo) ^ (big_hash(k.hi) * 0x85EBCA6Bu + 0x27D4EB2Fu);
}

// What a table entry holds for a key, and whether an occupied entry belongs to the same key.
// 8-byte keys are stored as they are (all-ones, the empty marker, is handled by the caller);
// 16-byte keys store hash:position and are confirmed against the key array.
__device__ __forceinline__ unsigned long long make_entry(uint64_t key, uint32_t, int64_t) {
  return key;
}
__device__ __forceinline__ unsigned long long make_entry(const Key128&, uint32_t h, int64_t k) {
  return (uint64_t(h) << 32) | uint64_t(uint32_t(k));
}
__device__ __forceinline__ bool same_key(unsigned long long e, uint64_t key, uint32_t,
                                         const uint64_t*) {
  return e == key;
}
__device__ __forceinline__ bool same_key(unsigned long long e, const Key128& key, uint32_t h,
                                         const Key128* keys) {
  return uint32_t(e >> 32) == h && key_eq(keys[uint32_t(e)], key);
}
__device__ __forceinline__ bool is_all_ones(uint64_t key) { return key == kEmptyEntry; }
__device__ __forceinline__ bool is_all_ones(const Key128&) { return false; }

template <typename KeyT>
__global__ __launch_bounds__(1024) void big_dictionary_kernel(BigArgs a, int want_wide) {
  __shared__ int scan_scratch[17];
  const Problem& pb = a.pb;
  const int nt = blockDim.x, tid = threadIdx.x;
  const int g = blockIdx.x / pb.N;
  const int n = blockIdx.x % pb.N + 1;
  if (a.ws.wide[n - 1] != want_wide) return;  // uniform: the other launch handles this order
  const int64_t S = a.slots;
  const uint32_t mask = uint32_t(S - 1);
  unsigned long long* table = a.tables + (int64_t(g) * pb.N + n - 1) * (S + 8);
  const KeyT* gkeys = reinterpret_cast<const KeyT*>(a.ws.keys[n - 1]) + int64_t(g) * pb.group_cap;
  uint32_t* ginv = a.ws.inv[n - 1] + int64_t(g) * pb.group_cap;
  const int64_t count = min(big_seq_start(pb, g, n, pb.R + 1), pb.group_cap);

  for (int64_t s = tid; s <= S; s += nt) table[s] = kEmptyEntry;
  __syncthreads();

  // insert every occurrence; remember its slot in the id array for now
  for (int64_t k = tid; k < count; k += nt) {
    const KeyT key = gkeys[k];
    uint32_t slot;
    if (is_all_ones(key)) {
      atomicCAS(&table[S], kEmptyEntry, 0ull);
      slot = uint32_t(S);
    } else {
      const uint32_t h = big_hash(key);
      const unsigned long long mine = make_entry(key, h, k);
      const uint32_t step = (h >> 3) | 1u;
      uint32_t s = h >> a.table_shift;
      for (int64_t probe = 0; probe < S; ++probe) {  // S probes reach every slot
        unsigned long long e = entry_load(&table[s]);
        if (e == kEmptyEntry) e = atomicCAS(&table[s], kEmptyEntry, mine);
        if (e == kEmptyEntry || same_key(e, key, h, gkeys)) break;
        s = (s + step) & mask;
      }
      slot = s;
    }
    ginv[k] = slot;
  }
  __syncthreads();

  // number the occupied entries densely, a workgroup-wide scan per stride of the table
  int base = 0;
  for (int64_t s0 = 0; s0 <= S; s0 += nt) {
    const int64_t s = s0 + tid;
    const int occupied = (s <= S && entry_load(&table[s]) != kEmptyEntry) ? 1 : 0;
    int total = 0;
    const int excl = block_exclusive_scan(occupied, scan_scratch, &total);
    if (occupied) table[s] = uint64_t(base + excl);
    base += total;
  }
  __syncthreads();

  const uint32_t gbase = uint32_t(int64_t(g) * pb.group_cap);
  for (int64_t k = tid; k < count; k += nt)
    ginv[k] = gbase + uint32_t(entry_load(&table[ginv[k]]));
  if (tid == 0) a.st.distinct[int64_t(g) * pb.N + n - 1] = base;
}

// Counters in the (now free) table memory: three 32-bit arrays per (group, order).
__global__ __launch_bounds__(1024) void big_count_kernel(BigArgs a) {
  __shared__ int red_scratch[17];
  const Problem& pb = a.pb;
  const int nt = blockDim.x, tid = threadIdx.x;
  // BLEU: one workgroup per (group, order).  ROUGE-N: one per group, order N, and every
  // reference's pass also sums min(candidate count, the reference's count) over the ids.
  const bool rouge = a.rouge_overlap != nullptr;
  const int g = rouge ? int(blockIdx.x) : int(blockIdx.x) / pb.N;
  const int n = rouge ? pb.N : int(blockIdx.x) % pb.N + 1;
  const int64_t cap = pb.group_cap;
  uint32_t* acc = reinterpret_cast<uint32_t*>(a.tables + (int64_t(g) * pb.N + n - 1) * (a.slots + 8));
  uint32_t* cur = acc + cap;
  uint32_t* mx = cur + cap;
  const uint32_t* ginv = a.ws.inv[n - 1] + int64_t(g) * cap;
  const uint32_t gbase = uint32_t(int64_t(g) * cap);
  const int64_t U = min(int64_t(max(a.st.distinct[int64_t(g) * pb.N + n - 1], 0)), cap);

  for (int64_t u = tid; u < U; u += nt) {
    acc[u] = 0;
    cur[u] = 0;
    mx[u] = 0;
  }
  __syncthreads();
  const int64_t ccnt = min(big_seq_start(pb, g, n, 1), cap);
  for (int64_t k = tid; k < ccnt; k += nt) {
    const uint32_t id = ginv[k] - gbase;
    if (id < U) atomicAdd(&acc[id], 1u);
  }
  int64_t lo = ccnt;
  for (int j = 0; j < pb.R; ++j) {
    const int64_t hi = min(lo + max(big_seq_len(pb, g, j + 1) - n + 1, 0), cap);
    for (int64_t k = lo + tid; k < hi; k += nt) {
      const uint32_t id = ginv[k] - gbase;
      if (id < U) atomicAdd(&cur[id], 1u);
    }
    lo = hi;
    __syncthreads();
    int both = 0;
    for (int64_t u = tid; u < U; u += nt) {  // entry u always belongs to the same thread
      const uint32_t c = word_load(&cur[u]);
      mx[u] = max(mx[u], c);
      if (rouge) both += int(min(word_load(&acc[u]), c));
      cur[u] = 0;
    }
    if (rouge) {  // uniform
      const int overlap = block_sum(both, red_scratch);
      if (tid == 0) a.rouge_overlap[int64_t(g) * pb.R + j] = overlap;
    }
    __syncthreads();
  }
  int part = 0;
  for (int64_t u = tid; u < U; u += nt) part += int(min(word_load(&acc[u]), mx[u]));
  const int clipped = block_sum(part, red_scratch);
  if (tid == 0) {
    a.st.clipped[int64_t(g) * pb.N + n - 1] = clipped;
    a.st.total[int64_t(g) * pb.N + n - 1] = int(ccnt);
  }
}

BigArgs make_args(const Problem& pb, const GlobalWs& ws, const BigPlan& plan,
                  const StatPtrs& st) {
  BigArgs a;
  a.pb = pb;
  a.ws = ws;
  a.st = st;
  a.tables = static_cast<unsigned long long*>(ws.tables);
  a.slots = plan.slots;
  int lg = 0;
  while ((int64_t(1) << lg) < plan.slots) ++lg;
  a.table_shift = 32 - lg;
  a.rouge_overlap = nullptr;
  return a;
}

}  // namespace

bool plan_big(int64_t group_cap, int N, BigPlan* plan) {
  (void)N;
  if (group_cap < 1 || group_cap > (int64_t(1) << 24)) return false;
  int64_t slots = 1024;
  while (slots < 2 * group_cap) slots <<= 1;
  plan->slots = slots;
  plan->table_entries = slots + 8;  // entry `slots` belongs to the all-ones key; padded
  return true;
}

hipError_t launch_big_dictionary(const Problem& pb, const GlobalWs& ws, const BigPlan& plan,
                                 const StatPtrs& st, hipStream_t s) {
  const BigArgs a = make_args(pb, ws, plan, st);
  const int64_t blocks = int64_t(pb.B) * pb.N;
  if (blocks <= 0 || blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
  bool any_wide = false, any_narrow = false;
  for (int n = 0; n < pb.N; ++n) (ws.wide[n] ? any_wide : any_narrow) = true;
  if (any_narrow) {
    hipLaunchKernelGGL(big_dictionary_kernel<uint64_t>, dim3(uint32_t(blocks)), dim3(1024), 0, s,
                       a, 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (any_wide) {
    hipLaunchKernelGGL(big_dictionary_kernel<Key128>, dim3(uint32_t(blocks)), dim3(1024), 0, s, a,
                       1);
    return hipGetLastError();
  }
  return hipSuccess;
}

hipError_t launch_big_count_clip(const Problem& pb, const GlobalWs& ws, const BigPlan& plan,
                                 const StatPtrs& st, hipStream_t s, int32_t* rouge_overlap) {
  BigArgs a = make_args(pb, ws, plan, st);
  a.rouge_overlap = rouge_overlap;
  const int64_t blocks = rouge_overlap ? int64_t(pb.B) : int64_t(pb.B) * pb.N;
  if (blocks <= 0 || blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
  hipLaunchKernelGGL(big_count_kernel, dim3(uint32_t(blocks)), dim3(1024), 0, s, a);
  return hipGetLastError();
}

}  // namespace tb
