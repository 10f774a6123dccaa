// GLOBAL path kernels: pack -> dictionary -> count/clip, with keys and inverse indices in HBM.
//
// Mapping to the paper (Sections 3.1-3.3):
//   pack_kernel        n-gram extraction and the flattened list of valid n-grams, stored as
//                      packed integer keys instead of (total_ngrams, n) token rows;
//   dictionary_kernel  the compact dictionary + inverse indices (the role of torch.unique with
//                      return_inverse), built per sentence group in an LDS hash table;
//   count_clip_kernel  offset ids -> counts (the batched bincount), maximum over references,
//                      minimum with the candidate counts, summed per sentence and order.
// Clipping never compares n-grams of different sentence groups, so each group (a candidate and
// its references) gets its own dictionary; the group's offset g*group_cap keeps id ranges
// disjoint exactly like the paper's i*num_unique offset, with an a-priori bound in place of the
// data-dependent num_unique so that no size ever travels back to the host.
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
  __shared__ int32_t tok[kPackTile + 4];
  const Problem& pb = a.pb;
  const int per_group = a.cand_chunks + pb.R * a.ref_chunks;
  const int g = blockIdx.x / per_group;
  int rem = blockIdx.x % per_group;
  const int32_t* row;
  int len, chunk;
  int64_t slot_base = int64_t(g) * pb.group_cap;
  if (rem < a.cand_chunks) {
    chunk = rem;
    row = pb.cand + int64_t(g) * pb.cand_stride;
    len = clamped_len(pb.cand_len[g], pb.cand_stride, pb.status);
  } else {
    rem -= a.cand_chunks;
    const int j = rem / a.ref_chunks;
    chunk = rem % a.ref_chunks;
    row = pb.refs + (int64_t(g) * pb.R + j) * pb.ref_stride;
    len = clamped_len(pb.ref_len[int64_t(g) * pb.R + j], pb.ref_stride, pb.status);
    slot_base += pb.cand_stride + int64_t(j) * pb.ref_stride;
  }
  const int p0 = chunk * kPackTile;
  if (p0 >= len) return;  // uniform over the workgroup
  const int ntok = min(kPackTile + 3, len - p0);
  bool bad = false;
  for (int i = threadIdx.x; i < ntok; i += kPackThreads) {
    const int32_t t = row[p0 + i];
    tok[i] = t;
    bad |= (uint32_t(t) >= uint32_t(pb.vocab));
  }
  if (bad && pb.status) atomicOr(pb.status, TB_DEV_TOKEN_RANGE);
  __syncthreads();
  const int bits = pb.bits;
#pragma unroll
  for (int k = 0; k < kPackTile / kPackThreads; ++k) {
    const int q = threadIdx.x + k * kPackThreads;
    if (q >= ntok) break;
    const int avail = ntok - q;  // tokens available from this start, capped at tile + 3
    const int64_t slot = slot_base + p0 + q;
    uint64_t lo = uint32_t(tok[q]), hi = 0;
    store_key(a.ws.keys[0], a.ws.wide[0], slot, lo, hi);
#pragma unroll
    for (int n = 2; n <= 4; ++n) {
      if (n > pb.N || n > avail) break;
      hi = (hi << bits) | (lo >> (64 - bits));
      lo = (lo << bits) | uint32_t(tok[q + n - 1]);
      store_key(a.ws.keys[n - 1], a.ws.wide[n - 1], slot, lo, hi);
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
  int table_slots;
  uint32_t lds_table_off, lds_slot_off;
};

bool plan_dictionary(int64_t group_cap, const int32_t* key_bytes, int N, DictPlan* plan) {
  if (group_cap < 1 || group_cap > 65535) return false;  // positions are 16-bit in table words
  int kb = 8;
  for (int n = 0; n < N; ++n) kb = key_bytes[n] > kb ? key_bytes[n] : kb;
  plan->key_bytes = kb;
  plan->threads = group_cap > 2048 ? 1024 : (group_cap > 768 ? 512 : 256);
  int slots = 1;
  while (slots < 2 * group_cap) slots <<= 1;
  if (slots < plan->threads) slots = plan->threads;
  plan->table_slots = slots;
  size_t off = size_t(group_cap) * kb;
  off = (off + 15) & ~size_t(15);
  plan->lds_table_off = off;
  off += size_t(slots) * 4;
  plan->lds_slot_off = off;
  off += ((size_t(group_cap) * 2 + 15) & ~size_t(15));
  plan->lds_bytes = off;
  return off + 256 <= size_t(kLdsBudget);  // 256 B head-room for the static scan scratch
}

// One workgroup builds the dictionary of one (group, order): stage the group's keys in LDS,
// insert every occurrence into an open-addressing table whose words are fingerprint:position,
// number the occupied slots densely, and write each occurrence's offset id.
template <typename KeyT>
__device__ __forceinline__ void dictionary_block(const DictArgs& a, int g, int n,
                                                 unsigned char* smem, int* scan_scratch) {
  const Problem& pb = a.pb;
  const int nt = blockDim.x, tid = threadIdx.x;
  KeyT* skeys = reinterpret_cast<KeyT*>(smem);
  uint32_t* table = reinterpret_cast<uint32_t*>(smem + a.lds_table_off);
  uint16_t* slot_of = reinterpret_cast<uint16_t*>(smem + a.lds_slot_off);
  const uint32_t mask = uint32_t(a.table_slots) - 1u;
  const KeyT* gkeys = reinterpret_cast<const KeyT*>(a.ws.keys[n - 1]) + int64_t(g) * pb.group_cap;
  uint32_t* ginv = a.ws.inv[n - 1] + int64_t(g) * pb.group_cap;

  for (int i = tid; i < a.table_slots; i += nt) table[i] = kEmpty;

  // stage keys, compacted over the group's sequences (candidate first, then references)
  int count = 0;
  for (int j = 0; j <= pb.R; ++j) {
    const int len = (j == 0)
        ? clamped_len(pb.cand_len[g], pb.cand_stride, nullptr)
        : clamped_len(pb.ref_len[int64_t(g) * pb.R + j - 1], pb.ref_stride, nullptr);
    const int cnt = max(len - n + 1, 0);
    const int64_t off = (j == 0) ? 0 : pb.cand_stride + int64_t(j - 1) * pb.ref_stride;
    for (int p = tid; p < cnt; p += nt) skeys[count + p] = gkeys[off + p];
    count += cnt;
  }
  __syncthreads();

  for (int k = tid; k < count; k += nt) {
    const KeyT key = skeys[k];
    const uint32_t h = key_hash(key);
    const uint32_t fp = h >> 16;
    const uint32_t mine = (fp << 16) | uint32_t(k);
    uint32_t slot = h & mask;
    while (true) {
      uint32_t w = table[slot];
      if (w == kEmpty) {
        w = atomicCAS(&table[slot], kEmpty, mine);
        if (w == kEmpty) break;  // this occurrence now represents its n-gram
      }
      if ((w >> 16) == fp && key_eq(skeys[w & 0xFFFFu], key)) break;
      slot = (slot + 1) & mask;
    }
    slot_of[k] = uint16_t(slot);
  }
  __syncthreads();

  // dense ids: thread t numbers slots t, t+nt, ... (bank-conflict free); any bijection will do
  int occupied = 0;
  for (int sidx = tid; sidx < a.table_slots; sidx += nt) occupied += (table[sidx] != kEmpty);
  int U = 0;
  int id = block_exclusive_scan(occupied, scan_scratch, &U);
  for (int sidx = tid; sidx < a.table_slots; sidx += nt)
    if (table[sidx] != kEmpty) table[sidx] = uint32_t(id++);
  __syncthreads();

  const uint32_t gbase = uint32_t(int64_t(g) * pb.group_cap);
  count = 0;
  for (int j = 0; j <= pb.R; ++j) {
    const int len = (j == 0)
        ? clamped_len(pb.cand_len[g], pb.cand_stride, nullptr)
        : clamped_len(pb.ref_len[int64_t(g) * pb.R + j - 1], pb.ref_stride, nullptr);
    const int cnt = max(len - n + 1, 0);
    const int64_t off = (j == 0) ? 0 : pb.cand_stride + int64_t(j - 1) * pb.ref_stride;
    for (int p = tid; p < cnt; p += nt) ginv[off + p] = gbase + table[slot_of[count + p]];
    count += cnt;
  }
  if (tid == 0) a.distinct[int64_t(g) * pb.N + n - 1] = U;
}

__global__ __launch_bounds__(1024) void dictionary_kernel(DictArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int scan_scratch[17];
  const int g = blockIdx.x / a.pb.N;
  const int n = blockIdx.x % a.pb.N + 1;
  if (a.ws.wide[n - 1])
    dictionary_block<Key128>(a, g, n, smem, scan_scratch);
  else
    dictionary_block<uint64_t>(a, g, n, smem, scan_scratch);
}

hipError_t launch_dictionary(const Problem& pb, const GlobalWs& ws, const DictPlan& plan,
                             int32_t* distinct, hipStream_t s) {
  DictArgs a;
  a.pb = pb;
  a.ws = ws;
  a.distinct = distinct;
  a.table_slots = plan.table_slots;
  a.lds_table_off = uint32_t(plan.lds_table_off);
  a.lds_slot_off = uint32_t(plan.lds_slot_off);
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(dictionary_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize,
                                     int(plan.lds_bytes));
  if (e != hipSuccess) return e;
  const int64_t blocks = int64_t(pb.B) * pb.N;
  if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
  hipLaunchKernelGGL(dictionary_kernel, dim3(uint32_t(blocks)), dim3(plan.threads),
                     plan.lds_bytes, s, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------- count + clip

struct CountArgs {
  Problem pb;
  GlobalWs ws;
  StatPtrs st;
};

bool plan_count(int64_t group_cap, int64_t cand_stride, int64_t ref_stride, CountPlan* plan) {
  // reference counters are 16-bit fields (current | maximum) of one LDS word
  if (group_cap < 1 || ref_stride > 65535 || cand_stride > 0x7FFFFFFF) return false;
  plan->threads = group_cap > 2048 ? 1024 : (group_cap > 768 ? 512 : 256);
  plan->lds_bytes = size_t(group_cap) * 8;
  return plan->lds_bytes + 256 <= size_t(kLdsBudget);
}

// One workgroup per (group, order): histogram the candidate's ids and, reference by reference,
// the reference's ids over the group's dictionary range with LDS atomics; fold each reference
// into a running maximum; sum min(candidate, maximum).
__global__ __launch_bounds__(1024) void count_clip_kernel(CountArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int red_scratch[17];
  const Problem& pb = a.pb;
  const int nt = blockDim.x, tid = threadIdx.x;
  const int g = blockIdx.x / pb.N;
  const int n = blockIdx.x % pb.N + 1;
  const int cap = int(pb.group_cap);
  uint32_t* cand_cnt = reinterpret_cast<uint32_t*>(smem);
  uint32_t* ref_cnt = cand_cnt + cap;  // low 16 bits: current reference, high 16: maximum so far
  const uint32_t* ginv = a.ws.inv[n - 1] + int64_t(g) * pb.group_cap;
  const uint32_t gbase = uint32_t(int64_t(g) * pb.group_cap);
  const int U = min(max(a.st.distinct[int64_t(g) * pb.N + n - 1], 0), cap);

  for (int u = tid; u < U; u += nt) {
    cand_cnt[u] = 0;
    ref_cnt[u] = 0;
  }
  __syncthreads();

  const int c = clamped_len(pb.cand_len[g], pb.cand_stride, nullptr);
  const int ccnt = max(c - n + 1, 0);
  for (int p = tid; p < ccnt; p += nt) {
    const uint32_t id = ginv[p] - gbase;
    if (id < uint32_t(U)) atomicAdd(&cand_cnt[id], 1u);
  }
  for (int j = 0; j < pb.R; ++j) {
    const int len = clamped_len(pb.ref_len[int64_t(g) * pb.R + j], pb.ref_stride, nullptr);
    const int rcnt = max(len - n + 1, 0);
    const uint32_t* rinv = ginv + pb.cand_stride + int64_t(j) * pb.ref_stride;
    for (int p = tid; p < rcnt; p += nt) {
      const uint32_t id = rinv[p] - gbase;
      if (id < uint32_t(U)) atomicAdd(&ref_cnt[id], 1u);
    }
    __syncthreads();
    if (j + 1 < pb.R) {
      for (int u = tid; u < U; u += nt) {
        const uint32_t w = ref_cnt[u];
        const uint32_t cur = w & 0xFFFFu, mx = w >> 16;
        ref_cnt[u] = max(cur, mx) << 16;
      }
      __syncthreads();
    }
  }
  int part = 0;
  for (int u = tid; u < U; u += nt) {
    const uint32_t w = ref_cnt[u];
    const uint32_t mx = max(w & 0xFFFFu, w >> 16);
    part += int(min(cand_cnt[u], mx));
  }
  const int clipped = block_sum(part, red_scratch);
  if (tid == 0) {
    a.st.clipped[int64_t(g) * pb.N + n - 1] = clipped;
    a.st.total[int64_t(g) * pb.N + n - 1] = ccnt;
  }
}

hipError_t launch_count_clip(const Problem& pb, const GlobalWs& ws, const CountPlan& plan,
                             const StatPtrs& st, hipStream_t s) {
  CountArgs a;
  a.pb = pb;
  a.ws = ws;
  a.st = st;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(count_clip_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize,
                                     int(plan.lds_bytes));
  if (e != hipSuccess) return e;
  const int64_t blocks = int64_t(pb.B) * pb.N;
  if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
  hipLaunchKernelGGL(count_clip_kernel, dim3(uint32_t(blocks)), dim3(plan.threads),
                     plan.lds_bytes, s, a);
  return hipGetLastError();
}

}  // namespace tb
