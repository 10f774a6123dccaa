// Shared device-side helpers and argument blocks of the gfx950 BLEU kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tensorbleu.h"

namespace tb {

constexpr int kWave = 64;                 // CDNA wavefront width
constexpr uint32_t kEmpty = 0xFFFFFFFFu;  // empty hash-table word
constexpr int kLdsBudget = 160 * 1024;    // LDS per compute unit (and per workgroup) on gfx950

// 128-bit key for orders whose n*bits exceeds 64.  lo holds the least significant 64 bits.
struct __attribute__((aligned(16))) Key128 {
  uint64_t lo, hi;
};

__device__ __forceinline__ bool key_eq(uint64_t a, uint64_t b) { return a == b; }
__device__ __forceinline__ bool key_eq(const Key128& a, const Key128& b) {
  return a.lo == b.lo && a.hi == b.hi;
}

// 32-bit avalanche of a packed key; the low bits pick the slot, the top 16 are the fingerprint.
__device__ __forceinline__ uint32_t fmix(uint32_t h) {
  h ^= h >> 16;
  h *= 0x7FEB352Du;
  h ^= h >> 15;
  h *= 0x846CA68Bu;
  h ^= h >> 16;
  return h;
}
__device__ __forceinline__ uint32_t key_hash(uint64_t k) {
  uint32_t lo = uint32_t(k), hi = uint32_t(k >> 32);
  return fmix(lo * 0x9E3779B1u ^ fmix(hi + 0x85EBCA77u));
}
__device__ __forceinline__ uint32_t key_hash(const Key128& k) {
  return fmix(key_hash(k.lo) ^ (key_hash(k.hi) * 0xC2B2AE3Du + 0x27D4EB2Fu));
}

// Cross-lane data movement inside the VALU (DPP): no LDS round trip, unlike ds_bpermute-based
// shuffles.  Lanes whose source is masked off or out of range receive 0.
template <int kCtrl, int kRowMask, int kBankMask>
__device__ __forceinline__ int dpp_or_zero(int v) {
  return __builtin_amdgcn_update_dpp(0, v, kCtrl, kRowMask, kBankMask, false);
}

// Inclusive prefix sum across the 64 lanes of a wavefront.  All 64 lanes must be active.
// Row-local shifts build the scan inside each row of 16 lanes; two row broadcasts (lane 15 of a
// row into the next row, lane 31 into the upper half) carry it across rows.
__device__ __forceinline__ int wave_inclusive_scan(int v) {
  int x = v;
  x += dpp_or_zero<0x111, 0xf, 0xf>(v);  // row_shr:1
  x += dpp_or_zero<0x112, 0xf, 0xf>(v);  // row_shr:2
  x += dpp_or_zero<0x113, 0xf, 0xf>(v);  // row_shr:3
  x += dpp_or_zero<0x114, 0xf, 0xe>(x);  // row_shr:4, lanes 4..15 of each row
  x += dpp_or_zero<0x118, 0xf, 0xc>(x);  // row_shr:8, lanes 8..15 of each row
  x += dpp_or_zero<0x142, 0xa, 0xf>(x);  // row_bcast:15 into rows 1 and 3
  x += dpp_or_zero<0x143, 0xc, 0xf>(x);  // row_bcast:31 into rows 2 and 3
  return x;
}

// Sum over the wavefront, returned in every lane (wave-uniform).  All 64 lanes must be active.
__device__ __forceinline__ int wave_sum(int v) {
  return __builtin_amdgcn_readlane(wave_inclusive_scan(v), kWave - 1);
}

// Value of `v` in lane `src` (wave-uniform index), as a scalar.
__device__ __forceinline__ int lane_value(int v, int src) {
  return __builtin_amdgcn_readlane(v, src);
}

// Exclusive scan of one int per thread over the workgroup (up to 1024 threads); also returns
// the workgroup total.  `scratch` needs 17 ints of LDS.  Contains two barriers.
__device__ __forceinline__ int block_exclusive_scan(int v, int* scratch, int* total) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int nwaves = (blockDim.x + kWave - 1) / kWave;
  int incl = wave_inclusive_scan(v);
  if (lane == kWave - 1) scratch[wave] = incl;
  __syncthreads();
  if (wave == 0) {
    int w = (lane < nwaves) ? scratch[lane] : 0;
    int wi = wave_inclusive_scan(w);
    if (lane < nwaves) scratch[lane] = wi - w;
    if (lane == nwaves - 1) scratch[16] = wi;
  }
  __syncthreads();
  *total = scratch[16];
  return scratch[wave] + incl - v;
}

// Dense ids for the table entries this thread created (any bijection onto 0..U-1 is a valid
// dictionary): every wavefront reserves a block of ids with one LDS atomic, lanes take their
// share in lane order.  Returns the first id of this thread.  All 64 lanes must be active.
__device__ __forceinline__ uint32_t reserve_ids(int created, int* next_id) {
  const int incl = wave_inclusive_scan(created);
  const int total = lane_value(incl, kWave - 1);
  int base = 0;
  if ((threadIdx.x & (kWave - 1)) == 0 && total) base = atomicAdd(next_id, total);
  return uint32_t(lane_value(base, 0) + incl - created);
}

// Sum of one int per thread over the workgroup; result valid in every thread.
// `scratch` needs 17 ints of LDS.  Contains two barriers.
__device__ __forceinline__ int block_sum(int v, int* scratch) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int nwaves = (blockDim.x + kWave - 1) / kWave;
  int s = wave_sum(v);
  if (lane == 0) scratch[wave] = s;
  __syncthreads();
  if (wave == 0) {
    int w = (lane < nwaves) ? scratch[lane] : 0;
    w = wave_sum(w);
    if (lane == 0) scratch[16] = w;
  }
  __syncthreads();
  return scratch[16];
}

// Problem description handed to every kernel (device pointers + shapes).
struct Problem {
  const void* cand;      // int32 or int64 token ids (tok64)
  const int32_t* cand_len;
  const void* refs;
  const int32_t* ref_len;
  int64_t cand_stride, ref_stride;
  int64_t group_cap;  // cand_stride + R * ref_stride
  int32_t B, R, N;
  int32_t bits;       // ceil(log2(vocab)), >= 1
  int32_t vocab;
  int32_t tok64;      // token ids are int64
  const int32_t* ref_count;  // per-candidate number of references in use, or null (= R)
  const int32_t* ref_offsets;  // CSR reference lists: candidate g owns the reference rows
                               // ref_offsets[g] .. ref_offsets[g + 1] - 1 (at most R); or null:
                               // the fixed layout, rows g * R .. g * R + R - 1
  int64_t ref_rows;   // CSR: number of reference rows (rows beyond are never touched)
  int32_t* status;    // may be null
};

// Token `idx` of a token array.  An int64 id that does not fit int32 becomes -1, which every
// range check reports.
__device__ __forceinline__ int32_t load_token(const void* base, int64_t idx, int tok64) {
  if (tok64) {
    const long long v = static_cast<const long long*>(base)[idx];
    return (v < 0 || v > 0x7FFFFFFFll) ? -1 : int32_t(v);
  }
  return static_cast<const int32_t*>(base)[idx];
}

// A load at an address that is the same in every lane, from memory that no workgroup of the
// RUNNING KERNEL writes (an input array, or what an earlier launch of the call left): read
// through the constant address space, so that it goes through the scalar cache -- no
// vector-memory round trip with a wait for every other outstanding vector load of the wavefront
// behind it.  (The scalar cache is invalidated when a kernel starts, not while it runs.)
__device__ __forceinline__ int32_t uniform_load(const int32_t* p, int64_t i) {
  typedef const int32_t __attribute__((address_space(4))) * constant_ptr;
  return *(constant_ptr)(p + i);
}

// Where candidate g's references are: rows row0 .. row0 + used - 1 of `refs` and `ref_len`.
// Fixed layout: row0 = g * R, used = R or the caller's count clamped into [1, R].  CSR: the span
// the offsets give, clamped into the reference rows that exist and to at most R rows (a candidate
// may then have no reference at all: used = 0).  `flag`: report a clamped count (set by one thread
// per group only).
struct RefRows {
  int64_t row0;
  int used;
};
__device__ __forceinline__ RefRows ref_rows(const Problem& pb, int g, bool flag = false) {
  RefRows r;
  if (pb.ref_offsets) {
    const int64_t b = uniform_load(pb.ref_offsets, g), e = uniform_load(pb.ref_offsets, g + 1);
    const int64_t row0 = min(max(b, int64_t(0)), max(pb.ref_rows, int64_t(0)));
    const int64_t used = min(min(max(e - row0, int64_t(0)), int64_t(pb.R)), pb.ref_rows - row0);
    if (flag && (row0 != b || used != e - b || used < 1) && pb.status)
      atomicOr(pb.status, TB_DEV_LENGTH_RANGE);
    r.row0 = row0;
    r.used = int(max(used, int64_t(0)));
    return r;
  }
  r.row0 = int64_t(g) * pb.R;
  r.used = pb.R;
  if (pb.ref_count) {
    const int c = uniform_load(pb.ref_count, g);
    if (flag && (c < 1 || c > pb.R) && pb.status) atomicOr(pb.status, TB_DEV_LENGTH_RANGE);
    r.used = min(max(c, 1), pb.R);
  }
  return r;
}
__device__ __forceinline__ int refs_used(const Problem& pb, int g, bool flag = false) {
  return ref_rows(pb, g, flag).used;
}
// Rows of `ref_len` that may be read for candidate g without knowing `used`: all R in the fixed
// layout (they exist), only the candidate's own with CSR.
__device__ __forceinline__ int ref_rows_readable(const Problem& pb, const RefRows& r) {
  return pb.ref_offsets ? r.used : pb.R;
}

// Length of a row as the kernels use it: clamped into [0, stride].
__device__ __forceinline__ int clamped_len(int len, int64_t stride, int32_t* status) {
  if (len < 0 || len > stride) {
    if (status) atomicOr(status, TB_DEV_LENGTH_RANGE);
    len = len < 0 ? 0 : int(stride);
  }
  return len;
}

struct ScoreParams {
  float w[8];
  int32_t N;
  int32_t smoothing;
  float param;
  int32_t out_bf16;  // scores are stored as bfloat16 (fp32 rounded to nearest even) instead of fp32
};

}  // namespace tb
