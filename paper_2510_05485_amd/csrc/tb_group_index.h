// Where the sequences of a sentence group start inside the group's compact slot range.
// Shared by the GLOBAL path's kernels (pack, dictionary, count/clip, LDS and partitioned).
#pragma once

#include "tb_common.h"

namespace tb {

// Clamped length of sequence j of group g (j = 0: candidate, j >= 1: reference j-1).
// A reference beyond the candidate's reference count has no n-grams: length 0.
__device__ __forceinline__ int seq_len(const Problem& pb, int g, int j) {
  if (j == 0) return clamped_len(pb.cand_len[g], pb.cand_stride, nullptr);
  const RefRows rr = ref_rows(pb, g);
  if (j > rr.used) return 0;
  return clamped_len(pb.ref_len[rr.row0 + j - 1], pb.ref_stride, nullptr);
}

// Where each sequence of group g starts inside the group's compact slot range for order n.
// With at most 64 sequences per group every wavefront loads all lengths with one vector load
// (lane j takes sequence j) and prefix-sums the n-gram counts with cross-lane shuffles, so no
// chain of dependent scalar loads sits in front of the kernel's real work.  Larger groups fall
// back to a loop.  Must be constructed and queried in wave-uniform control flow.
class GroupIndex {
 public:
  // Issues the loads of the lengths and nothing else: the values are first touched by
  // set_order(), so loads that the caller issues in between are in flight together with them.
  __device__ __forceinline__ GroupIndex(const Problem& pb, int g)
      : pb_(pb), g_(g), n_(1), fast_(pb.R < kWave), raw_(0), used_(pb.R), incl_(0) {
    if (fast_) load_raw();
  }
  __device__ __forceinline__ GroupIndex(const Problem& pb, int g, int n) : GroupIndex(pb, g) {
    set_order(n);
  }
  // For kernels that are only launched with fewer than 64 sequences per group: no loop fallback.
  struct WaveOnly {};
  __device__ __forceinline__ GroupIndex(const Problem& pb, int g, WaveOnly)
      : pb_(pb), g_(g), n_(1), fast_(true), raw_(0), used_(pb.R), incl_(0) {
    load_raw();
  }
  __device__ __forceinline__ void set_order(int n) {
    n_ = n;
    if (fast_) {
      const int lane = threadIdx.x & (kWave - 1);
      // (readfirstlane keeps the two strides in scalar registers: a select between the two
      // fields would otherwise be turned into one vector load from a selected address)
      const int cs = __builtin_amdgcn_readfirstlane(int(min(pb_.cand_stride, int64_t(1) << 30)));
      const int rs = __builtin_amdgcn_readfirstlane(int(min(pb_.ref_stride, int64_t(1) << 30)));
      const int len = lane <= used_ ? clamped_len(raw_, lane == 0 ? cs : rs, nullptr) : 0;
      incl_ = wave_inclusive_scan(max(len - n + 1, 0));
    }
  }
  // First slot of sequence j (0 = candidate); j = R + 1 gives the group's n-gram count.
  __device__ __forceinline__ int start(int j) const {
    if (j == 0) return 0;
    if (fast_) return lane_value(incl_, j - 1);
    int s = 0;
    for (int jj = 0; jj < j; ++jj) s += max(seq_len(pb_, g_, jj) - n_ + 1, 0);
    return s;
  }
  // Lane j <= R: one past the last slot of sequence j.  Only when the group has < 64 sequences.
  __device__ __forceinline__ int end_in_lane() const { return incl_; }
  // Lane j <= R: the clamped length of sequence j (0 for a reference not in use); and the number
  // of references in use.  Only when the group has < 64 sequences.
  __device__ __forceinline__ int length_in_lane() const {
    const int lane = threadIdx.x & (kWave - 1);
    const int cs = __builtin_amdgcn_readfirstlane(int(min(pb_.cand_stride, int64_t(1) << 30)));
    const int rs = __builtin_amdgcn_readfirstlane(int(min(pb_.ref_stride, int64_t(1) << 30)));
    return lane <= used_ ? clamped_len(raw_, lane == 0 ? cs : rs, nullptr) : 0;
  }
  __device__ __forceinline__ int refs_in_use() const { return used_; }

 private:
  // lane j <= R: the stored length of sequence j; other lanes: 0
  __device__ __forceinline__ void load_raw() {
    const int lane = threadIdx.x & (kWave - 1);
    const RefRows rr = ref_rows(pb_, g_);
    // (two separate values and a select: an if / else over one variable would make the compiler
    // wait for the vector load where the branches join)
    const int raw_cand = uniform_load(pb_.cand_len, g_);
    int raw_ref = 0;
    if (lane >= 1 && lane <= ref_rows_readable(pb_, rr)) raw_ref = pb_.ref_len[rr.row0 + lane - 1];
    raw_ = lane == 0 ? raw_cand : raw_ref;
    used_ = rr.used;
  }
  const Problem& pb_;
  int g_, n_;
  bool fast_;
  int raw_, used_, incl_;
};

}  // namespace tb
