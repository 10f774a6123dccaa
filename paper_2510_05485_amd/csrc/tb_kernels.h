// Host-side launch interface between the C-ABI dispatcher and the kernel translation units.
#pragma once

#include "tb_common.h"

namespace tb {

// Raises a kernel's dynamic-LDS limit to `bytes` (hipFuncSetAttribute) unless an earlier launch
// on the same device already raised it at least that far: the attribute call costs a few
// microseconds, which matters for calls that take ten.  `kernel` is the host-side kernel symbol.
hipError_t grant_dynamic_lds(const void* kernel, size_t bytes);

// Resolved pointers into the caller's workspace for the GLOBAL path.
struct GlobalWs {
  void* keys[8];      // packed keys per order, B * group_cap entries of 8 or 16 bytes
  uint32_t* inv[8];   // offset dictionary ids per order, B * group_cap entries
  int32_t wide[8];    // 1 when the order uses 16-byte keys
  void* tables;       // hash tables / counters in HBM (groups too large for LDS), or the
                      // per-partition dictionary sizes of the partitioned kernels, else null
  int32_t* overflow;  // [B], partitioned kernels only (else null): non-zero where a partition of
                      // the group received more distinct n-grams than it can number; the score
                      // kernels turn such a group's score into NaN
  int32_t* arrivals;  // [B], hierarchical-key kernels only (else null; the same words as
                      // `overflow`): how many of a group's count workgroups have finished; the
                      // dictionary kernel zeroes it, and in a whole call the last count workgroup
                      // to arrive scores the sentence
};

// Integer statistics (either the caller's arrays or workspace scratch; never null).
struct StatPtrs {
  int32_t* clipped;   // [B, N]
  int32_t* total;     // [B, N]
  int32_t* closest;   // [B]
  int32_t* distinct;  // [B, N]
  int64_t* corpus;    // [2N+2]
};

// Launch shape shared by the dictionary and count/clip kernels: every thread keeps up to
// `items` of its group's n-grams in registers (threads * items >= group_cap).
struct DictPlan {
  int threads;          // workgroup size (256, 512 or 1024)
  int items;            // register-resident n-grams per thread: 2, 4, 6, 8 or 12
  int narrow_orders[8]; // orders with 8-byte keys, and how many
  int n_narrow;
  int slot32_mask;      // bit n: order n's keys fit 32 bits (4-byte table entries, 2x the slots)
  int narrow_slots;     // hash-table slots (power of two, >= 4/3 group_cap), 8-byte entries
  size_t narrow_lds;
  int wide_orders[8];   // orders with 16-byte keys
  int n_wide;
  int wide_slots;       // 4-byte tag:position entries
  int wide_compact;     // 1: keys within 64 + 18 bits, only their low halves are staged in LDS
  size_t wide_lds, wide_table_off;
};
struct CountPlan {
  int threads, items;
  int fields;   // 1: one 16-bit LDS field per sequence (count_fields_kernel); 0: pair phases
  int words;    // 32-bit words per dictionary entry in the fields kernel
  size_t lds_bytes;
};
struct FusedPlan {
  int threads;         // workgroup size
  int items;           // token positions staged per thread: 2, 4, 6, 8 or 12
  int table_slots;     // power of two >= 4/3 * cand_stride (larger when LDS allows)
  int words;           // 32-bit counter words per id (two 16-bit sequence fields each)
  int tok_bytes;       // staged tokens are 2 bytes when bits <= 16, else 4
  int list_per_wave;   // work-list entries reserved per wavefront (multiple of 64)
  size_t lds_bytes, off_ids, off_cnt, off_cstate, off_tok, off_list;
};

// Groups within one LDS table whose (prefix id, last token) keys fit 31 bits: one workgroup per
// group builds the dictionaries of all orders on hierarchical 32-bit keys, and one workgroup per
// group (or per share of its orders) counts and clips all of them at once.
struct HierPlan {
  int threads, items;        // workgroup size; token positions / slots per thread
  int table_slots;           // power of two > group_cap, 4-byte entries
  size_t dict_lds;
  int words;                 // count/clip: 32-bit words of 16-bit fields per entry
  int count_threads, count_rows;  // count/clip: workgroup size; 16-byte id requests per thread
  int count_pairs_fit;       // count/clip: the counters of two orders fit one workgroup's LDS
};
bool plan_hier(int64_t group_cap, int64_t cand_stride, int64_t ref_stride, int R, int N, int bits,
               HierPlan* plan);
// cand_distinct [B, N]: written by the dictionary pass, read by the count/clip pass
hipError_t launch_hier_dictionary(const Problem& pb, const GlobalWs& ws, const HierPlan& plan,
                                  const StatPtrs& st, int32_t* cand_distinct, hipStream_t s);
// rouge_overlap != null: ROUGE-N instead -- only order N is counted, and overlap[B, R] receives
// per reference the sum over n-grams of min(candidate count, the reference's count)
// tail != null (BLEU only): the last workgroup of a group to finish also computes what the
// sentence score kernel computes (closest reference length, Section 3.4's score into tail->out),
// which then is not to be launched; needs ws.arrivals zeroed by the dictionary pass
struct ScoreTail {
  ScoreParams sp;
  void* out;  // [B] fp32 or bfloat16 (sp.out_bf16)
};
hipError_t launch_hier_count_clip(const Problem& pb, const GlobalWs& ws, const HierPlan& plan,
                                  const StatPtrs& st, const int32_t* cand_distinct,
                                  hipStream_t s, int32_t* rouge_overlap = nullptr,
                                  const ScoreTail* tail = nullptr);

// Groups beyond the LDS plans: table and counters live in the workspace.
struct BigPlan {
  int64_t slots;          // hash-table slots per (group, order): power of two >= 2 * group_cap
  int64_t table_entries;  // slots + padding, 8 bytes each
};
// Groups of up to 2 097 152 n-gram slots beyond the LDS plans: P workgroups per (group, order),
// each with the dictionary entries / counters of one hash partition in LDS.
struct PartPlan {
  int log2_parts;     // P = 1 << log2_parts workgroups per (group, order), 2 .. 512
  int id_cap;         // ids a partition may hand out
  int words;          // count/clip: 32-bit counter words per id
  int refs_per_pass;  // count/clip: 0 = every sequence has its field; else references per pass
  int fields_per_word;  // 2: 16-bit counters, 1: 32-bit (a stride above 65 535)
  int64_t id_stride;  // id range per group: max(group_cap, P * id_cap)
  size_t dict_lds, count_lds;
  int count_in_dictionary;  // the counter fields of a partition fit the dictionary table's LDS
};
bool plan_part(int64_t group_cap, int64_t cand_stride, int64_t ref_stride, int R, int N,
               const int32_t* key_bytes, PartPlan* plan);
// bytes the partitioned kernels need at GlobalWs::tables
size_t part_workspace_bytes(int64_t B, int N, int64_t group_cap, const PartPlan& plan);
// whole_call: the count/clip pass follows at once and nobody else reads the id array, so ids are
// stored only where a later order's keys are derived from them and, if
// plan.count_in_dictionary, the dictionary kernel also does the count/clip pass's work, which is
// then not to be launched.  from_tokens: pb.cand / pb.refs are set and the keys are built from
// them; otherwise they are read from ws.keys as the pack kernel left them
hipError_t launch_part_dictionary(const Problem& pb, const GlobalWs& ws, const PartPlan& plan,
                                  const StatPtrs& st, bool whole_call, bool from_tokens,
                                  hipStream_t s);
// rouge_overlap != null: ROUGE-N instead, as for launch_hier_count_clip
hipError_t launch_part_count_clip(const Problem& pb, const GlobalWs& ws, const PartPlan& plan,
                                  const StatPtrs& st, hipStream_t s,
                                  int32_t* rouge_overlap = nullptr);

bool plan_big(int64_t group_cap, int N, BigPlan* plan);
hipError_t launch_big_dictionary(const Problem& pb, const GlobalWs& ws, const BigPlan& plan,
                                 const StatPtrs& st, hipStream_t s);
// rouge_overlap != null: ROUGE-N instead, as for launch_hier_count_clip
hipError_t launch_big_count_clip(const Problem& pb, const GlobalWs& ws, const BigPlan& plan,
                                 const StatPtrs& st, hipStream_t s,
                                 int32_t* rouge_overlap = nullptr);

bool plan_dictionary(int64_t group_cap, const int32_t* key_bytes, int N, int bits,
                     DictPlan* plan);
bool plan_count(int64_t group_cap, int64_t cand_stride, int64_t ref_stride, int R,
                CountPlan* plan);
bool plan_fused(int64_t cand_stride, int64_t ref_stride, int R, int N, int bits,
                FusedPlan* plan);

hipError_t launch_pack(const Problem& pb, const GlobalWs& ws, hipStream_t s);
hipError_t launch_dictionary(const Problem& pb, const GlobalWs& ws, const DictPlan& plan,
                             int32_t* distinct, hipStream_t s);
hipError_t launch_count_clip(const Problem& pb, const GlobalWs& ws, const CountPlan& plan,
                             const StatPtrs& st, hipStream_t s);
// sentence_scores: out_bleu[B] per-sentence scores; corpus_sums: fill st.corpus;
// corpus_score: additionally write the corpus score to out_bleu[0] (not with sentence_scores).
// overflow: GlobalWs::overflow or null
hipError_t launch_finalize(const Problem& pb, const StatPtrs& st, const ScoreParams& sp,
                           bool sentence_scores, bool corpus_sums, bool corpus_score,
                           void* out_bleu, hipStream_t s, const int32_t* overflow = nullptr);
// ROUGE-N scores from overlap counts (GLOBAL path): precision, recall, F of the best reference.
struct RougeOut;
hipError_t launch_rouge_finalize(const Problem& pb, const ScoreParams& sp, const int32_t* overlap,
                                 const RougeOut& out, hipStream_t s);
// ROUGE-N outputs of the fused kernel (order n = pb.N): see tensorrouge_n.
struct RougeOut {
  void* prf;         // [B, 3] fp32 or bfloat16 (ScoreParams::out_bf16)
  int32_t* overlap;  // [B, R] or null
  int32_t* best;     // [B] or null
  float beta2;
};
// rouge == null: BLEU (statistics and, if out_bleu_or_null, per-sentence scores).
hipError_t launch_fused(const Problem& pb, const FusedPlan& plan, const StatPtrs& st,
                        const ScoreParams& sp, void* out_bleu_or_null, hipStream_t s,
                        const RougeOut* rouge = nullptr);

}  // namespace tb
