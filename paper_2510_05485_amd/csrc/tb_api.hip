// C-ABI dispatcher: argument validation, workspace carving, path selection, kernel launches.
// Nothing here allocates, synchronises or keeps state between calls.
#include <atomic>
#include <cstring>
#include <mutex>

#include "tb_kernels.h"

// Scratch memory of tensorbleu_sentence_static: a device array that is part of the loaded code
// object, so that entry point never allocates.  Every GPU the library runs on holds its own copy
// at its own address until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; kernels and copies get the address that call returns, never the name.
constexpr size_t kStaticScratchBytes = size_t(4) << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace tb {

// Process-wide state of the library (besides the static scratch buffer's address): which kernels already had their dynamic-LDS limit
// raised on which device (a cache of an idempotent runtime setting, invisible to callers).
hipError_t grant_dynamic_lds(const void* kernel, size_t bytes) {
  struct Grant {
    const void* kernel;
    int device;
    std::atomic<size_t> bytes;
  };
  constexpr int kMaxGrants = 512;
  static Grant grants[kMaxGrants];
  static std::atomic<int> count{0};
  static std::mutex mu;
  int device = 0;
  hipError_t e = hipGetDevice(&device);
  if (e != hipSuccess) return e;
  // lock-free look-up of what earlier calls published (entries are immutable once counted,
  // except `bytes`, which only grows under the lock; a stale smaller value just takes the lock)
  const int seen = count.load(std::memory_order_acquire);
  for (int i = 0; i < seen; ++i)
    if (grants[i].kernel == kernel && grants[i].device == device &&
        grants[i].bytes.load(std::memory_order_relaxed) >= bytes)
      return hipSuccess;
  std::lock_guard<std::mutex> lock(mu);
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, int(bytes));
  if (e != hipSuccess) return e;
  const int n = count.load(std::memory_order_relaxed);
  for (int i = 0; i < n; ++i)
    if (grants[i].kernel == kernel && grants[i].device == device) {
      if (grants[i].bytes.load(std::memory_order_relaxed) < bytes)
        grants[i].bytes.store(bytes, std::memory_order_relaxed);
      return hipSuccess;
    }
  if (n < kMaxGrants) {  // a full table only costs the attribute call again next time
    grants[n].kernel = kernel;
    grants[n].device = device;
    grants[n].bytes.store(bytes, std::memory_order_relaxed);
    count.store(n + 1, std::memory_order_release);
  }
  return hipSuccess;
}

}  // namespace tb

namespace {

using namespace tb;

// Device address of `scratch` on the current device: looked up once per device (with that device
// current) and kept.
hipError_t static_scratch_address(void** out) {
  constexpr int kMaxDevices = 64;
  static void* address[kMaxDevices];
  static std::atomic<bool> known[kMaxDevices];
  static std::mutex mu;
  int device = 0;
  hipError_t e = hipGetDevice(&device);
  if (e != hipSuccess) return e;
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  if (!known[device].load(std::memory_order_acquire)) {
    std::lock_guard<std::mutex> lock(mu);
    if (!known[device].load(std::memory_order_relaxed)) {
      void* ptr = nullptr;
      e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
      if (e != hipSuccess) return e;
      if (!ptr || (reinterpret_cast<uintptr_t>(ptr) & 255u)) return hipErrorInvalidSymbol;
      address[device] = ptr;
      known[device].store(true, std::memory_order_release);
    }
  }
  *out = address[device];
  return hipSuccess;
}

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) & ~(kAlign - 1); }

int ceil_log2(int32_t v) {
  int b = 0;
  while ((int64_t(1) << b) < int64_t(v)) ++b;
  return b < 1 ? 1 : b;
}

bool config_ok(const tb_config_t* cfg) {
  if (!cfg) return false;
  if (cfg->max_n < 1 || cfg->max_n > 8) return false;
  if (cfg->vocab_size < 1) return false;
  if (cfg->smoothing < TB_SMOOTH_NONE || cfg->smoothing > TB_SMOOTH_EXP) return false;
  if (cfg->force_path < TB_PATH_AUTO || cfg->force_path > TB_PATH_GLOBAL) return false;
  if (cfg->token_bytes != 0 && cfg->token_bytes != 4 && cfg->token_bytes != 8) return false;
  if (cfg->score_bytes != 0 && cfg->score_bytes != 4 && cfg->score_bytes != 2) return false;
  if (cfg->ref_offsets && (cfg->ref_count || cfg->ref_rows < 0)) return false;
  return true;
}

struct Plans {
  tb_layout_t layout;
  DictPlan dict;
  CountPlan count;
  FusedPlan fused;
  BigPlan big;
  PartPlan part;
  HierPlan hier;
  size_t overflow_off;
  bool use_hier;  // GLOBAL path on the hierarchical-key kernels (a subset of the LDS shapes)
  bool use_part;  // GLOBAL path with P workgroups per (group, order), tables split over their LDS
  bool use_big;   // GLOBAL path with tables in the workspace (group too large for that, too)
};

// Everything that depends on shapes only.  Returns TB_OK or an error.
int make_plans(int32_t B, int32_t R, int64_t cand_stride, int64_t ref_stride,
               const tb_config_t* cfg, Plans* p) {
  if (!config_ok(cfg) || B < 0 || R < 1 || cand_stride < 1 || ref_stride < 1)
    return TB_ERR_INVALID_ARG;
  tb_layout_t& L = p->layout;
  std::memset(&L, 0, sizeof(L));
  const int N = cfg->max_n;
  L.bits = ceil_log2(cfg->vocab_size);
  for (int n = 1; n <= 8; ++n) L.key_bytes[n - 1] = (n * L.bits > 64) ? 16 : 8;
  if (cand_stride > (int64_t(1) << 30) || ref_stride > (int64_t(1) << 30) || R > (1 << 20))
    return TB_ERR_UNSUPPORTED;
  L.group_cap = cand_stride + int64_t(R) * ref_stride;
  // group_cap can reach 2^50 here: bound it first so that the product below cannot overflow
  const bool global_n = N * L.bits <= 128;  // the GLOBAL path packs whole n-grams into keys
  // one LDS table per group: the hierarchical-key kernels where their plan fits, else the
  // packed-key ones
  // (cfg->workspace_tables: none of the LDS plans, tables in the workspace for every shape)
  const bool lds_allowed = global_n && !cfg->workspace_tables;
  p->use_hier =
      lds_allowed && plan_hier(L.group_cap, cand_stride, ref_stride, R, N, L.bits, &p->hier);
  const bool lds_ok = p->use_hier ||
                      (lds_allowed &&
                       plan_dictionary(L.group_cap, L.key_bytes, N, L.bits, &p->dict) &&
                       plan_count(L.group_cap, cand_stride, ref_stride, R, &p->count));
  p->use_part = lds_allowed && !lds_ok &&
                plan_part(L.group_cap, cand_stride, ref_stride, R, N, L.key_bytes, &p->part);
  p->use_big = global_n && !lds_ok && !p->use_part && plan_big(L.group_cap, N, &p->big);
  L.id_stride = p->use_part ? p->part.id_stride : L.group_cap;
  const bool ids_fit = L.id_stride < (int64_t(1) << 32) &&
                       int64_t(B) * L.id_stride < (int64_t(1) << 32);
  L.global_ok = ids_fit && (lds_ok || p->use_part || p->use_big);
  L.global_tables_in_hbm = p->use_big ? 1 : 0;
  L.global_partitions = p->use_part ? (1 << p->part.log2_parts) : 0;
  L.global_candidate_first = p->use_hier ? 1 : 0;
  L.fused_ok = plan_fused(cand_stride, ref_stride, R, N, L.bits, &p->fused);
  int path = cfg->force_path;
  if (path == TB_PATH_AUTO) path = L.fused_ok ? TB_PATH_FUSED : TB_PATH_GLOBAL;
  if (path == TB_PATH_FUSED && !L.fused_ok) return TB_ERR_UNSUPPORTED;
  if (path == TB_PATH_GLOBAL && !L.global_ok) return TB_ERR_UNSUPPORTED;
  L.path = path;

  size_t off = 0;
  const size_t bn = size_t(B) * N;
  L.clipped_off = off;  off = align_up(off + bn * 4);
  L.total_off = off;    off = align_up(off + bn * 4);
  L.closest_off = off;  off = align_up(off + size_t(B) * 4);
  L.distinct_off = off; off = align_up(off + bn * 4);
  L.cand_distinct_off = off; off = align_up(off + bn * 4);
  L.corpus_off = off;   off = align_up(off + 18 * 8);
  const size_t overflow_off = off;  // int32 [B]: groups whose partitioned dictionary overflowed
  off = align_up(off + size_t(B) * 4);
  p->overflow_off = overflow_off;
  if (path == TB_PATH_GLOBAL) {
    L.overlap_off = off;  // int32 [B, R]: ROUGE-N overlap counts (count pass -> score kernel)
    off = align_up(off + size_t(B) * size_t(R) * 4);
    const size_t slots = size_t(B) * size_t(L.group_cap);
    for (int n = 0; n < N; ++n) {
      L.keys_off[n] = off;
      off = align_up(off + slots * L.key_bytes[n]);
    }
    for (int n = 0; n < N; ++n) {
      L.inv_off[n] = off;
      off = align_up(off + slots * 4 + 16);  // 16 spare bytes: ids are also read four at a time
    }
    if (p->use_big) {
      L.tables_off = off;
      off = align_up(off + size_t(B) * N * size_t(p->big.table_entries) * 8);
    }
    if (p->use_part) {  // per partition: dictionary size, segment start; slots by partition
      L.tables_off = off;
      off = align_up(off + part_workspace_bytes(B, N, L.group_cap, p->part));
    }
  }
  L.bytes = off < kAlign ? kAlign : off;
  return TB_OK;
}

struct Call {
  Plans plans;
  Problem pb;
  GlobalWs ws;
  StatPtrs st;
  int32_t* cand_distinct;  // [B, N] in the workspace: dictionary pass -> count/clip pass
  ScoreParams sp;
  hipStream_t stream;
  bool want_corpus_stats;
};

int prepare(const void* cand, int64_t cand_stride, const int32_t* cand_len,
            const void* refs, int64_t ref_stride, const int32_t* ref_len, int32_t B, int32_t R,
            const tb_config_t* cfg, const tb_stats_t* stats, void* workspace,
            size_t workspace_bytes, void* hip_stream, bool need_tokens, int forced_path,
            Call* c) {
  tb_config_t local;
  if (cfg && forced_path != TB_PATH_AUTO) {
    local = *cfg;
    local.force_path = forced_path;
    cfg = &local;
  }
  int rc = make_plans(B, R, cand_stride, ref_stride, cfg, &c->plans);
  if (rc != TB_OK) return rc;
  if (B == 0) return TB_OK;
  if (!cand_len || !ref_len || (need_tokens && (!cand || !refs))) return TB_ERR_INVALID_ARG;
  const tb_layout_t& L = c->plans.layout;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) ||
      workspace_bytes < L.bytes)
    return TB_ERR_WORKSPACE;
  unsigned char* w = static_cast<unsigned char*>(workspace);
  Problem& pb = c->pb;
  pb.cand = cand;
  pb.cand_len = cand_len;
  pb.refs = refs;
  pb.ref_len = ref_len;
  pb.ref_count = cfg->ref_count;
  pb.ref_offsets = cfg->ref_offsets;
  pb.ref_rows = cfg->ref_offsets ? cfg->ref_rows : 0;
  pb.cand_stride = cand_stride;
  pb.ref_stride = ref_stride;
  pb.group_cap = L.group_cap;
  pb.B = B;
  pb.R = R;
  pb.N = cfg->max_n;
  pb.bits = L.bits;
  pb.vocab = cfg->vocab_size;
  pb.tok64 = cfg->token_bytes == 8;
  pb.status = stats ? stats->device_status : nullptr;
  for (int n = 0; n < 8; ++n) {
    c->ws.keys[n] = (L.path == TB_PATH_GLOBAL && n < pb.N) ? w + L.keys_off[n] : nullptr;
    c->ws.inv[n] = (L.path == TB_PATH_GLOBAL && n < pb.N)
                       ? reinterpret_cast<uint32_t*>(w + L.inv_off[n]) : nullptr;
    c->ws.wide[n] = L.key_bytes[n] == 16;
  }
  c->ws.tables = (L.path == TB_PATH_GLOBAL && (c->plans.use_big || c->plans.use_part))
                     ? w + L.tables_off : nullptr;
  c->ws.overflow = (L.path == TB_PATH_GLOBAL && c->plans.use_part)
                       ? reinterpret_cast<int32_t*>(w + c->plans.overflow_off) : nullptr;
  c->ws.arrivals = (L.path == TB_PATH_GLOBAL && c->plans.use_hier)
                       ? reinterpret_cast<int32_t*>(w + c->plans.overflow_off) : nullptr;
  StatPtrs& st = c->st;
  st.clipped = (stats && stats->clipped) ? stats->clipped
                                         : reinterpret_cast<int32_t*>(w + L.clipped_off);
  st.total = (stats && stats->total) ? stats->total : reinterpret_cast<int32_t*>(w + L.total_off);
  st.closest = (stats && stats->closest_ref_len) ? stats->closest_ref_len
                                                 : reinterpret_cast<int32_t*>(w + L.closest_off);
  st.distinct = (stats && stats->group_distinct) ? stats->group_distinct
                                                 : reinterpret_cast<int32_t*>(w + L.distinct_off);
  st.corpus = (stats && stats->corpus_stats) ? stats->corpus_stats
                                             : reinterpret_cast<int64_t*>(w + L.corpus_off);
  c->cand_distinct = reinterpret_cast<int32_t*>(w + L.cand_distinct_off);
  c->want_corpus_stats = stats && stats->corpus_stats;
  ScoreParams& sp = c->sp;
  sp.N = cfg->max_n;
  sp.smoothing = cfg->smoothing;
  sp.param = cfg->smooth_param;
  sp.out_bf16 = cfg->score_bytes == 2;
  bool all_zero = true;
  for (int n = 0; n < sp.N; ++n) all_zero = all_zero && cfg->weights[n] == 0.0f;
  for (int n = 0; n < 8; ++n)
    sp.w[n] = (n < sp.N) ? (all_zero ? 1.0f / float(sp.N) : cfg->weights[n]) : 0.0f;
  c->stream = static_cast<hipStream_t>(hip_stream);
  return TB_OK;
}

inline int hip_rc(hipError_t e) { return e == hipSuccess ? TB_OK : TB_ERR_HIP; }

// whole_call: the partitioned dictionary kernel then may take over the count/clip pass
// (counts_in_dictionary says whether it does) and stores only the ids that later orders need
bool counts_in_dictionary(const Call& c) {
  return c.plans.use_part && c.plans.part.count_in_dictionary;
}
// from_tokens: the caller handed over the token rows (c.pb.cand / c.pb.refs are set); the
// partitioned kernels then extract the n-grams themselves and the pack kernel need not have run
hipError_t run_dictionary(const Call& c, bool whole_call, bool from_tokens) {
  if (c.plans.use_hier)
    return launch_hier_dictionary(c.pb, c.ws, c.plans.hier, c.st, c.cand_distinct, c.stream);
  if (c.plans.use_part)
    return launch_part_dictionary(c.pb, c.ws, c.plans.part, c.st, whole_call, from_tokens,
                                  c.stream);
  return c.plans.use_big ? launch_big_dictionary(c.pb, c.ws, c.plans.big, c.st, c.stream)
                         : launch_dictionary(c.pb, c.ws, c.plans.dict, c.st.distinct, c.stream);
}
// tail: see launch_hier_count_clip (only for the hierarchical-key kernels)
hipError_t run_count_clip(const Call& c, const ScoreTail* tail = nullptr) {
  if (c.plans.use_hier)
    return launch_hier_count_clip(c.pb, c.ws, c.plans.hier, c.st, c.cand_distinct, c.stream,
                                  nullptr, tail);
  if (c.plans.use_part) return launch_part_count_clip(c.pb, c.ws, c.plans.part, c.st, c.stream);
  return c.plans.use_big ? launch_big_count_clip(c.pb, c.ws, c.plans.big, c.st, c.stream)
                         : launch_count_clip(c.pb, c.ws, c.plans.count, c.st, c.stream);
}

int run_all(const void* cand, int64_t cand_stride, const int32_t* cand_len,
            const void* refs, int64_t ref_stride, const int32_t* ref_len, int32_t B, int32_t R,
            const tb_config_t* cfg, void* out_bleu, const tb_stats_t* stats, void* workspace,
            size_t workspace_bytes, void* hip_stream, bool corpus) {
  Call c{};
  int rc = prepare(cand, cand_stride, cand_len, refs, ref_stride, ref_len, B, R, cfg, stats,
                   workspace, workspace_bytes, hip_stream, true, TB_PATH_AUTO, &c);
  if (rc != TB_OK || B == 0) return rc;
  if (!out_bleu) return TB_ERR_INVALID_ARG;
  if (c.plans.layout.path == TB_PATH_FUSED) {
    rc = hip_rc(launch_fused(c.pb, c.plans.fused, c.st, c.sp, corpus ? nullptr : out_bleu,
                             c.stream));
    if (rc != TB_OK) return rc;
    if (corpus || c.want_corpus_stats) {
      // per-sentence work is done by the fused kernel; only the batch sums remain
      Problem quiet = c.pb;
      quiet.status = nullptr;
      return hip_rc(launch_finalize(quiet, c.st, c.sp, false, true, corpus, out_bleu, c.stream));
    }
    return TB_OK;
  }
  if (!c.plans.use_part && (rc = hip_rc(launch_pack(c.pb, c.ws, c.stream))) != TB_OK) return rc;
  if ((rc = hip_rc(run_dictionary(c, true, true))) != TB_OK) return rc;
  if (c.plans.use_hier && !corpus && !c.want_corpus_stats) {
    // per-sentence scores only: the count kernel's last workgroup per group scores the sentence
    ScoreTail tail;
    tail.sp = c.sp;
    tail.out = out_bleu;
    return hip_rc(run_count_clip(c, &tail));
  }
  if (!counts_in_dictionary(c) && (rc = hip_rc(run_count_clip(c))) != TB_OK) return rc;
  return hip_rc(launch_finalize(c.pb, c.st, c.sp, !corpus, corpus || c.want_corpus_stats, corpus,
                                out_bleu, c.stream, c.ws.overflow));
}

}  // namespace

extern "C" {

size_t tensorbleu_workspace_bytes(int32_t B, int32_t R, int64_t cand_stride, int64_t ref_stride,
                                  const tb_config_t* cfg) {
  Plans p{};
  if (make_plans(B, R, cand_stride, ref_stride, cfg, &p) != TB_OK) return 0;
  return p.layout.bytes;
}

int tensorbleu_workspace_layout(int32_t B, int32_t R, int64_t cand_stride, int64_t ref_stride,
                                const tb_config_t* cfg, tb_layout_t* layout) {
  if (!layout) return TB_ERR_INVALID_ARG;
  Plans p{};  // zeroed: on an invalid argument the caller reads an all-zero layout
  int rc = make_plans(B, R, cand_stride, ref_stride, cfg, &p);
  *layout = p.layout;
  return rc;
}

int tensorbleu_sentence(const void* cand, int64_t cand_stride, const int32_t* cand_len,
                        const void* refs, int64_t ref_stride, const int32_t* ref_len,
                        int32_t B, int32_t R, const tb_config_t* cfg, void* out_bleu,
                        const tb_stats_t* stats, void* workspace, size_t workspace_bytes,
                        void* hip_stream) {
  return run_all(cand, cand_stride, cand_len, refs, ref_stride, ref_len, B, R, cfg, out_bleu,
                 stats, workspace, workspace_bytes, hip_stream, false);
}

int tensorbleu_corpus(const void* cand, int64_t cand_stride, const int32_t* cand_len,
                      const void* refs, int64_t ref_stride, const int32_t* ref_len, int32_t B,
                      int32_t R, const tb_config_t* cfg, void* out_bleu, const tb_stats_t* stats,
                      void* workspace, size_t workspace_bytes, void* hip_stream) {
  return run_all(cand, cand_stride, cand_len, refs, ref_stride, ref_len, B, R, cfg, out_bleu,
                 stats, workspace, workspace_bytes, hip_stream, true);
}

int tensorrouge_n(const void* cand, int64_t cand_stride, const int32_t* cand_len,
                  const void* refs, int64_t ref_stride, const int32_t* ref_len, int32_t B,
                  int32_t R, const tb_config_t* cfg, void* out_prf, int32_t* overlap,
                  int32_t* best_ref, const tb_stats_t* stats, void* workspace,
                  size_t workspace_bytes, void* hip_stream) {
  Call c{};
  int rc = prepare(cand, cand_stride, cand_len, refs, ref_stride, ref_len, B, R, cfg, stats,
                   workspace, workspace_bytes, hip_stream, true, TB_PATH_AUTO, &c);
  if (rc != TB_OK || B == 0) return rc;
  if (!out_prf) return TB_ERR_INVALID_ARG;
  const float beta = cfg->smooth_param > 0.0f ? cfg->smooth_param : 1.0f;
  RougeOut ro;
  ro.prf = out_prf;
  ro.overlap = overlap;
  ro.best = best_ref;
  ro.beta2 = float(double(beta) * double(beta));
  // the integer BLEU statistics of the run are scratch here: never the caller's arrays
  unsigned char* w = static_cast<unsigned char*>(workspace);
  const tb_layout_t& L = c.plans.layout;
  c.st.clipped = reinterpret_cast<int32_t*>(w + L.clipped_off);
  c.st.total = reinterpret_cast<int32_t*>(w + L.total_off);
  c.st.closest = reinterpret_cast<int32_t*>(w + L.closest_off);
  c.st.distinct = reinterpret_cast<int32_t*>(w + L.distinct_off);
  if (L.path == TB_PATH_FUSED)
    return hip_rc(launch_fused(c.pb, c.plans.fused, c.st, c.sp, nullptr, c.stream, &ro));
  // GLOBAL: pack and dictionary as for BLEU (the keys of order n build on the ids of the orders
  // below), then the count pass for order n alone, which also sums the per-reference overlaps
  // (the packed-key LDS count kernels are BLEU-only: such a shape is served with
  // cfg->workspace_tables set)
  if (!c.plans.use_hier && !c.plans.use_part && !c.plans.use_big) return TB_ERR_UNSUPPORTED;
  int32_t* ov = reinterpret_cast<int32_t*>(w + L.overlap_off);
  if (!c.plans.use_part && (rc = hip_rc(launch_pack(c.pb, c.ws, c.stream))) != TB_OK) return rc;
  if ((rc = hip_rc(run_dictionary(c, false, true))) != TB_OK) return rc;
  rc = hip_rc(c.plans.use_hier
                  ? launch_hier_count_clip(c.pb, c.ws, c.plans.hier, c.st, c.cand_distinct,
                                           c.stream, ov)
              : c.plans.use_part
                  ? launch_part_count_clip(c.pb, c.ws, c.plans.part, c.st, c.stream, ov)
                  : launch_big_count_clip(c.pb, c.ws, c.plans.big, c.st, c.stream, ov));
  if (rc != TB_OK) return rc;
  return hip_rc(launch_rouge_finalize(c.pb, c.sp, ov, ro, c.stream));
}

int tensorbleu_pack(const void* cand, int64_t cand_stride, const int32_t* cand_len,
                    const void* refs, int64_t ref_stride, const int32_t* ref_len, int32_t B,
                    int32_t R, const tb_config_t* cfg, const tb_stats_t* stats, void* workspace,
                    size_t workspace_bytes, void* hip_stream) {
  Call c{};
  int rc = prepare(cand, cand_stride, cand_len, refs, ref_stride, ref_len, B, R, cfg, stats,
                   workspace, workspace_bytes, hip_stream, true, TB_PATH_GLOBAL, &c);
  if (rc != TB_OK || B == 0) return rc;
  return hip_rc(launch_pack(c.pb, c.ws, c.stream));
}

int tensorbleu_dictionary(const int32_t* cand_len, const int32_t* ref_len, int64_t cand_stride,
                          int64_t ref_stride, int32_t B, int32_t R, const tb_config_t* cfg,
                          const tb_stats_t* stats, void* workspace, size_t workspace_bytes,
                          void* hip_stream) {
  Call c{};
  int rc = prepare(nullptr, cand_stride, cand_len, nullptr, ref_stride, ref_len, B, R, cfg, stats,
                   workspace, workspace_bytes, hip_stream, false, TB_PATH_GLOBAL, &c);
  if (rc != TB_OK || B == 0) return rc;
  return hip_rc(run_dictionary(c, false, false));
}

int tensorbleu_count_clip(const int32_t* cand_len, const int32_t* ref_len, int64_t cand_stride,
                          int64_t ref_stride, int32_t B, int32_t R, const tb_config_t* cfg,
                          const tb_stats_t* stats, void* workspace, size_t workspace_bytes,
                          void* hip_stream) {
  Call c{};
  int rc = prepare(nullptr, cand_stride, cand_len, nullptr, ref_stride, ref_len, B, R, cfg, stats,
                   workspace, workspace_bytes, hip_stream, false, TB_PATH_GLOBAL, &c);
  if (rc != TB_OK || B == 0) return rc;
  return hip_rc(run_count_clip(c));
}

int tensorbleu_finalize(const int32_t* cand_len, const int32_t* ref_len, int32_t B, int32_t R,
                        int64_t cand_stride, int64_t ref_stride, const tb_config_t* cfg,
                        int32_t corpus, void* out_bleu, const tb_stats_t* stats, void* workspace,
                        size_t workspace_bytes, void* hip_stream) {
  Call c{};
  int rc = prepare(nullptr, cand_stride, cand_len, nullptr, ref_stride, ref_len, B, R, cfg, stats,
                   workspace, workspace_bytes, hip_stream, false, TB_PATH_GLOBAL, &c);
  if (rc != TB_OK || B == 0) return rc;
  if (!out_bleu) return TB_ERR_INVALID_ARG;
  return hip_rc(launch_finalize(c.pb, c.st, c.sp, corpus == 0,
                                corpus != 0 || c.want_corpus_stats, corpus != 0, out_bleu,
                                c.stream, c.ws.overflow));
}

size_t tensorbleu_static_scratch_bytes(void) { return kStaticScratchBytes; }

int tensorbleu_sentence_static(const void* cand, int64_t cand_stride, const int32_t* cand_len,
                               const void* refs, int64_t ref_stride, const int32_t* ref_len,
                               int32_t B, int32_t R, const tb_config_t* cfg, void* out_bleu,
                               const tb_stats_t* stats, void* hip_stream) {
  // size check first: a problem beyond the built-in buffer is refused before anything else
  Plans p{};
  int rc = make_plans(B, R, cand_stride, ref_stride, cfg, &p);
  if (rc != TB_OK) return rc;
  if (p.layout.bytes > kStaticScratchBytes) return TB_ERR_STATIC_SCRATCH;
  if (B == 0) return TB_OK;
  void* scratch_ptr = nullptr;
  if (static_scratch_address(&scratch_ptr) != hipSuccess) return TB_ERR_HIP;
  return run_all(cand, cand_stride, cand_len, refs, ref_stride, ref_len, B, R, cfg, out_bleu,
                 stats, scratch_ptr, kStaticScratchBytes, hip_stream, false);
}

const char* tensorbleu_status_string(int status) {
  switch (status) {
    case TB_OK: return "ok";
    case TB_ERR_INVALID_ARG: return "invalid argument";
    case TB_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case TB_ERR_UNSUPPORTED: return "shape not supported by the selected path";
    case TB_ERR_HIP: return "HIP runtime error";
    case TB_ERR_STATIC_SCRATCH:
      return "problem needs more scratch memory than the built-in static buffer holds";
    default: return "unknown status";
  }
}

}  // extern "C"
