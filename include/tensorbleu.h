/*
 * tensorbleu.h -- C ABI of the MI355X (gfx950) batched token-ID BLEU library.
 *
 * The library computes, for a batch of B candidate token-ID sequences with R references each,
 * one BLEU score per candidate (tensorbleu_sentence) or one score for the batch
 * (tensorbleu_corpus): n-gram extraction for n = 1..N, a compact dictionary of the n-grams
 * present, offset batched counting, clipping against the maximum reference count, modified
 * precisions, brevity penalty, smoothing and the weighted geometric mean (paper Sections
 * 3.1-3.4 and the BLEU equation of Section 2.1).
 *
 * Conventions that hold for every entry point unless stated otherwise
 *   - Every data pointer is a DEVICE pointer owned by the caller (the library never allocates,
 *     frees or keeps a pointer after the call returns).  `cfg`, `stats` and `layout` structs are
 *     HOST memory, read (or written, for layout) during the call only.
 *   - All work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL = the default
 *     stream).  No entry point synchronises; outputs are valid once the stream has been
 *     synchronised by the caller.
 *   - Layout: candidate i is the row `cand + i*cand_stride`, valid for `cand_len[i]` tokens;
 *     reference j of candidate i is the row `refs + (i*R + j)*ref_stride`, valid for
 *     `ref_len[i*R + j]` tokens (or, with cfg->ref_offsets, row ref_offsets[i] + j of a packed
 *     list of reference rows).  Token ids are int32, or int64 when cfg->token_bytes == 8 (the
 *     usual dtype of tokenizer output; read directly, no conversion pass).  Strides are in
 *     elements and bound the lengths; lengths are always int32; cells
 *     at or beyond a row's length are never interpreted (token id 0 inside the length is an
 *     ordinary token).  Lengths found outside [0, stride] on the device are clamped and
 *     reported through TB_DEV_LENGTH_RANGE.
 *   - Host-detectable problems are reported through the return value (tb_status_t) before any
 *     work is enqueued.  Conditions only visible on the device are OR-ed into
 *     `stats->device_status` (caller clears it; may be NULL); scores of affected rows are then
 *     unspecified but every access stays in bounds.
 *   - B == 0 returns TB_OK without enqueuing work.
 */
#ifndef TENSORBLEU_H
#define TENSORBLEU_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  TB_OK = 0,
  TB_ERR_INVALID_ARG = 1, /* NULL required pointer, B < 0, R < 1, max_n outside 1..8, bad stride */
  TB_ERR_WORKSPACE = 2,   /* workspace NULL, misaligned (256 B) or smaller than workspace_bytes */
  TB_ERR_UNSUPPORTED = 3, /* shape outside what the kernels handle (see tensorbleu_workspace_layout) */
  TB_ERR_HIP = 4,         /* a HIP runtime call or kernel launch failed */
  TB_ERR_STATIC_SCRATCH = 5 /* tensorbleu_sentence_static: the problem needs more scratch memory
                             than the library's built-in buffer holds */
} tb_status_t;

/* Smoothing of the modified precisions p_n (paper Section 3.4 names 'floor', 'add-k', 'exp'
 * after Chen & Cherry 2014).  With c_n the clipped count and d_n = max(total_n, 1):
 *   NONE   p_n = c_n / d_n; any p_n == 0 with w_n > 0 gives score 0
 *   FLOOR  c_n == 0  ->  p_n = smooth_param / d_n
 *   ADD_K  n >= 2    ->  p_n = (c_n + smooth_param) / (d_n + smooth_param); n = 1 unsmoothed
 *   EXP    the z-th order (scanning n = 1..N) with c_n == 0 gets p_n = 1 / (2^z * d_n)
 * In every mode a candidate with no matching unigram, or of length 0, scores 0. */
typedef enum { TB_SMOOTH_NONE = 0, TB_SMOOTH_FLOOR = 1, TB_SMOOTH_ADD_K = 2, TB_SMOOTH_EXP = 3 } tb_smooth_t;

/* Execution paths.  FUSED: one kernel, one workgroup per sentence group, tokens staged once in
 * LDS and dictionary + counts kept in LDS.  GLOBAL: pack -> dictionary -> count/clip -> finalize
 * with packed keys and inverse indices materialised in the workspace. */
typedef enum { TB_PATH_AUTO = 0, TB_PATH_FUSED = 1, TB_PATH_GLOBAL = 2 } tb_path_t;

/* Bits of *stats->device_status. */
enum { TB_DEV_TOKEN_RANGE = 1,  /* a token inside a row's length was outside [0, vocab_size) */
       TB_DEV_LENGTH_RANGE = 2, /* a length outside [0, stride], or a reference count outside
                                   [1, R], was clamped */
       TB_DEV_TABLE_OVERFLOW = 4 /* GLOBAL path with partitioned tables (global_partitions > 0):
                                   more distinct n-grams hashed into one partition than it can
                                   hold; cannot happen unless keys are built to collide.  The
                                   score of such a group is NaN (and so is a corpus score it
                                   enters), so that it cannot pass for a reward; its integer
                                   statistics are unspecified.  The same call with
                                   cfg->workspace_tables set cannot overflow */ };

typedef struct tb_config {
  int32_t max_n;        /* N: highest n-gram order, 1..8 (Section 2.1 names 1 to 4 as the usual range);
                           the GLOBAL path packs whole n-grams into keys and so needs
                           N * bits <= 128, the FUSED path has no such limit */
  float   weights[8];   /* w_1..w_N of the BLEU equation, used as given (not renormalised);
                           w_n == 0 drops order n; all zero means uniform 1/N */
  int32_t smoothing;    /* tb_smooth_t */
  float   smooth_param; /* eps for FLOOR, k for ADD_K; ignored otherwise */
  int32_t vocab_size;   /* token ids lie in [0, vocab_size); fixes the key width:
                           bits = ceil(log2(vocab_size)), order-n keys take n*bits bits and are
                           stored in 8 bytes, or 16 bytes when n*bits > 64 */
  int32_t force_path;   /* tb_path_t; TB_PATH_AUTO picks FUSED when a group fits its LDS budget */
  int32_t token_bytes;  /* element size of `cand` / `refs`: 4 (int32; 0 means 4) or 8 (int64).
                           An int64 id outside [0, vocab_size) is reported like any other
                           out-of-range token */
  int32_t score_bytes;  /* element size of the score outputs: 4 (float32; 0 means 4) or 2
                           (bfloat16: the float32 score rounded to nearest even, the direction
                           Section 6 names; the arithmetic itself stays float32) */
  const int32_t* ref_count; /* optional DEVICE pointer [B] (NULL: every candidate has R references):
                           candidate i is scored against its first ref_count[i] references only;
                           the remaining rows of its R reference rows are ignored entirely (no
                           n-grams, no part in the closest reference length).  Values outside
                           [1, R] are clamped and reported through TB_DEV_LENGTH_RANGE.  The
                           staged GLOBAL entry points must all see the same array. */
  const int32_t* ref_offsets; /* optional DEVICE pointer [B + 1] (NULL: the fixed layout above):
                           reference lists in CSR form, for batches whose candidates have very
                           different numbers of references.  `refs` is then ref_rows packed rows
                           of ref_stride elements and `ref_len` has one entry per row; candidate i
                           owns the rows ref_offsets[i] .. ref_offsets[i + 1] - 1, its references
                           in order.  The R argument of the call is the largest number of
                           references any candidate has (it sizes workspace and plans; the
                           ROUGE-N overlap output stays [B, R]).  A candidate without rows has no
                           reference: its statistics and score are 0 and its closest reference
                           length is 0.  Spans that leave [0, ref_rows] or hold more than R rows
                           are clamped and reported through TB_DEV_LENGTH_RANGE, as is an empty
                           span.  Not together with ref_count (TB_ERR_INVALID_ARG). */
  int64_t ref_rows;     /* with ref_offsets: the number of reference rows in `refs` / `ref_len` */
  int32_t workspace_tables; /* non-zero: the GLOBAL path keeps its hash tables and counters in the
                           workspace whatever the shape (the kernels it otherwise uses beyond
                           2 097 152 slots per group).  Several times slower than tables in LDS,
                           but no table has a capacity that data can exceed: the way to re-issue a
                           call that reported TB_DEV_TABLE_OVERFLOW, and to get ROUGE-N for the
                           shapes tensorrouge_n otherwise refuses on the GLOBAL path.  Workspace
                           sizes and layouts depend on it like on the other fields */
} tb_config_t;

/* Optional integer outputs (each pointer may be NULL).  These are what the parity tests compare
 * bit-exactly with the CPU oracle. */
typedef struct tb_stats {
  int32_t* clipped;         /* [B, N] sum over distinct candidate n-grams of min(count in candidate,
                               max over references of count in reference)   (Section 3.3 step 3) */
  int32_t* total;           /* [B, N] number of candidate n-grams, max(len - n + 1, 0) (Section 3.4) */
  int32_t* closest_ref_len; /* [B] reference length closest to the candidate's (shorter on ties) */
  int32_t* group_distinct;  /* [B, N] size of the group's dictionary: distinct n-grams over the
                               candidate and its references (GLOBAL path only; FUSED writes the
                               candidate's distinct count, its dictionary holds candidates only).
                               Written by the dictionary pass; with global_partitions > 0 by the
                               count/clip pass, which sums the partitions' sizes */
  int64_t* corpus_stats;    /* [2N+2] clipped_1..N, total_1..N, sum of candidate lengths, sum of
                               closest reference lengths (Section 3.4, corpus variant) */
  int32_t* device_status;   /* [1] OR of TB_DEV_* bits; cleared by the caller */
} tb_stats_t;

/* Where the GLOBAL path keeps its intermediates inside the workspace (byte offsets).  Slot
 * numbering of the per-order key / inverse-index arrays: sentence group g owns slots
 * [g*group_cap, (g+1)*group_cap) and fills them compactly from the front with its valid n-grams
 * of that order: the candidate's (in position order), then reference 0's, reference 1's, ...
 * Sequence s of the group therefore starts at g*group_cap + sum over earlier sequences of
 * max(len - n + 1, 0).  Slots past the group's last n-gram are never written.  The staged entry
 * points below fill these arrays as described; what tensorbleu_sentence / tensorbleu_corpus
 * leave in the workspace is unspecified (they skip stores that only a staged caller would
 * read). */
typedef struct tb_layout {
  int32_t path;            /* path AUTO resolves to for this shape (TB_PATH_FUSED / TB_PATH_GLOBAL) */
  int32_t bits;            /* ceil(log2(vocab_size)), at least 1 */
  int32_t key_bytes[8];    /* 8 or 16 per order */
  int64_t group_cap;       /* cand_stride + R*ref_stride */
  size_t  keys_off[8];     /* packed keys of order n: B*group_cap entries of key_bytes[n-1] */
  size_t  inv_off[8];      /* uint32 offset ids: g*id_stride + the n-gram's id in the group's
                              dictionary (ids are below id_stride; dense 0..distinct-1 unless
                              global_partitions > 0) */
  size_t  clipped_off, total_off, closest_off, distinct_off; /* int32 [B,N],[B,N],[B],[B,N] */
  size_t  cand_distinct_off; /* int32 [B,N]: distinct n-grams of the candidate alone (GLOBAL path,
                              written by the dictionary pass when global_candidate_first is set) */
  size_t  corpus_off;      /* int64 [2N+2] */
  size_t  overlap_off;     /* int32 [B, R]: ROUGE-N overlap counts (GLOBAL path) */
  size_t  bytes;           /* total workspace size for this path */
  int32_t fused_ok;        /* 1 if the FUSED path supports this shape */
  int32_t global_ok;       /* 1 if the GLOBAL path supports this shape */
  int32_t global_tables_in_hbm; /* 1 if the group is too large for the LDS kernels: the GLOBAL
                              path then keeps its hash tables and counters at tables_off */
  size_t  tables_off;      /* ... or, with global_partitions > 0, int32 [B, N, P]: the dictionary
                              size of every partition, followed by the partitioned kernels'
                              private arrays (per order and slot: the n-grams sorted by
                              partition as slot number, partition-local id | sequence index << 16,
                              and 8-byte key) */
  int64_t id_stride;       /* id range per group on the GLOBAL path: group_cap, or more when
                              global_partitions > 0 */
  int32_t global_candidate_first; /* 1: the dictionary pass numbers the candidate's n-grams first:
                              ids below cand_distinct[g][n] are exactly the n-grams that occur
                              in candidate g (the count/clip pass then keeps counters for those
                              only).  Set for groups within one LDS table whose (prefix id, last
                              token) keys fit 31 bits: ceil(log2(group_cap)) + bits <= 31 */
  int32_t global_partitions; /* P > 0: groups beyond the single-table LDS kernels (12 288 slots)
                              but within 2 097 152 are handled by P workgroups per (group, order),
                              each keeping one hash partition of the dictionary in LDS; ids are
                              then p*6144 + a number dense within partition p.  Orders whose
                              packed keys take 16 bytes are keyed there by (id of the (n-1)-gram
                              at the same position, last token) */
} tb_layout_t;

/* Workspace size in bytes for a problem shape (pure host function of the shapes; 0 on invalid
 * arguments).  The size covers whichever path cfg->force_path selects (AUTO: the resolved one).
 * The workspace must be 256-byte aligned device memory; its contents need no initialisation and
 * are undefined afterwards. */
size_t tensorbleu_workspace_bytes(int32_t B, int32_t R, int64_t cand_stride, int64_t ref_stride,
                                  const tb_config_t* cfg);

/* Same computation as tensorbleu_workspace_bytes, returning the full layout.  Host only. */
int tensorbleu_workspace_layout(int32_t B, int32_t R, int64_t cand_stride, int64_t ref_stride,
                                const tb_config_t* cfg, tb_layout_t* layout);

/* One BLEU score per candidate: out_bleu[B] float32, or bfloat16 when cfg->score_bytes == 2
 * (device).  Implements Sections 3.1-3.4 with
 * the brevity penalty BP = 1 if c > r else exp(1 - r/c) and BLEU = BP * exp(sum_n w_n log p_n). */
int tensorbleu_sentence(const void* cand, int64_t cand_stride, const int32_t* cand_len,
                        const void* refs, int64_t ref_stride, const int32_t* ref_len,
                        int32_t B, int32_t R, const tb_config_t* cfg, void* out_bleu,
                        const tb_stats_t* stats, void* workspace, size_t workspace_bytes,
                        void* hip_stream);

/* One score for the whole batch: numerators, denominators, candidate lengths and closest
 * reference lengths are summed over the batch before the precisions are formed (Section 3.4,
 * second paragraph).  out_bleu[1] float32 or bfloat16 (device). */
int tensorbleu_corpus(const void* cand, int64_t cand_stride, const int32_t* cand_len,
                      const void* refs, int64_t ref_stride, const int32_t* ref_len,
                      int32_t B, int32_t R, const tb_config_t* cfg, void* out_bleu,
                      const tb_stats_t* stats, void* workspace, size_t workspace_bytes,
                      void* hip_stream);

/* tensorbleu_sentence for callers that cannot allocate device memory and have no workspace to
 * pass: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, outputs and error behaviour as tensorbleu_sentence, minus the workspace: the
 * intermediates (integer statistics the caller did not ask for; on the GLOBAL path also keys,
 * ids and tables) live in a buffer of tensorbleu_static_scratch_bytes() = 4 MiB that is part of
 * the library's device code, one copy per GPU, held until the process ends.  The call allocates
 * nothing and frees nothing.  A problem whose workspace (tensorbleu_workspace_bytes for the same
 * arguments) exceeds that size returns TB_ERR_STATIC_SCRATCH before any work is enqueued: the
 * headline shape on the FUSED path needs 25 KB, B = 65 536 candidates at N = 4 about 3.3 MB.
 * All calls on one GPU share that GPU's buffer, which keeps the last call's bytes (no kernel
 * relies on its contents): calls that may overlap in time on one GPU - different streams, or
 * several host threads - race and must be serialised by the caller; calls on one stream are
 * ordered and safe. */
int tensorbleu_sentence_static(const void* cand, int64_t cand_stride, const int32_t* cand_len,
                               const void* refs, int64_t ref_stride, const int32_t* ref_len,
                               int32_t B, int32_t R, const tb_config_t* cfg, void* out_bleu,
                               const tb_stats_t* stats, void* hip_stream);

/* Size of the built-in scratch buffer of tensorbleu_sentence_static (host function). */
size_t tensorbleu_static_scratch_bytes(void);

/* ROUGE-N on the same n-gram counting core (the paper's Section 6 names ROUGE as the first
 * metric the method extends to; the metric is Lin 2004).  For the single order n = cfg->max_n
 * (1..8) and every candidate i and reference j:
 *   overlap[i][j] = sum over distinct n-grams of min(count in candidate i, count in reference j),
 *   precision = overlap / candidate n-grams, recall = overlap / reference n-grams (0 when the
 *   denominator is 0), F = (1 + beta^2) P R / (R + beta^2 P) (0 when P + R = 0),
 *   beta = cfg->smooth_param (<= 0 means 1).
 * out_prf[B, 3] float32 or bfloat16 (cfg->score_bytes; device) receives precision, recall and F of the candidate's best
 * reference: the first one with the largest overlap / (candidate n-grams + beta^2 * reference
 * n-grams), to which F is proportional.  overlap[B, R] int32 and best_ref[B] int32 (index of that
 * reference) are optional device outputs (NULL to skip); entries of references beyond
 * cfg->ref_count[i] are 0.  cfg->weights and cfg->smoothing are ignored; vocab_size, token_bytes
 * and ref_count mean what they mean for BLEU.  Paths as for BLEU (cfg->force_path; AUTO takes
 * FUSED where the shape fits it, else GLOBAL: pack and dictionary for the orders 1..n, then the
 * count pass for order n with per-reference sums).  On GLOBAL, one kind of shape returns
 * TB_ERR_UNSUPPORTED: LDS-resident groups on plain packed-key tables (global_candidate_first == 0,
 * global_partitions == 0, global_tables_in_hbm == 0: more than 62 references, or (id, token) keys
 * beyond 32 bits); the same call with cfg->workspace_tables set serves it.  Workspace:
 * tensorbleu_workspace_bytes for the same arguments (cfg->max_n = n).  stats: only
 * device_status is used. */
int tensorrouge_n(const void* cand, int64_t cand_stride, const int32_t* cand_len,
                  const void* refs, int64_t ref_stride, const int32_t* ref_len, int32_t B,
                  int32_t R, const tb_config_t* cfg, void* out_prf, int32_t* overlap,
                  int32_t* best_ref, const tb_stats_t* stats, void* workspace,
                  size_t workspace_bytes, void* hip_stream);

/* ---- The GLOBAL path one pass at a time (same arguments and workspace as above; the workspace
 * must have been sized with force_path = TB_PATH_GLOBAL).  tensorbleu_sentence on the GLOBAL
 * path computes exactly what pack, dictionary, count_clip, finalize compute in this order.
 * Exposed so that each pass can be checked and timed on its own.  (With partitioned tables,
 * global_partitions > 0, the single call itself fuses neighbouring passes: its dictionary pass
 * extracts the n-grams from the token rows, so no key array is written, and counts in place
 * where the counters fit the table's memory.  The staged calls below keep the pass boundaries.) */

/* Section 3.1 + 3.2 step 1: every valid n-gram, n = 1..N, packed big-endian into a key
 * (first token in the most significant bits) and written to its slot in keys_off[n-1]. */
int tensorbleu_pack(const void* cand, int64_t cand_stride, const int32_t* cand_len,
                    const void* refs, int64_t ref_stride, const int32_t* ref_len, int32_t B,
                    int32_t R, const tb_config_t* cfg, const tb_stats_t* stats, void* workspace,
                    size_t workspace_bytes, void* hip_stream);

/* Section 3.2 step 2: per sentence group and order, a dictionary of the distinct keys (LDS hash
 * table, exact key comparison) giving every n-gram occurrence a dense id in [0, U_g); written
 * with the group's offset (Section 3.3 step 1) to inv_off[n-1]; U_g goes to distinct_off. */
int tensorbleu_dictionary(const int32_t* cand_len, const int32_t* ref_len, int64_t cand_stride,
                          int64_t ref_stride, int32_t B, int32_t R, const tb_config_t* cfg,
                          const tb_stats_t* stats, void* workspace, size_t workspace_bytes,
                          void* hip_stream);

/* Section 3.3 steps 2-3: counts of the offset ids for the candidate and for each reference (LDS
 * atomics), maximum over references, minimum with the candidate count, summed to clipped[B,N];
 * total[B,N] from the lengths. */
int tensorbleu_count_clip(const int32_t* cand_len, const int32_t* ref_len, int64_t cand_stride,
                          int64_t ref_stride, int32_t B, int32_t R, const tb_config_t* cfg,
                          const tb_stats_t* stats, void* workspace, size_t workspace_bytes,
                          void* hip_stream);

/* Section 3.4: closest reference length, brevity penalty, smoothing, geometric mean from the
 * integer statistics in the workspace.  corpus != 0 writes out_bleu[1], else out_bleu[B]. */
int tensorbleu_finalize(const int32_t* cand_len, const int32_t* ref_len, int32_t B, int32_t R,
                        int64_t cand_stride, int64_t ref_stride, const tb_config_t* cfg,
                        int32_t corpus, void* out_bleu, const tb_stats_t* stats, void* workspace,
                        size_t workspace_bytes, void* hip_stream);

/* Text for a tb_status_t value (static storage, host). */
const char* tensorbleu_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* TENSORBLEU_H */
