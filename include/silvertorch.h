/*
 * silvertorch.h -- C ABI of the MI355X (gfx950) filtered int8 top-K retrieval library.
 *
 * The library implements the retrieval hot path of the SilverTorch paper on one GPU:
 * a per-item Bloom signature index used as a feature filter (Sec. 4.1), int8 dot-product
 * scoring with int32 accumulation that streams item rows straight from the embedding
 * table (Sec. 4.2), scoring only the items whose filter bit is 1 and selecting the global
 * top-K (Sec. 4.3, Algorithm 1 phases 3-4 with every item in scope, i.e. brute force), and
 * the weighted-sum Value Model over per-task scores (Sec. 5.2).
 *
 * Conventions for every entry point
 *   - returns ST_OK (0) or a negative st_status; never throws, never aborts.  After a
 *     failure st_last_error() (thread local) describes it.
 *   - "dev_" pointers are device memory on the current HIP device, "host_" pointers are
 *     host memory; the caller owns every buffer it passes and keeps it alive until the
 *     stream has finished the enqueued work.
 *   - hip_stream is a hipStream_t passed as void* (NULL = the default stream).  Work is
 *     enqueued asynchronously; outputs are valid once the stream has synchronised.
 *   - the search entry points allocate no device memory: the caller passes a workspace of
 *     at least st_search_workspace_bytes() bytes, 256-byte aligned.
 *
 * Numerical contract (checked bit for bit against the CPU oracle)
 *   hash       h_j(f) = splitmix64(f XOR j) mod m_bits, j = 0 .. k_hashes-1
 *   pass_i     (QB & VB_i) == QB                                   Eq. 4
 *   dot        sum_c (int32)q[c] * (int32)e_i[c]                   int32, cannot overflow for d <= 65536/4
 *   score      ((float)dot * s_q) * s_i                            two rounded fp32 multiplies
 *   aggregate  agg = fmaf(w[t], score_t, agg), t ascending from +0.0f
 *   order      score descending, ties by lower item id
 */
#ifndef SILVERTORCH_H
#define SILVERTORCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum st_status {
    ST_OK = 0,
    ST_EINVAL = -1,     /* bad argument (null pointer, size out of range, misaligned buffer) */
    ST_ENOMEM = -2,     /* host or device allocation failed */
    ST_EHIP = -3,       /* a HIP runtime call failed; st_last_error() has hipGetErrorString */
    ST_EWORKSPACE = -4  /* workspace smaller than st_search_workspace_bytes() */
} st_status;

/* limits (arguments outside them give ST_EINVAL) */
#define ST_MAX_M_BITS 65536     /* Bloom bits per item */
#define ST_MAX_K_HASHES 16
#define ST_MAX_FILTER_BITS 64   /* distinct signature bits one query's filter may set (<= k * terms) */
#define ST_MAX_BATCH 4096
#define ST_MAX_TASKS 8
#define ST_MAX_TOP_K 131072    /* the paper's pre-filter sizes reach O(10^5) items, Sec. 5.1 */
#define ST_MAX_DIM 4096         /* d, a multiple of 16 */
#define ST_MAX_CLUSTERS 65536   /* clusters of st_search_ivf */
#define ST_MAX_PROBES 2048      /* clusters probed per query */
#define ST_MAX_EXPR_OPS 256     /* entries of one filter program */
#define ST_MAX_EXPR_DEPTH 16    /* results a filter program may hold on its stack at once */

#define ST_MAX_VM_OPS 64        /* entries of a Value Model formula */
#define ST_MAX_VM_DEPTH 16      /* values a formula may hold on its stack at once */

/* operations of a Value Model formula (st_value_model): code = entry & 255 */
#define ST_VM_TASK 0            /* push the item's score of task (entry >> 8) */
#define ST_VM_CONST 1           /* push the entry's constant */
#define ST_VM_ADD 2             /* pop b, pop a, push a + b (one fp32 rounding; likewise below) */
#define ST_VM_SUB 3             /* a - b */
#define ST_VM_MUL 4             /* a * b */
#define ST_VM_MIN 5             /* a < b ? a : b */
#define ST_VM_MAX 6             /* a > b ? a : b */
#define ST_VM_GT 7              /* a > b ? 1.0f : 0.0f */
#define ST_VM_SELECT 8          /* pop y, pop x, pop c, push c != 0 ? x : y */

/* operations of a filter program (st_bloom_mask_expr, st_search_expr) */
#define ST_OP_LEAF 0            /* push: the item passes the Bloom test of one feature id */
#define ST_OP_AND 1             /* pop two results, push their conjunction */
#define ST_OP_OR 2              /* pop two results, push their disjunction */
#define ST_OP_NOT 3             /* pop one result, push its negation */

/* Thread-local text of the last failure in the calling thread ("" if none). */
const char* st_last_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int32_t st_version(void);

/* ------------------------------------------------------------------ Bloom index
 * Opaque handle owning the device-resident index: for every item an m_bits-bit Bloom
 * filter over its feature ids (Sec. 4.1).  Stored bit-sliced ("rotated", Sec. 4.1):
 * one row per signature bit, 64 items per 64-bit word, blocked in tiles of 1024 items so
 * that one row segment of a tile is one 128-byte line. */
typedef struct st_bloom st_bloom;

/* Builds the index.  The items' feature lists arrive as CSR (the forward-index shape of
 * Sec. 4.1): feat_offsets[n_items+1] (non-decreasing, feat_offsets[0] == 0) and
 * feat_ids[feat_offsets[n_items]].  Both arrays may be host or device memory (detected).
 * Duplicate ids in a list are harmless; an empty list gives the zero signature.
 * 1 <= m_bits <= ST_MAX_M_BITS (any value, not only powers of two), 1 <= k_hashes <=
 * ST_MAX_K_HASHES, 0 <= n_items < 2^31.  Synchronises hip_stream before returning.
 * On success *out receives a handle to be released with st_bloom_free. */
int st_bloom_build(const int64_t* feat_offsets, const uint64_t* feat_ids, int64_t n_items,
                   int32_t m_bits, int32_t k_hashes, void* hip_stream, st_bloom** out);

/* Frees the handle and its device memory (NULL is allowed). */
int st_bloom_free(st_bloom* bloom);

/* Device bytes of the index: n_items*m_bits/8 rounded up to whole 1024-item tiles (the
 * paper's N*M/8 accounting, Sec. 6.2.2).  st_bloom_layout_bytes is the same figure from
 * the sizes alone and touches no GPU.  Negative st_status on bad arguments. */
int64_t st_bloom_bytes(const st_bloom* bloom);
int64_t st_bloom_layout_bytes(int64_t n_items, int32_t m_bits);
int64_t st_bloom_n_items(const st_bloom* bloom);

/* Parity/debug export, not on the timed path: item-major signatures,
 * dev_out[n_items][ceil(m_bits/64)], bit b of item i in word b/64 at position b%64. */
int st_bloom_export_signatures(const st_bloom* bloom, uint64_t* dev_out, void* hip_stream);

/* Parity/debug export of the Bloom test (Eq. 4) as 1 bit per item (Sec. 4.3):
 * dev_mask[n_filters][ceil(n_items/64)], bit (i%64) of word i/64 is pass_i, bits at or
 * past n_items are 0.  Filter f is the conjunction of
 * host_filt_ids[host_filt_offsets[f] .. host_filt_offsets[f+1]); empty = every item passes. */
int st_bloom_mask(const st_bloom* bloom, const uint64_t* host_filt_ids,
                  const int64_t* host_filt_offsets, int32_t n_filters, uint64_t* dev_mask,
                  void* hip_stream);

/* ------------------------------------------------------------------ search
 * Bytes of device workspace st_search / st_search_multitask need for these sizes
 * (n_tasks = 1 for st_search).  Pure host arithmetic.  Negative st_status on bad sizes. */
int64_t st_search_workspace_bytes(int64_t n_items, int32_t d, int32_t batch, int32_t n_tasks,
                                  int32_t K);

/* Filtered top-K for a batch of queries (Algorithm 1, phases 3-4, all items in scope).
 *   bloom            index built over the same n_items items
 *   dev_items        [n_items, d] int8 row-major, 16-byte aligned; d % 16 == 0, d <= ST_MAX_DIM
 *   dev_item_scale   [n_items] fp32, finite and > 0, 16-byte aligned
 *   dev_queries      [batch, d] int8, 16-byte aligned;  dev_query_scale [batch] fp32, finite and > 0
 *   host_filt_ids / host_filt_offsets[batch+1]
 *                    query b keeps item i iff i passes the Bloom test for the conjunction of
 *                    ids [offsets[b], offsets[b+1]); an empty range keeps every item.  A
 *                    filter may set at most ST_MAX_FILTER_BITS distinct signature bits.
 *   K                1 <= K <= ST_MAX_TOP_K
 *   dev_out_ids      [batch, K] int64, dev_out_scores [batch, K] fp32, dev_out_count [batch]
 *                    int32: the min(K, #passing) best items by (score desc, id asc); rows past
 *                    count are id = -1, score = -inf.
 *   dev_workspace    >= st_search_workspace_bytes(...) bytes, 256-byte aligned; contents are
 *                    scratch.  Concurrent searches need distinct workspaces.
 * The host filter arrays are consumed before the call returns. */
int st_search(const st_bloom* bloom, const int8_t* dev_items, const float* dev_item_scale,
              int64_t n_items, int32_t d, const int8_t* dev_queries, const float* dev_query_scale,
              int32_t batch, const uint64_t* host_filt_ids, const int64_t* host_filt_offsets,
              int32_t K, int64_t* dev_out_ids, float* dev_out_scores, int32_t* dev_out_count,
              void* dev_workspace, int64_t workspace_bytes, void* hip_stream);

/* st_search for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation.  The workspace is a
 * fixed device array of ST_STATIC_SCRATCH_BYTES inside the library (one copy per GPU, held until
 * the process ends); the call allocates nothing, on the device or pinned (the staging slots and
 * the array's address are set up by st_bloom_build on that device).  Sizes whose
 * st_search_workspace_bytes() exceeds ST_STATIC_SCRATCH_BYTES give ST_EWORKSPACE (the Mid shape,
 * 1 M items x batch 64 x K 100, fits); a batch whose filter tables exceed a 64 KB staging slot gives
 * ST_EINVAL.  Every call on a GPU uses that GPU's one array: calls that overlap in time on one
 * GPU (two streams, two threads) race, callers serialise them.  Nothing in the array has to
 * survive from call to call and nothing has to be cleared: every kernel of a search writes what
 * it later reads.  Arguments, outputs, ordering, asynchrony and errors otherwise as for st_search. */
#define ST_STATIC_SCRATCH_BYTES (80ll << 20)
int st_search_static(const st_bloom* bloom, const int8_t* dev_items, const float* dev_item_scale,
                     int64_t n_items, int32_t d, const int8_t* dev_queries, const float* dev_query_scale,
                     int32_t batch, const uint64_t* host_filt_ids, const int64_t* host_filt_offsets,
                     int32_t K, int64_t* dev_out_ids, float* dev_out_scores, int32_t* dev_out_count,
                     void* hip_stream);

/* Multi-task variant (Sec. 5.2): one embedding per task and query, item embeddings shared,
 * one result list per query on the Value Model's weighted sum of the per-task scores.
 *   dev_queries [batch, n_tasks, d], dev_query_scale [batch, n_tasks],
 *   host_task_weight [n_tasks] fp32 (finite), 1 <= n_tasks <= ST_MAX_TASKS.
 * score_t as in st_search; agg = fmaf(w[t], score_t, agg) for t = 0 .. n_tasks-1 from +0.0f;
 * ranking and outputs are on agg.  Everything else as st_search. */
int st_search_multitask(const st_bloom* bloom, const int8_t* dev_items,
                        const float* dev_item_scale, int64_t n_items, int32_t d,
                        const int8_t* dev_queries, const float* dev_query_scale, int32_t batch,
                        int32_t n_tasks, const float* host_task_weight,
                        const uint64_t* host_filt_ids, const int64_t* host_filt_offsets,
                        int32_t K, int64_t* dev_out_ids, float* dev_out_scores,
                        int32_t* dev_out_count, void* dev_workspace, int64_t workspace_bytes,
                        void* hip_stream);

/* Parity/debug export of the scoring arithmetic for chosen (query, item) pairs (Sec. 4.2):
 * dev_out_dot[p] = int32 dot of query dev_pair_query[p] (a row of dev_queries [*, d]) and item
 * dev_pair_item[p]; dev_out_score[p] = ((float)dot * s_q) * s_i.  Either output may be NULL. */
int st_score_pairs(const int8_t* dev_items, const float* dev_item_scale, int32_t d,
                   const int8_t* dev_queries, const float* dev_query_scale,
                   const int64_t* dev_pair_item, const int32_t* dev_pair_query, int64_t n_pairs,
                   int32_t* dev_out_dot, float* dev_out_score, void* hip_stream);

/* Diagnostic: byte offset, inside a workspace laid out for these sizes (the arguments of
 * st_search_workspace_bytes), of the per-query overflow flags: uint32 [batch], valid once a
 * search on that workspace has completed.  1 = one of the query's candidate regions overflowed
 * in some level, or fewer than K keys reached a threshold tighter than the K-th best so far,
 * and the query was recomputed by the slow exact path (Algorithm 1 phases 3-4 are
 * then evaluated for that query alone, over the whole corpus); results are exact either way, the
 * flag only tells that the fast path did not hold.  Negative st_status on bad sizes. */
int64_t st_search_overflow_flags_offset(int64_t n_items, int32_t d, int32_t batch, int32_t n_tasks,
                                        int32_t K);

/* Host-side description of how a search of these sizes is scheduled (pure arithmetic, no
 * GPU): writes up to max_levels rows of 3 int64 {item_begin, item_end, segment_items} and
 * returns the number of levels, or a negative st_status.  The corpus is scanned once, in
 * consecutive chunks ("levels"); after each chunk a selection keeps the best keys seen so far
 * and the last of them becomes the admission threshold of the next (fewer than K keys are kept
 * before the last level: a tighter threshold, checked and backed by the exact slow path at the
 * end).  The rows give the sizes; a search served by the 8-wavefront MFMA scan alone takes the
 * items of its first level as segments spread evenly over the corpus rather than as the prefix
 * [item_begin, item_end) and scans the rest from item 0, and then also halves that level where the
 * schedule has two levels and the second would still hand the last selection few keys (small K).
 * q_split (a power of two, 1 unless the query rows of a large batch are
 * spread over several rows of workgroups) divides the workgroups that share one query's
 * candidates.  out_caps receives {workgroups, region_capacity}. */
int32_t st_search_plan(int64_t n_items, int32_t batch, int32_t K, int32_t q_split,
                       int64_t* out_levels, int32_t max_levels, int64_t* out_caps);

/* ------------------------------------------------------------------ filter expressions
 * Filters with AND, OR and NOT (Sec. 4: a query is the embedding search AND OR-groups of
 * feature = value terms; Sec. 4.3: per-feature Bloom results and operators in an operation
 * array that is run in order on a stack).  A program is a sequence of entries in postfix order
 * (operands before their operator): host_expr_ops[i] is an ST_OP_* code and host_expr_ids[i]
 * the feature id of an ST_OP_LEAF entry (ignored for operators).  A leaf is true for an item
 * when all k hash bits of the id are set in the item's signature (Eq. 4 with one id), so a
 * conjunction of leaves is exactly the filter st_search takes.  Program p occupies entries
 * [host_expr_offsets[p], host_expr_offsets[p+1]); an empty program passes every item.
 * ST_EINVAL for an ill-formed program: unknown code, an operator without operands, more or
 * fewer than one result left, more than ST_MAX_EXPR_OPS entries, stack deeper than
 * ST_MAX_EXPR_DEPTH.  Bloom false positives make a leaf pass too many items; under a NOT
 * the error turns round (too few).
 *
 * Parity/debug export (Sec. 4.3: 1 bit per item), like st_bloom_mask:
 * dev_mask[n_exprs][ceil(n_items/64)], bits at or past n_items are 0.  Allocates a small
 * table and synchronises hip_stream before returning. */
int st_bloom_mask_expr(const st_bloom* bloom, const int32_t* host_expr_ops,
                       const uint64_t* host_expr_ids, const int64_t* host_expr_offsets,
                       int32_t n_exprs, uint64_t* dev_mask, void* hip_stream);

/* Workspace of st_search_expr: that of st_search / st_search_multitask plus one mask row per
 * query and the program tables; n_expr_entries = host_expr_offsets[batch] of the call (or an
 * upper bound, at most batch * ST_MAX_EXPR_OPS).  Pure host arithmetic. */
int64_t st_search_expr_workspace_bytes(int64_t n_items, int32_t d, int32_t batch,
                                       int32_t n_tasks, int32_t K, int64_t n_expr_entries);

/* st_search (host_task_weight == NULL, n_tasks == 1) or st_search_multitask (weights given)
 * where query b's filter is program b.  One kernel evaluates every distinct program of the
 * batch into a 1-bit-per-item mask in the workspace (Sec. 4.3: the search takes a bit mask
 * from the Bloom index); the fused scan then tests one mask row per query group instead of
 * the signature rows.  Arguments, outputs, ordering, asynchrony and errors as for st_search;
 * the host arrays may be reused when the call returns. */
int st_search_expr(const st_bloom* bloom, const int8_t* dev_items, const float* dev_item_scale,
                   int64_t n_items, int32_t d, const int8_t* dev_queries,
                   const float* dev_query_scale, int32_t batch, int32_t n_tasks,
                   const float* host_task_weight, const int32_t* host_expr_ops,
                   const uint64_t* host_expr_ids, const int64_t* host_expr_offsets, int32_t K,
                   int64_t* dev_out_ids, float* dev_out_scores, int32_t* dev_out_count,
                   void* dev_workspace, int64_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------ cluster probing (IVF)
 * The co-designed search of Sec. 4.3 / Algorithm 1 in its four phases: (1) score every
 * centroid against the query and keep the n_probe best clusters, (2) run the filter only over
 * the item ranges of those clusters, (3) score the items that pass, (4) top-K over all probed
 * clusters.  Items must be stored cluster by cluster: cluster c is the item range
 * [dev_cluster_offsets[c], dev_cluster_offsets[c+1]) (int64 [n_clusters+1], device memory,
 * non-decreasing from 0 to n_items; empty clusters allowed; ranges are clipped to the corpus).
 * dev_centroids [n_clusters, d] int8 (16-byte aligned) with dev_centroid_scale [n_clusters] fp32:
 * a centroid's score is the item score expression ((float)dot * s_q) * s_c; clusters rank by
 * score descending, then id ascending; min(n_probe, n_clusters) are probed.  Queries are
 * single-task ([batch, d]); filters are programs as for st_search_expr (a conjunction is its
 * leaves ANDed).  dev_out_probes (int32 [batch, n_probe], may be NULL) receives the probed
 * cluster ids in rank order, -1 past n_clusters.  With n_probe >= n_clusters the result is that
 * of st_search_expr.  1 <= n_clusters <= ST_MAX_CLUSTERS, 1 <= n_probe <= ST_MAX_PROBES.
 * Up to 512 probes run as one kernel per batch over the probed ranges alone; more probes go
 * through per-query mask rows and the fused scan of st_search_expr.
 * Everything else (outputs, ordering, workspace ownership, asynchrony, errors) as for st_search. */
int64_t st_search_ivf_workspace_bytes(int64_t n_items, int32_t d, int32_t batch, int32_t K,
                                      int32_t n_clusters, int32_t n_probe, int64_t n_expr_entries);
int st_search_ivf(const st_bloom* bloom, const int8_t* dev_items, const float* dev_item_scale,
                  int64_t n_items, int32_t d, const int8_t* dev_centroids,
                  const float* dev_centroid_scale, const int64_t* dev_cluster_offsets,
                  int32_t n_clusters, int32_t n_probe, const int8_t* dev_queries,
                  const float* dev_query_scale, int32_t batch, const int32_t* host_expr_ops,
                  const uint64_t* host_expr_ids, const int64_t* host_expr_offsets, int32_t K,
                  int64_t* dev_out_ids, float* dev_out_scores, int32_t* dev_out_count,
                  int32_t* dev_out_probes, void* dev_workspace, int64_t workspace_bytes,
                  void* hip_stream);

/* ------------------------------------------------------------------ publish-time quantisation
 * Int8 quantisation of an embedding table with one global scale (Sec. 4.2: global min / max
 * over all embeddings, scaled to the int8 range).  Reading: symmetric about zero, so that zero
 * maps to zero and inner products need no offset terms: a = max(|min|, |max|), s = a / 127
 * (s = 1 for an all-zero table), q = round-half-even(x / s) kept inside [-127, 127].
 *   dev_x          [n_rows, d] fp32 row-major, 16-byte aligned, finite values
 *   dev_q          [n_rows, d] int8 out, 16-byte aligned: the items / queries layout of st_search
 *   dev_row_scale  [n_rows] fp32 out, every entry = s (the search takes per-row scales)
 *   dev_minmax     [2] fp32 out: global min and max (0, 0 for an empty table)
 *   dev_scratch8   8 bytes of device scratch, 8-byte aligned (the running min / max)
 * 1 <= d <= ST_MAX_DIM (any d, not only multiples of 16), n_rows * d <= 2^40.  Three kernels on
 * hip_stream, asynchronous, no allocation. */
int st_quantize_global(const float* dev_x, int64_t n_rows, int32_t d, int8_t* dev_q,
                       float* dev_row_scale, float* dev_minmax, void* dev_scratch8,
                       void* hip_stream);

/* ------------------------------------------------------------------ Value Model formulas
 * Combines the per-task scores of n items into one score each by a user formula with
 * conditions (Sec. 5.2: formulas are parsed into a tree and a GPU kernel evaluates them for
 * many items in parallel).  The tree is passed flattened in postfix order: host_ops[i] is an
 * ST_VM_* code (ST_VM_TASK | task << 8 for a task's score), host_consts[i] the constant of an
 * ST_VM_CONST entry (ignored otherwise, but finite).  The weighted sum of st_search_multitask
 * is one such formula (with separately rounded multiply and add instead of its fused chain).
 *   dev_task_scores [n, n_tasks] fp32 row-major; dev_out [n] fp32; 1 <= n_tasks <= 64
 * ST_EINVAL for an ill-formed formula (unknown code, missing operands, task out of range, not
 * exactly one result, more than ST_MAX_VM_OPS entries, deeper than ST_MAX_VM_DEPTH).
 * One kernel on hip_stream, asynchronous, no allocation; the formula travels in its arguments. */
int st_value_model(const float* dev_task_scores, int64_t n, int32_t n_tasks,
                   const int32_t* host_ops, const float* host_consts, int32_t n_ops,
                   float* dev_out, void* hip_stream);

/* Bandwidth probe for benchmarks: one kernel that reads bytes / 16 16-byte pieces of dev_src
 * (16-byte aligned) with `workgroups` workgroups of 256 threads and writes one uint32 per workgroup
 * to dev_sink ([workgroups]).  Its measured rate is the practical HBM read ceiling that the
 * roofline fractions of the search kernels are quoted against beside the published peak.
 * Asynchronous on hip_stream, no allocation; timed by st_timing_begin / _end as kind 0. */
int st_stream_read(const void* dev_src, int64_t bytes, void* dev_sink, int32_t workgroups, void* hip_stream);

/* Host part of st_search / st_search_multitask alone, for tests of the host logic and for timing
 * it without a GPU: the argument checks on the sizes, the hashing of every filter id into
 * signature rows (Eq. 4), the grouping of queries with equal filters, the split of the groups
 * between the two scorers, the schedule, and the table blob a real call would upload.  Touches no
 * device memory and enqueues nothing.  m_bits / k_hashes are those of the index a real call would
 * pass.  host_out_summary[8] receives {distinct filters, groups scored with int8 MFMA, groups
 * scored with the wavefront dot product, rows of workgroups the resident queries are split
 * over, wavefronts per MFMA workgroup (0: none), levels, bytes of tables uploaded, 1 if the
 * search starts with the per-query seed pass}.  Errors as for st_search. */
int st_search_host_plan(int64_t n_items, int32_t d, int32_t batch, int32_t n_tasks, int32_t K,
                        int32_t m_bits, int32_t k_hashes, const uint64_t* host_filt_ids,
                        const int64_t* host_filt_offsets, int32_t* host_out_summary);

/* Search scheduling knob for tests: path = 0 auto, 1 force the wavefront dot-product scorer,
 * 2 force the int8 MFMA scorer where it applies.  The setting belongs to the calling thread
 * (searches of other threads are not affected).  Returns the thread's old value. */
int32_t st_set_scoring_path(int32_t path);

/* Per-kernel timing for benchmarks.  Between st_timing_begin and st_timing_end every kernel the
 * search entry points launch from the calling thread is bracketed by two HIP events recorded on
 * the caller's stream (up to max_launches launches; the state belongs to the calling thread).
 * st_timing_end waits for the recorded events and returns, per kernel kind (0 = scan,
 * 1 = select, 2 = slow exact path, 3 = filter expressions), the summed elapsed milliseconds in
 * host_out_ms[4] and the number of launches in host_out_launches[4]. */
int st_timing_begin(int32_t max_launches);
int st_timing_end(double* host_out_ms, int64_t* host_out_launches);

#ifdef __cplusplus
}
#endif
#endif /* SILVERTORCH_H */
