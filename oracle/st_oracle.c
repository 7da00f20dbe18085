/*
 * CPU oracle for the SilverTorch retrieval hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition that the GPU library is checked
 * against.  It shares no code with the GPU path and must never be called from
 * it: only the tests, the smoke check and the benchmark's cpu_baseline leg may
 * load it.
 *
 * What it computes (paper sections in brackets):
 *   - per-item m-bit Bloom signatures VB_i, item-major          [Sec. 4.1, text before Eq. 4]
 *   - the Bloom match rule (QB & VB_i) == QB                    [Sec. 4.1, Eq. 4]
 *   - the exact set rule Q subset-of V_i (no hashing)           [Sec. 4.1, Eq. 3]
 *   - int8 x int8 -> int32 dot products                         [Sec. 4.2, Int8 ANN]
 *   - scoring only the items whose mask bit is 1, then ArgTopK  [Sec. 4.3, Alg. 1 phases 3-4,
 *                                                                 every item in scope = all clusters probed]
 *   - the weighted-sum form of the Value Model over T tasks     [Sec. 5.2]
 *   - publish-time int8 quantisation with one global scale      [Sec. 4.2]
 *   - Value Model formulas over per-task scores, as a postfix program [Sec. 5.2]
 *   - cluster probing in front of the filter and the scoring (IVF): centroid
 *     scores, the n_p best clusters, filter and scoring inside them [Sec. 4.2, Alg. 1 phases 1-4]
 *   - boolean filter expressions (AND / OR / NOT) over per-feature
 *     Bloom results, as an operation array run on a stack       [Sec. 4 query form, Sec. 4.3]
 *
 * Constants the paper leaves open are fixed by the build's problem statement:
 *   hash  h_j(f) = splitmix64(f XOR j) mod m,  j = 0..k-1
 *   score = ((float)dot * s_q) * s_i          two separately rounded fp32 multiplies
 *   agg   = fmaf(w_t, score_t, agg), t ascending, agg starts at +0.0f
 *   order = score descending, ties (== on floats) by lower item id
 *   fewer than K passing items: count < K, padding id = -1, score = -inf
 *
 * Floating point is fp32 because the problem statement fixes the precision and
 * the rounding order; the file must be compiled with -ffp-contract=off and
 * without -ffast-math so that no multiply-add is fused behind our back.
 *
 * Pins (tests/test_oracle_pins.py): published splitmix64 outputs, brute force
 * on raw id sets, no-false-negative and false-positive-rate closed form,
 * numpy int32 matmul + stable argsort, exact rational arithmetic for the
 * rescale and the fused multiply-add chain; for the expressions a recursive
 * evaluation of the expression tree on the per-feature masks, the raw id sets
 * of a hand-written corpus, and De Morgan's laws; for the probing a numpy
 * argsort of the centroid scores with the probed ranges masked by hand, the
 * all-clusters-probed case against the plain search, and the paper's
 * probed-fraction arithmetic.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* splitmix64 output function applied to x: add the golden-ratio increment, then mix. */
uint64_t sto_splitmix64(uint64_t x)
{
    uint64_t z = x + 0x9E3779B97F4A7C15ULL;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

/* Bit position of hash j of feature f in an m-bit filter.  [Sec. 4.1] */
int64_t sto_bit_index(uint64_t f, int32_t j, int32_t m)
{
    return (int64_t)(sto_splitmix64(f ^ (uint64_t)j) % (uint64_t)m);
}

static int64_t sig_words(int32_t m) { return ((int64_t)m + 63) / 64; }

/* OR the k hash bits of each of n feature ids into sig (W = ceil(m/64) words,
 * bit b lives in word b/64 at position b%64, least significant first). */
void sto_signature(const uint64_t* ids, int64_t n, int32_t m, int32_t k, uint64_t* sig)
{
    int64_t W = sig_words(m);
    memset(sig, 0, (size_t)W * sizeof(uint64_t));
    for (int64_t a = 0; a < n; ++a)
        for (int32_t j = 0; j < k; ++j) {
            int64_t b = sto_bit_index(ids[a], j, m);
            sig[b / 64] |= 1ULL << (b % 64);
        }
}

/* Item-major Bloom index: sigs[i*W .. i*W+W) = VB_i.  Items given as CSR. */
void sto_bloom_build(const int64_t* feat_offsets, const uint64_t* feat_ids, int64_t n_items,
                     int32_t m, int32_t k, uint64_t* sigs)
{
    int64_t W = sig_words(m);
    for (int64_t i = 0; i < n_items; ++i)
        sto_signature(feat_ids + feat_offsets[i], feat_offsets[i + 1] - feat_offsets[i], m, k,
                      sigs + i * W);
}

static int bloom_pass(const uint64_t* qb, const uint64_t* vb, int64_t W)
{
    for (int64_t w = 0; w < W; ++w)
        if ((qb[w] & vb[w]) != qb[w]) return 0;
    return 1;
}

/* mask[w] bit (i%64) = pass_i for i = 64w + bit; bits at or past n_items are 0.  [Eq. 4] */
void sto_bloom_mask(const uint64_t* sigs, int64_t n_items, int32_t m, int32_t k,
                    const uint64_t* filt_ids, int64_t n_filt, uint64_t* mask)
{
    int64_t W = sig_words(m);
    uint64_t* qb = (uint64_t*)malloc((size_t)W * sizeof(uint64_t));
    sto_signature(filt_ids, n_filt, m, k, qb);
    memset(mask, 0, (size_t)((n_items + 63) / 64) * sizeof(uint64_t));
    for (int64_t i = 0; i < n_items; ++i)
        if (bloom_pass(qb, sigs + i * W, W)) mask[i / 64] |= 1ULL << (i % 64);
    free(qb);
}

/* Exact filter on the raw id lists: pass_i iff every filter id occurs in F_i.  [Eq. 3] */
void sto_exact_mask(const int64_t* feat_offsets, const uint64_t* feat_ids, int64_t n_items,
                    const uint64_t* filt_ids, int64_t n_filt, uint64_t* mask)
{
    memset(mask, 0, (size_t)((n_items + 63) / 64) * sizeof(uint64_t));
    for (int64_t i = 0; i < n_items; ++i) {
        int all = 1;
        for (int64_t a = 0; a < n_filt && all; ++a) {
            int found = 0;
            for (int64_t p = feat_offsets[i]; p < feat_offsets[i + 1]; ++p)
                if (feat_ids[p] == filt_ids[a]) { found = 1; break; }
            all = found;
        }
        if (all) mask[i / 64] |= 1ULL << (i % 64);
    }
}

/* int8 dot product with int32 accumulation.  [Sec. 4.2] */
int32_t sto_dot(const int8_t* q, const int8_t* e, int32_t d)
{
    int32_t acc = 0;
    for (int32_t c = 0; c < d; ++c) acc += (int32_t)q[c] * (int32_t)e[c];
    return acc;
}

/* Two separately rounded fp32 multiplies, left to right. */
float sto_rescale(int32_t dot, float s_q, float s_i)
{
    volatile float a = (float)dot * s_q; /* volatile: forces the intermediate rounding */
    volatile float b = a * s_i;
    return b;
}

/* Score of (query b, item i): single task when task_weight is NULL, else the
 * weighted sum over T tasks as a fused-multiply-add chain, t ascending. */
float sto_pair_score(const int8_t* queries, const float* query_scale, int32_t n_tasks,
                     const float* task_weight, int64_t b, const int8_t* item, float s_i, int32_t d)
{
    if (task_weight == NULL)
        return sto_rescale(sto_dot(queries + b * d, item, d), query_scale[b], s_i);
    float agg = 0.0f;
    for (int32_t t = 0; t < n_tasks; ++t) {
        const int8_t* q = queries + (b * n_tasks + t) * (int64_t)d;
        float st = sto_rescale(sto_dot(q, item, d), query_scale[b * n_tasks + t], s_i);
        agg = fmaf(task_weight[t], st, agg);
    }
    return agg;
}

typedef struct { float score; int64_t id; } sto_cand;

static int cand_cmp(const void* pa, const void* pb)
{
    const sto_cand* a = (const sto_cand*)pa;
    const sto_cand* b = (const sto_cand*)pb;
    if (a->score > b->score) return -1;
    if (a->score < b->score) return 1;
    if (a->id < b->id) return -1;
    if (a->id > b->id) return 1;
    return 0;
}

/*
 * Filtered top-K for a batch.  [Alg. 1 phases 3-4 with every item in scope]
 *   sigs            item-major signatures from sto_bloom_build
 *   items           [n_items, d] int8 row-major;  item_scale [n_items]
 *   queries         [batch, d] (task_weight == NULL) or [batch, n_tasks, d]
 *   query_scale     [batch] or [batch, n_tasks]
 *   filt_offsets    [batch+1] into filt_ids; query b's filter is the conjunction
 *                   of filt_ids[filt_offsets[b] .. filt_offsets[b+1]); empty = all pass
 *   out_ids/out_scores [batch, K]; out_count [batch]
 * Every passing item is scored, the full list is sorted, the first K are kept.
 * Returns 0, or -1 when memory runs out.
 */
int sto_search(const uint64_t* sigs, int64_t n_items, int32_t m, int32_t k,
               const int8_t* items, const float* item_scale, int32_t d,
               const int8_t* queries, const float* query_scale, int32_t batch,
               int32_t n_tasks, const float* task_weight,
               const uint64_t* filt_ids, const int64_t* filt_offsets, int32_t K,
               int64_t* out_ids, float* out_scores, int32_t* out_count)
{
    int64_t W = sig_words(m);
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t b = 0; b < batch; ++b) {
        uint64_t* qb = (uint64_t*)malloc((size_t)W * sizeof(uint64_t));
        sto_cand* cand = (sto_cand*)malloc((size_t)(n_items > 0 ? n_items : 1) * sizeof(sto_cand));
        if (!qb || !cand) {
#pragma omp atomic write
            failed = 1;
            free(qb); free(cand);
            continue;
        }
        sto_signature(filt_ids + filt_offsets[b], filt_offsets[b + 1] - filt_offsets[b], m, k, qb);
        int64_t n = 0;
        for (int64_t i = 0; i < n_items; ++i) {
            if (!bloom_pass(qb, sigs + i * W, W)) continue;
            cand[n].score = sto_pair_score(queries, query_scale, n_tasks, task_weight, b,
                                           items + i * (int64_t)d, item_scale[i], d);
            cand[n].id = i;
            ++n;
        }
        qsort(cand, (size_t)n, sizeof(sto_cand), cand_cmp);
        int64_t keep = n < K ? n : K;
        for (int64_t r = 0; r < K; ++r) {
            out_ids[(int64_t)b * K + r] = r < keep ? cand[r].id : -1;
            out_scores[(int64_t)b * K + r] = r < keep ? cand[r].score : -INFINITY;
        }
        out_count[b] = (int32_t)keep;
        free(qb); free(cand);
    }
    return failed ? -1 : 0;
}

/* ------------------------------------------------------------------------------------------
 * Boolean filter expressions.  [Sec. 4: a query is a conjunction of OR-groups of
 * feature = value terms; Sec. 4.3: per-feature Bloom results and operators are stored in an
 * operation array that is processed in order with a stack]
 *
 * A program is n entries in postfix order.  ops[i] is one of
 *   STO_LEAF (0)  push "item passes the Bloom test of the single feature id ids[i]"
 *                 (all k hash bits of that id are set in VB_i; Eq. 4 with a one-element Q)
 *   STO_AND  (1)  pop two results, push their conjunction
 *   STO_OR   (2)  pop two results, push their disjunction
 *   STO_NOT  (3)  pop one result, push its negation
 * ids[i] is read for leaves only.  A well-formed program never pops an empty stack and leaves
 * exactly one result; the empty program (n == 0) passes every item.
 *
 * A Bloom leaf can be true for an item that lacks the feature (false positive), so a program
 * without NOT can only pass too many items, while under a NOT the error turns round: an item
 * that lacks the feature may be rejected.
 */
enum { STO_LEAF = 0, STO_AND = 1, STO_OR = 2, STO_NOT = 3 };
#define STO_MAX_EXPR_DEPTH 64

/* Largest stack depth the program reaches, or -1 if it is ill-formed (unknown operator,
 * pop from an empty stack, more or less than one result left, deeper than the oracle's stack). */
int32_t sto_expr_depth(const int32_t* ops, int64_t n)
{
    int32_t depth = 0, deepest = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (ops[i] == STO_LEAF) {
            ++depth;
        } else if (ops[i] == STO_AND || ops[i] == STO_OR) {
            if (depth < 2) return -1;
            --depth;
        } else if (ops[i] == STO_NOT) {
            if (depth < 1) return -1;
        } else {
            return -1;
        }
        if (depth > deepest) deepest = depth;
    }
    if (n > 0 && depth != 1) return -1;
    if (deepest > STO_MAX_EXPR_DEPTH) return -1;
    return deepest;
}

/* Value of a (well-formed) program for the item whose signature is vb. */
static int expr_pass(const int32_t* ops, const uint64_t* ids, int64_t n, const uint64_t* vb, int32_t m, int32_t k)
{
    int stack[STO_MAX_EXPR_DEPTH];
    int top = 0;
    if (n == 0) return 1;
    for (int64_t i = 0; i < n; ++i) {
        if (ops[i] == STO_LEAF) {
            int all = 1;
            for (int32_t j = 0; j < k; ++j) {
                int64_t bit = sto_bit_index(ids[i], j, m);
                if (!((vb[bit / 64] >> (bit % 64)) & 1)) all = 0;
            }
            stack[top++] = all;
        } else if (ops[i] == STO_NOT) {
            stack[top - 1] = !stack[top - 1];
        } else {
            int rhs = stack[--top];
            int lhs = stack[--top];
            stack[top++] = ops[i] == STO_AND ? (lhs && rhs) : (lhs || rhs);
        }
    }
    return stack[0];
}

/* mask bit i = value of the program for item i; bits at or past n_items are 0 (also under a
 * NOT).  Returns 0, or -1 for an ill-formed program (mask untouched). */
int sto_expr_mask(const uint64_t* sigs, int64_t n_items, int32_t m, int32_t k,
                  const int32_t* ops, const uint64_t* ids, int64_t n_ops, uint64_t* mask)
{
    if (sto_expr_depth(ops, n_ops) < 0) return -1;
    int64_t W = sig_words(m);
    int64_t n_words = (n_items + 63) / 64;
    for (int64_t w = 0; w < n_words; ++w) mask[w] = 0;
    for (int64_t i = 0; i < n_items; ++i)
        if (expr_pass(ops, ids, n_ops, sigs + i * W, m, k)) mask[i / 64] |= 1ULL << (i % 64);
    return 0;
}

/*
 * Filtered top-K where query b's filter is the program
 * (expr_ops, expr_ids)[expr_offsets[b] .. expr_offsets[b+1]); everything else as in sto_search.
 * Returns 0, -1 when memory runs out, -2 for an ill-formed program.
 */
int sto_search_expr(const uint64_t* sigs, int64_t n_items, int32_t m, int32_t k,
                    const int8_t* items, const float* item_scale, int32_t d,
                    const int8_t* queries, const float* query_scale, int32_t batch,
                    int32_t n_tasks, const float* task_weight,
                    const int32_t* expr_ops, const uint64_t* expr_ids, const int64_t* expr_offsets, int32_t K,
                    int64_t* out_ids, float* out_scores, int32_t* out_count)
{
    int64_t W = sig_words(m);
    int failed = 0;
    for (int32_t b = 0; b < batch; ++b)
        if (sto_expr_depth(expr_ops + expr_offsets[b], expr_offsets[b + 1] - expr_offsets[b]) < 0) return -2;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t b = 0; b < batch; ++b) {
        sto_cand* cand = (sto_cand*)malloc((size_t)(n_items > 0 ? n_items : 1) * sizeof(sto_cand));
        if (!cand) {
#pragma omp atomic write
            failed = 1;
            continue;
        }
        const int32_t* ops = expr_ops + expr_offsets[b];
        const uint64_t* ids = expr_ids + expr_offsets[b];
        int64_t n_ops = expr_offsets[b + 1] - expr_offsets[b];
        int64_t n = 0;
        for (int64_t i = 0; i < n_items; ++i) {
            if (!expr_pass(ops, ids, n_ops, sigs + i * W, m, k)) continue;
            cand[n].score = sto_pair_score(queries, query_scale, n_tasks, task_weight, b,
                                           items + i * (int64_t)d, item_scale[i], d);
            cand[n].id = i;
            ++n;
        }
        qsort(cand, (size_t)n, sizeof(sto_cand), cand_cmp);
        int64_t keep = n < K ? n : K;
        for (int64_t r = 0; r < K; ++r) {
            out_ids[(int64_t)b * K + r] = r < keep ? cand[r].id : -1;
            out_scores[(int64_t)b * K + r] = r < keep ? cand[r].score : -INFINITY;
        }
        out_count[b] = (int32_t)keep;
        free(cand);
    }
    return failed ? -1 : 0;
}

/* ------------------------------------------------------------------------------------------
 * Cluster probing (IVF).  [Sec. 4.2: probe the clusters closest to the query, top-K inside
 * them; Sec. 4.3 / Alg. 1: phase 1 scores the centroids and keeps the n_p best clusters,
 * phase 2 runs the Bloom filter only over the item ranges of those clusters, phase 3 scores
 * the items that pass, phase 4 takes the top K over all probed clusters]
 *
 * Items are stored cluster by cluster: cluster c holds items
 * [cluster_offsets[c], cluster_offsets[c+1]), offsets non-decreasing from 0 to n_items (empty
 * clusters allowed).  Centroids are int8 rows with an fp32 scale like the items, and a
 * centroid's score for query b is the same expression as an item's: rescale(dot, s_q, s_c).
 * Clusters are ranked by (score descending, cluster id ascending), the first
 * min(n_probe, n_clusters) are probed.  Single-task queries only (the paper probes with one
 * user embedding).  out_probes[batch][n_probe] receives the probed cluster ids in rank order
 * (-1 past n_clusters) when not NULL.
 * Returns 0, -1 out of memory, -2 ill-formed program.
 */
typedef struct { float score; int32_t id; } sto_ccand;

static int ccand_cmp(const void* pa, const void* pb)
{
    const sto_ccand* a = (const sto_ccand*)pa;
    const sto_ccand* b = (const sto_ccand*)pb;
    if (a->score > b->score) return -1;
    if (a->score < b->score) return 1;
    if (a->id < b->id) return -1;
    if (a->id > b->id) return 1;
    return 0;
}

int sto_search_ivf(const uint64_t* sigs, int64_t n_items, int32_t m, int32_t k,
                   const int8_t* items, const float* item_scale, int32_t d,
                   const int8_t* centroids, const float* centroid_scale, const int64_t* cluster_offsets,
                   int32_t n_clusters, int32_t n_probe,
                   const int8_t* queries, const float* query_scale, int32_t batch,
                   const int32_t* expr_ops, const uint64_t* expr_ids, const int64_t* expr_offsets, int32_t K,
                   int64_t* out_ids, float* out_scores, int32_t* out_count, int32_t* out_probes)
{
    int64_t W = sig_words(m);
    int failed = 0;
    for (int32_t b = 0; b < batch; ++b)
        if (sto_expr_depth(expr_ops + expr_offsets[b], expr_offsets[b + 1] - expr_offsets[b]) < 0) return -2;
    int32_t np = n_probe < n_clusters ? n_probe : n_clusters;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t b = 0; b < batch; ++b) {
        sto_cand* cand = (sto_cand*)malloc((size_t)(n_items > 0 ? n_items : 1) * sizeof(sto_cand));
        sto_ccand* cl = (sto_ccand*)malloc((size_t)(n_clusters > 0 ? n_clusters : 1) * sizeof(sto_ccand));
        if (!cand || !cl) {
#pragma omp atomic write
            failed = 1;
            free(cand); free(cl);
            continue;
        }
        const int8_t* q = queries + (int64_t)b * d;
        /* phase 1: centroid scores, best n_p clusters */
        for (int32_t c = 0; c < n_clusters; ++c) {
            cl[c].score = sto_rescale(sto_dot(q, centroids + (int64_t)c * d, d), query_scale[b], centroid_scale[c]);
            cl[c].id = c;
        }
        qsort(cl, (size_t)n_clusters, sizeof(sto_ccand), ccand_cmp);
        if (out_probes)
            for (int32_t j = 0; j < n_probe; ++j) out_probes[(int64_t)b * n_probe + j] = j < np ? cl[j].id : -1;
        const int32_t* ops = expr_ops + expr_offsets[b];
        const uint64_t* ids = expr_ids + expr_offsets[b];
        int64_t n_ops = expr_offsets[b + 1] - expr_offsets[b];
        int64_t n = 0;
        for (int32_t j = 0; j < np; ++j) {
            int32_t c = cl[j].id;
            /* phases 2 and 3 inside the cluster's item range */
            for (int64_t i = cluster_offsets[c]; i < cluster_offsets[c + 1]; ++i) {
                if (!expr_pass(ops, ids, n_ops, sigs + i * W, m, k)) continue;
                cand[n].score = sto_rescale(sto_dot(q, items + i * (int64_t)d, d), query_scale[b], item_scale[i]);
                cand[n].id = i;
                ++n;
            }
        }
        /* phase 4 */
        qsort(cand, (size_t)n, sizeof(sto_cand), cand_cmp);
        int64_t keep = n < K ? n : K;
        for (int64_t r = 0; r < K; ++r) {
            out_ids[(int64_t)b * K + r] = r < keep ? cand[r].id : -1;
            out_scores[(int64_t)b * K + r] = r < keep ? cand[r].score : -INFINITY;
        }
        out_count[b] = (int32_t)keep;
        free(cand); free(cl);
    }
    return failed ? -1 : 0;
}

/* ------------------------------------------------------------------------------------------
 * Publish-time quantisation.  [Sec. 4.2: global min / max over all embeddings, scaled to the
 * int8 range, integer representations assigned]
 * Reading: one scale for the whole table, symmetric about zero so that zero maps to zero and
 * inner products need no offset terms: a = max(|min|, |max|), s = a / 127 (1 when the table is
 * all zero), q = round-half-even(x / s) kept inside [-127, 127].  Every row then has the
 * scale s, which is what row_scale receives (the search takes per-row scales).  minmax[0..1]
 * receive the global min and max (0, 0 for an empty table).  Values must be finite.
 */
void sto_quantize_global(const float* x, int64_t n_rows, int32_t d, int8_t* q, float* row_scale, float* minmax)
{
    int64_t n = n_rows * (int64_t)d;
    float mn = n > 0 ? x[0] : 0.0f, mx = mn;
    for (int64_t i = 1; i < n; ++i) {
        if (x[i] < mn) mn = x[i];
        if (x[i] > mx) mx = x[i];
    }
    float a = fabsf(mn) > fabsf(mx) ? fabsf(mn) : fabsf(mx);
    volatile float s = a > 0.0f ? a / 127.0f : 1.0f;
    for (int64_t i = 0; i < n; ++i) {
        volatile float r = x[i] / s;
        float v = nearbyintf(r);  /* default rounding mode: ties to even */
        if (v > 127.0f) v = 127.0f;
        if (v < -127.0f) v = -127.0f;
        q[i] = (int8_t)v;
    }
    for (int64_t i = 0; i < n_rows; ++i) row_scale[i] = s;
    minmax[0] = mn;
    minmax[1] = mx;
}

/* ------------------------------------------------------------------------------------------
 * Value Model formulas.  [Sec. 5.2: per-task predictions are combined into one score by a
 * user-defined formula with conditions, parsed into a tree and evaluated for many items]
 * The tree arrives flattened in postfix order.  Entry i has code ops[i] & 255:
 *   0 TASK   push the item's score of task (ops[i] >> 8)
 *   1 CONST  push consts[i]
 *   2 ADD  3 SUB  4 MUL  5 MIN  6 MAX      pop b, pop a, push a op b   (one fp32 rounding each)
 *   7 GT     pop b, pop a, push (a > b ? 1.0f : 0.0f)
 *   8 SELECT pop y, pop x, pop c, push (c != 0 ? x : y)                   (the conditions)
 * One result must remain.  scores is [n, n_tasks] row-major, out is [n].
 * Returns 0, or -1 for an ill-formed program (unknown code, missing operands, task out of
 * range, more than one result, deeper than 16).
 */
enum { STO_VM_TASK = 0, STO_VM_CONST, STO_VM_ADD, STO_VM_SUB, STO_VM_MUL, STO_VM_MIN, STO_VM_MAX, STO_VM_GT, STO_VM_SELECT };

int32_t sto_vm_depth(const int32_t* ops, int32_t n_ops, int32_t n_tasks)
{
    int32_t depth = 0, deepest = 0;
    for (int32_t i = 0; i < n_ops; ++i) {
        int32_t code = ops[i] & 255;
        if (code == STO_VM_TASK) {
            if ((ops[i] >> 8) < 0 || (ops[i] >> 8) >= n_tasks) return -1;
            ++depth;
        } else if (code == STO_VM_CONST) {
            ++depth;
        } else if (code >= STO_VM_ADD && code <= STO_VM_GT) {
            if (depth < 2) return -1;
            --depth;
        } else if (code == STO_VM_SELECT) {
            if (depth < 3) return -1;
            depth -= 2;
        } else {
            return -1;
        }
        if (depth > deepest) deepest = depth;
    }
    if (depth != 1 || deepest > 16) return -1;
    return deepest;
}

int sto_value_model(const float* scores, int64_t n, int32_t n_tasks, const int32_t* ops, const float* consts,
                    int32_t n_ops, float* out)
{
    if (sto_vm_depth(ops, n_ops, n_tasks) < 0) return -1;
    for (int64_t it = 0; it < n; ++it) {
        volatile float st[16];
        int top = 0;
        for (int32_t i = 0; i < n_ops; ++i) {
            int32_t code = ops[i] & 255;
            if (code == STO_VM_TASK) {
                st[top++] = scores[it * n_tasks + (ops[i] >> 8)];
            } else if (code == STO_VM_CONST) {
                st[top++] = consts[i];
            } else if (code == STO_VM_SELECT) {
                float y = st[--top], x = st[--top], c = st[--top];
                st[top++] = c != 0.0f ? x : y;
            } else {
                float b = st[--top], a = st[--top], r;
                switch (code) {
                case STO_VM_ADD: r = a + b; break;
                case STO_VM_SUB: r = a - b; break;
                case STO_VM_MUL: r = a * b; break;
                case STO_VM_MIN: r = a < b ? a : b; break;
                case STO_VM_MAX: r = a > b ? a : b; break;
                default: r = a > b ? 1.0f : 0.0f; break;
                }
                st[top++] = r;
            }
        }
        out[it] = st[0];
    }
    return 0;
}

/* Threads sto_search uses (for reporting the CPU baseline honestly). */
int32_t sto_num_threads(void)
{
#ifdef _OPENMP
    return (int32_t)omp_get_max_threads();
#else
    return 1;
#endif
}
