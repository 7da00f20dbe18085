// Cluster probing (Sec. 4.2; Sec. 4.3, Alg. 1).
//
// Items are stored cluster by cluster; cluster c is the item range [off[c], off[c+1]).
// Phase 1 (ivf_probe_kernel): one workgroup per query scores every centroid like an item
// (int8 dot, two fp32 multiplies), and an exact top-n_p by (score descending, cluster id
// ascending) gives the probed clusters.
// Phases 2-4, up to kQueryProbes probes (ivf_query_kernel): one workgroup per query filters and
// scores the items of its probed ranges alone and selects the top K.
// Phase 2, any number of probes (ivf_mask_kernel): 32 threads per (query, probed cluster) run the
// query's filter program only over the words of that cluster's range and OR the result into the
// query's row of a bit-sliced mask index (zeroed beforehand), laid out like the Bloom index; phases
// 3-4 are then the ordinary fused scan and selection reading that mask index: items outside the
// probed ranges have mask bit 0 and are never loaded.
#pragma once
#include "st_bloom_kernels.h"
#include "st_search_kernels.h"

namespace st {

constexpr int kProbeThreads = 256;

struct IvfParams {
    const int8_t* queries;        // [batch][d]
    const float* qscale;          // [batch]
    const int8_t* centroids;      // [n_clusters][d]
    const float* cscale;          // [n_clusters]
    const int64_t* cluster_off;   // [n_clusters + 1]
    int32_t d, n_clusters, n_probe, k_pad, batch;
    int64_t n_items;
    uint64_t* keys;               // [batch][n_clusters]  scratch: centroid keys
    int32_t* probes;              // [batch][n_probe]     probed clusters in rank order, -1 = none
    int32_t* user_probes;         // the same for the caller, or null
};

// Dynamic LDS: sorted keys [k_pad], histogram [256], misc [8], reduction [2 * waves].
inline size_t probe_lds_bytes(int k_pad) { return (size_t)k_pad * 8 + 256 * 4 + 8 * 4 + 2 * (kProbeThreads / 64) * 8 + 16; }

__global__ __launch_bounds__(kProbeThreads) void ivf_probe_kernel(IvfParams p)
{
    extern __shared__ uint64_t probe_lds[];
    uint64_t* s_sorted = probe_lds;                                       // [k_pad]
    uint64_t* s_red = s_sorted + p.k_pad;                                 // [2 * waves]
    uint32_t* s_hist = reinterpret_cast<uint32_t*>(s_red + 2 * (kProbeThreads / 64));  // [256]
    uint32_t* s_misc = s_hist + 256;                                      // [8]
    const int tid = threadIdx.x, b = blockIdx.x;
    const float sq = p.qscale[b];
    uint64_t* keys = p.keys + (int64_t)b * p.n_clusters;
    int64_t qoff[kRowBlock];
#pragma unroll
    for (int r = 0; r < kRowBlock; ++r) qoff[r] = (int64_t)b * p.d;
    for (int c = tid; c < p.n_clusters; c += kProbeThreads) {
        // (query chunks through the scalar cache, centroid chunks four loads at a time)
        int acc[kRowBlock] = {0, 0, 0, 0, 0, 0, 0, 0};
        dot_block<1>(reinterpret_cast<const int4*>(p.centroids + (int64_t)c * p.d), p.queries, qoff, p.d >> 4, acc);
        const float s = rescale(acc[0], sq, p.cscale[c]);
        keys[c] = make_key(s, (uint32_t)c);
    }
    __threadfence_block();
    __syncthreads();
    const int want = p.n_probe < p.n_clusters ? p.n_probe : p.n_clusters;
    const int n_out = wg_topk(keys, p.n_clusters, want, s_sorted, p.k_pad, s_hist, s_misc, s_red);
    __syncthreads();
    for (int j = tid; j < p.n_probe; j += kProbeThreads) {
        const int32_t c = j < n_out ? (int32_t)key_item(s_sorted[j]) : -1;
        p.probes[(int64_t)b * p.n_probe + j] = c;
        if (p.user_probes) p.user_probes[(int64_t)b * p.n_probe + j] = c;
    }
}

// Phase 1 for many centroids, in two kernels.  Part kernel, grid (batch, parts): a workgroup
// scores its slice of the centroids (at most kTopkRegs * kProbeThreads of them) into LDS, keeps the
// best min(n_probe, slice) keys with the register-resident select and leaves them, unordered, at
// the head of its slice of the key scratch.  Merge kernel, one workgroup per query: the parts'
// survivors (at most kTopkRegs * kProbeMergeThreads in all: the host chooses the number of parts
// accordingly) are selected and sorted in LDS and the probed ids written.
constexpr int kProbeParts = 16;
constexpr int kProbeMergeThreads = 512;

__global__ __launch_bounds__(kProbeThreads) void ivf_probe_part_kernel(IvfParams p, int chunk, uint32_t* part_cnt)
{
    __shared__ uint64_t s_keys[kTopkRegs * kProbeThreads];
    __shared__ uint64_t s_sorted[kLdsSortMax];
    __shared__ uint32_t s_hist[3 * 256], s_misc[8];
    __shared__ uint64_t s_red[32];
    const int tid = threadIdx.x, b = blockIdx.x, part = blockIdx.y;
    const int c0 = part * chunk;
    int n = p.n_clusters - c0;
    n = n < 0 ? 0 : (n > chunk ? chunk : n);
    const float sq = p.qscale[b];
    int64_t qoff[kRowBlock];
#pragma unroll
    for (int r = 0; r < kRowBlock; ++r) qoff[r] = (int64_t)b * p.d;
    for (int i = tid; i < n; i += kProbeThreads) {
        const int c = c0 + i;
        int acc[kRowBlock] = {0, 0, 0, 0, 0, 0, 0, 0};
        dot_block<1>(reinterpret_cast<const int4*>(p.centroids + (int64_t)c * p.d), p.queries, qoff, p.d >> 4, acc);
        s_keys[i] = make_key(rescale(acc[0], sq, p.cscale[c]), (uint32_t)c);
    }
    __syncthreads();
    const int want = p.n_probe < n ? p.n_probe : n;
    int kept = 0;
    if (n > 0) {
        uint64_t kth;
        kept = lds_topk(s_keys, n, want, s_sorted, p.k_pad, s_hist, s_misc, s_red, false, kth);
        __syncthreads();
    }
    uint64_t* dst = p.keys + (int64_t)b * p.n_clusters + c0;  // kept <= n: inside this part's slice
    for (int i = tid; i < kept; i += kProbeThreads) dst[i] = s_sorted[i];
    if (tid == 0) part_cnt[b * kProbeParts + part] = (uint32_t)kept;
}

__global__ __launch_bounds__(kProbeMergeThreads) void ivf_probe_merge_kernel(IvfParams p, int chunk, int parts,
                                                                           const uint32_t* part_cnt)
{
    __shared__ uint64_t s_keys[kTopkRegs * kProbeMergeThreads];
    __shared__ uint64_t s_sorted[kLdsSortMax];
    __shared__ uint32_t s_hist[3 * 256], s_misc[8];
    __shared__ uint64_t s_red[32];
    const int tid = threadIdx.x, b = blockIdx.x;
    uint32_t at = 0;
    for (int pp = 0; pp < parts; ++pp) {
        uint32_t c = part_cnt[b * kProbeParts + pp];
        c = c < (uint32_t)p.n_probe ? c : (uint32_t)p.n_probe;  // (a part keeps at most n_probe, whatever the memory says)
        const uint64_t* src = p.keys + (int64_t)b * p.n_clusters + (int64_t)pp * chunk;
        if (at + c > (uint32_t)(kTopkRegs * kProbeMergeThreads)) c = (uint32_t)(kTopkRegs * kProbeMergeThreads) - at;
        for (uint32_t i = tid; i < c; i += kProbeMergeThreads) s_keys[at + i] = src[i];
        at += c;
    }
    __syncthreads();
    const int want = p.n_probe < p.n_clusters ? p.n_probe : p.n_clusters;
    uint64_t kth;
    const int n_out = lds_topk(s_keys, (int)at, want, s_sorted, p.k_pad, s_hist, s_misc, s_red, true, kth);
    __syncthreads();
    for (int j = tid; j < p.n_probe; j += kProbeMergeThreads) {
        const int32_t c = j < n_out ? (int32_t)key_item(s_sorted[j]) : -1;
        p.probes[(int64_t)b * p.n_probe + j] = c;
        if (p.user_probes) p.user_probes[(int64_t)b * p.n_probe + j] = c;
    }
}

// grid (ceil(n_probe / kMaskProbes), batch): a workgroup takes kMaskProbes probed clusters of one
// query, 32 threads per cluster (a cluster of a thousand items is 16 words).  prog_off / code /
// leaf_rows as for bloom_expr_kernel, one program per query.  mask_rows: bit-sliced index with
// `batch` rows; row b belongs to query b.
constexpr int kMaskProbes = 8;
__global__ __launch_bounds__(256) void ivf_mask_kernel(const uint64_t* __restrict__ bloom, int32_t m_bits,
                                                       int32_t k_hashes, IvfParams p,
                                                       const int32_t* __restrict__ prog_off,
                                                       const int32_t* __restrict__ code,
                                                       const int32_t* __restrict__ leaf_rows,
                                                       uint64_t* __restrict__ mask_rows)
{
    __shared__ uint64_t s_stack[kExprDepth][256];
    __shared__ int32_t s_code[kExprOps];
    __shared__ int32_t s_rows[kExprOps * kExprHashes];
    const int tid = threadIdx.x, b = blockIdx.y;
    const int sub = tid >> 5, wl = tid & 31;
    const int j = (int)blockIdx.x * kMaskProbes + sub;
    const int32_t c = j < p.n_probe ? p.probes[(int64_t)b * p.n_probe + j] : -1;
    // the range, kept inside the corpus whatever the offsets say (empty when there is no cluster)
    int64_t lo = 0, hi = 0;
    if (c >= 0) {
        lo = p.cluster_off[c];
        hi = p.cluster_off[c + 1];
        lo = lo < 0 ? 0 : (lo > p.n_items ? p.n_items : lo);
        hi = hi < lo ? lo : (hi > p.n_items ? p.n_items : hi);
    }
    const int i0 = prog_off[b], n_ops = prog_off[b + 1] - i0;
    for (int i = tid; i < n_ops; i += 256) s_code[i] = code[i0 + i];
    for (int i = tid; i < n_ops * k_hashes; i += 256) s_rows[i] = leaf_rows[(int64_t)i0 * k_hashes + i];
    __syncthreads();  // the only barrier: threads without work may leave below
    if (lo >= hi) return;
    const int64_t w_first = lo >> 6, w_last = (hi - 1) >> 6;
    for (int64_t gw = w_first + wl; gw <= w_last; gw += 32) {
        // bits of this word that belong to [lo, hi)
        const int64_t first = gw * 64;
        uint64_t in = ~0ULL;
        if (first < lo) in &= ~0ULL << (lo - first);
        if (first + 64 > hi) in &= ~0ULL >> (first + 64 - hi);
        const uint64_t* base = bloom + ((gw >> 4) * (int64_t)m_bits) * kTileWords + (gw & 15);
        const uint64_t res = expr_eval_word(s_code, s_rows, n_ops, k_hashes, base, s_stack, tid) & in;
        // neighbouring clusters of one query share their boundary word: OR, not store
        if (res) atomicOr((unsigned long long*)&mask_rows[((gw >> 4) * (int64_t)p.batch + b) * kTileWords + (gw & 15)],
                          (unsigned long long)res);
    }
}

// ------------------------------------------------------------------------------------------
// Phases 2-4 in one kernel, for up to kQueryProbes probes: one workgroup per query walks the
// words of its probed clusters (all of them laid end to end, one word per thread and round), runs
// the filter program on each word, scores the items that pass itself (one v_dot4 row product per
// set bit), appends their keys to the query's buffer and prunes the buffer to the best K whenever
// it cannot take another round; the final selection writes the result rows.  The work is
// proportional to the probed items, nothing is written for the rest of the corpus, and no
// candidate can be lost (no regions, no thresholds from elsewhere).
constexpr int kQueryThreads = 512;
constexpr int kQueryProbes = 512;   // one probe per thread when the ranges are laid out
constexpr int kQueryParts = 8;      // workgroups per query, at most

struct IvfQueryParams {
    IvfParams ivf;
    const uint64_t* bloom;
    int32_t m_bits, k_hashes;
    const int8_t* items;
    const float* iscale;
    const int32_t *prog_off, *code, *leaf_rows;
    uint64_t* gath;            // [batch][gath_cap] key buffer
    int64_t gath_cap;
    uint64_t* srt;             // [batch][k_pad] when k_pad > kLdsSortMax, else null
    int32_t K, k_pad;
    int64_t* out_ids;
    float* out_scores;
    int32_t* out_count;
    uint32_t* ovf;             // [batch] "took the slow exact path" flags of the workspace: reset (this path has none)
    // several workgroups per query (grid.y = parts <= kQueryParts): each takes every parts-th round
    // with its own share of the key buffer and keeps its best K; ivf_merge_kernel merges them
    uint32_t* part_cnt;        // [batch][kQueryParts] keys each part kept
};

__global__ __launch_bounds__(kQueryThreads) void ivf_query_kernel(IvfQueryParams p)
{
    __shared__ uint64_t s_stack[kExprDepth][kQueryThreads];
    __shared__ int32_t s_code[kExprOps];
    __shared__ int32_t s_rows[kExprOps * kExprHashes];
    __shared__ uint64_t s_sorted[kLdsSortMax];
    __shared__ int64_t s_lo[kQueryProbes], s_hi[kQueryProbes];
    __shared__ uint32_t s_first[kQueryProbes + 1];  // first word (in the laid-out order) of each probe
    __shared__ uint32_t s_hist[3 * 256], s_misc[8], s_wsum[kQueryThreads / 64];
    __shared__ uint64_t s_red[32];
    __shared__ int64_t s_word[kQueryThreads];  // first item of the word each thread evaluated this round
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, b = blockIdx.x;
    const IvfParams& v = p.ivf;
    static_assert(sizeof(s_stack) >= (size_t)kTopkRegs * kQueryThreads * 8, "the stack doubles as the final key buffer");

    // the program, and the item ranges of the probed clusters (clipped to the corpus)
    const int i0 = p.prog_off[b], n_ops = p.prog_off[b + 1] - i0;
    for (int i = tid; i < n_ops; i += kQueryThreads) s_code[i] = p.code[i0 + i];
    for (int i = tid; i < n_ops * p.k_hashes; i += kQueryThreads) s_rows[i] = p.leaf_rows[(int64_t)i0 * p.k_hashes + i];
    uint32_t words = 0;
    if (tid < kQueryProbes) {
        int64_t lo = 0, hi = 0;
        const int32_t c = tid < v.n_probe ? v.probes[(int64_t)b * v.n_probe + tid] : -1;
        if (c >= 0) {
            lo = v.cluster_off[c];
            hi = v.cluster_off[c + 1];
            lo = lo < 0 ? 0 : (lo > v.n_items ? v.n_items : lo);
            hi = hi < lo ? lo : (hi > v.n_items ? v.n_items : hi);
        }
        s_lo[tid] = lo;
        s_hi[tid] = hi;
        words = hi > lo ? (uint32_t)(((hi - 1) >> 6) - (lo >> 6) + 1) : 0u;
    }
    // exclusive prefix sum of the word counts over the workgroup
    uint32_t incl = words;
    incl = wave_scan_add(incl);
    if (lane == 63) s_wsum[wv] = incl;
    if (tid == 0) {
        s_misc[4] = 0;  // keys in the buffer
        p.ovf[b] = 0u;
    }
    __syncthreads();
    uint32_t base = 0, total = 0;
    for (int w = 0; w < kQueryThreads / 64; ++w) {
        const uint32_t t = s_wsum[w];
        if (w < wv) base += t;
        total += t;
    }
    if (tid < kQueryProbes) s_first[tid] = base + incl - words;
    if (tid == 0) s_first[kQueryProbes] = total;
    __syncthreads();

    const int part = blockIdx.y, parts = gridDim.y;
    const int64_t cap = p.gath_cap / parts;  // this workgroup's share of the query's key buffer
    uint64_t* buf = p.gath + (int64_t)b * p.gath_cap + part * cap;
    uint64_t* sorted = p.srt ? p.srt + (int64_t)b * p.k_pad : s_sorted;
    uint32_t* s_n = &s_misc[4];
    int64_t qoff[kRowBlock];
#pragma unroll
    for (int r = 0; r < kRowBlock; ++r) qoff[r] = (int64_t)b * v.d;
    const float sq = v.qscale[b];
    uint64_t tau = 0;
    // words per round: as many as the buffer is sure to hold beside the K keys kept
    int64_t wpr = (cap - p.K) / 64;
    wpr = wpr > kQueryThreads ? kQueryThreads : (wpr < 1 ? 1 : wpr);
    {   // no longer than an even share of the query's words (whole wavefronts), so that every part has work
        const int64_t share = (((int64_t)total + parts - 1) / parts + 63) & ~63LL;
        if (share < wpr) wpr = share < 64 ? 64 : share;
    }
    for (uint32_t w0 = (uint32_t)(part * wpr); w0 < total; w0 += (uint32_t)(parts * wpr)) {
        if ((int64_t)*s_n + wpr * 64 > cap) {  // uniform: *s_n is stable between barriers
            const int n_out = wg_topk(buf, (int64_t)*s_n, p.K, sorted, p.k_pad, s_hist, s_misc, s_red, false, &tau);
            for (int i = tid; i < n_out; i += kQueryThreads) buf[i] = sorted[i];
            __syncthreads();
            if (tid == 0) *s_n = (uint32_t)n_out;
            __syncthreads();
        }
        const uint32_t wi = w0 + tid;
        uint64_t m = 0;
        int64_t first = 0;
        if (tid < wpr && wi < total) {
            // the probe this word belongs to: last j with s_first[j] <= wi
            int a = 0, z = kQueryProbes;
            while (z - a > 1) {
                const int mid = (a + z) >> 1;
                if (s_first[mid] <= wi) a = mid; else z = mid;
            }
            const int64_t lo = s_lo[a], hi = s_hi[a];
            const int64_t gw = (lo >> 6) + (wi - s_first[a]);
            first = gw * 64;
            uint64_t in = ~0ULL;
            if (first < lo) in &= ~0ULL << (lo - first);
            if (first + 64 > hi) in &= ~0ULL >> (first + 64 - hi);
            const uint64_t* wbase = p.bloom + ((gw >> 4) * (int64_t)p.m_bits) * kTileWords + (gw & 15);
            m = expr_eval_word(s_code, s_rows, n_ops, p.k_hashes, wbase, s_stack, tid) & in;
        }
        // The wavefront's passing items, dealt out evenly over its lanes: every lane lists its set
        // bits as (lane, bit) pairs in the wavefront's own columns of the stack (free once the words
        // are evaluated; 16 rows x 64 columns x 8 bytes = 4096 pairs, the most 64 words can hold).
        s_word[tid] = first;
        const int cnt = __popcll(m);
        int inc = cnt;
        inc = (int)wave_scan_add((uint32_t)inc);
        const int wave_total = (int)lane_value((uint32_t)inc, 63);
        auto pair_at = [&](int e) -> uint16_t* {
            return reinterpret_cast<uint16_t*>(&s_stack[e >> 8][wv * 64]) + (e & 255);
        };
        {
            int e = inc - cnt;
            uint64_t mm = m;
            while (mm) {
                const int bit = __ffsll((long long)mm) - 1;
                mm &= mm - 1;
                *pair_at(e++) = (uint16_t)((lane << 6) | bit);
            }
        }
        __syncthreads();
        for (int k = lane; k < wave_total; k += 64) {
            const int pr = *pair_at(k);
            const int64_t item = s_word[wv * 64 + (pr >> 6)] + (pr & 63);
            // (query chunks through the scalar cache, item chunks four loads at a time)
            int acc[kRowBlock] = {0, 0, 0, 0, 0, 0, 0, 0};
            dot_block<1>(reinterpret_cast<const int4*>(p.items + item * v.d), v.queries, qoff, v.d >> 4, acc);
            const float sc = rescale(acc[0], sq, p.iscale[item]);
            const uint64_t key = make_key(sc, (uint32_t)item);
            if (key >= tau) buf[atomicAdd(s_n, 1u)] = key;
        }
        __syncthreads();
    }
    uint32_t n_keys = *s_n;
    if (parts > 1) {
        // keep this part's best K (unordered) at the head of its share
        if (n_keys > (uint32_t)p.K) {
            uint64_t kth;
            int kept;
            if (n_keys <= (uint32_t)(kTopkRegs * kQueryThreads)) {  // register-resident select on a copy in LDS
                uint64_t* s_keys = &s_stack[0][0];
                __syncthreads();
                for (uint32_t i = tid; i < n_keys; i += kQueryThreads) s_keys[i] = buf[i];
                __syncthreads();
                kept = lds_topk(s_keys, (int)n_keys, p.K, s_sorted, p.k_pad, s_hist, s_misc, s_red, false, kth);
                __syncthreads();
            } else {
                kept = wg_topk(buf, (int64_t)n_keys, p.K, s_sorted, p.k_pad, s_hist, s_misc, s_red, false, &kth);
            }
            for (int i = tid; i < kept; i += kQueryThreads) buf[i] = s_sorted[i];
            n_keys = (uint32_t)kept;
        }
        // the merge is a kernel of its own (ivf_merge_kernel): a device-wide fence here, for a
        // last-finisher merge in this kernel, measured 30 us per workgroup
        if (tid == 0) p.part_cnt[b * kQueryParts + part] = n_keys;
        return;
    }
    // final selection: in LDS (the stack is free now) when the keys and the result fit there
    int n_out;
    if (!p.srt && n_keys <= (uint32_t)(kTopkRegs * kQueryThreads)) {
        uint64_t* s_keys = &s_stack[0][0];
        __syncthreads();
        for (uint32_t i = tid; i < n_keys; i += kQueryThreads) s_keys[i] = buf[i];
        __syncthreads();
        uint64_t kth;
        n_out = lds_topk(s_keys, (int)n_keys, p.K, s_sorted, p.k_pad, s_hist, s_misc, s_red, true, kth);
    } else {
        n_out = wg_topk(buf, (int64_t)n_keys, p.K, sorted, p.k_pad, s_hist, s_misc, s_red);
    }
    write_result(sorted, n_out, p.K, p.out_ids + (int64_t)b * p.K, p.out_scores + (int64_t)b * p.K, p.out_count + b);
}

// Merge of the parts' survivors (at most kTopkRegs * kQueryThreads keys per query: the host chooses
// the number of parts accordingly): one workgroup per query, selection and sort in LDS.
__global__ __launch_bounds__(kQueryThreads) void ivf_merge_kernel(IvfQueryParams p, int parts)
{
    __shared__ uint64_t s_keys[kTopkRegs * kQueryThreads];
    __shared__ uint64_t s_sorted[kLdsSortMax];
    __shared__ uint32_t s_hist[3 * 256], s_misc[8];
    __shared__ uint64_t s_red[32];
    const int tid = threadIdx.x, b = blockIdx.x;
    const int64_t cap = p.gath_cap / parts;
    uint32_t at = 0;
    for (int pp = 0; pp < parts; ++pp) {
        uint32_t c = p.part_cnt[b * kQueryParts + pp];
        c = c < (uint32_t)p.K ? c : (uint32_t)p.K;  // (a part keeps at most K, whatever the memory says)
        const uint64_t* src = p.gath + (int64_t)b * p.gath_cap + pp * cap;
        for (uint32_t i = tid; i < c; i += kQueryThreads) s_keys[at + i] = src[i];
        at += c;
    }
    __syncthreads();
    uint64_t kth;
    const int n_fin = lds_topk(s_keys, (int)at, p.K, s_sorted, p.k_pad, s_hist, s_misc, s_red, true, kth);
    write_result(s_sorted, n_fin, p.K, p.out_ids + (int64_t)b * p.K, p.out_scores + (int64_t)b * p.K, p.out_count + b);
}

__global__ __launch_bounds__(256) void fill_zero_kernel(uint64_t* __restrict__ dst, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) dst[i] = 0ULL;
}

}  // namespace st
