// Cluster probing in front of the fused search (Sec. 4.2; Sec. 4.3, Alg. 1 phases 1-2).
//
// Items are stored cluster by cluster; cluster c is the item range [off[c], off[c+1]).
// Phase 1 (ivf_probe_kernel): one workgroup per query scores every centroid like an item
// (int8 dot, two fp32 multiplies), and an exact top-n_p by (score descending, cluster id
// ascending) gives the probed clusters.
// Phase 2 (ivf_mask_kernel): 32 threads per (query, probed cluster) run the query's filter
// program only over the words of that cluster's range and ORs the result into the query's row of
// a bit-sliced mask index (zeroed beforehand), laid out like the Bloom index.  Phases 3-4 are the
// ordinary fused scan and selection reading that mask index: items outside the probed ranges have
// mask bit 0 and are never loaded.
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
    const int8_t* q = p.queries + (int64_t)b * p.d;
    const float sq = p.qscale[b];
    uint64_t* keys = p.keys + (int64_t)b * p.n_clusters;
    for (int c = tid; c < p.n_clusters; c += kProbeThreads) {
        const float s = rescale(dot_rows(p.centroids + (int64_t)c * p.d, q, p.d), sq, p.cscale[c]);
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

__global__ __launch_bounds__(256) void fill_zero_kernel(uint64_t* __restrict__ dst, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) dst[i] = 0ULL;
}

}  // namespace st
