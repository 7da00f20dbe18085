// Search kernels: fused Bloom test + compaction + int8 scoring + threshold admission (scan),
// per-query selection of the running top-K (select), and the slow exact path for queries whose
// candidate regions overflowed (rescue).  Paper: Sec. 4.1 (Eq. 4), Sec. 4.2, Sec. 4.3
// (Algorithm 1 phases 3-4), Sec. 5.2.
#pragma once
#include "st_bloom_kernels.h"
#include "st_device.h"
#include "st_plan.h"

namespace st {

constexpr int kScanThreads = 256;
constexpr int kFilterBatch = 16;  // distinct filters handled per pass over a segment

struct ScanParams {
    // Bloom index
    const uint64_t* bloom;
    int32_t m_bits;
    // corpus
    const int8_t* items;
    const float* iscale;
    int64_t n_items;
    int32_t d;
    // queries
    const int8_t* queries;  // [B, T, d]
    const float* qscale;    // [B, T]
    int32_t batch;
    int32_t n_tasks;
    int32_t weighted;       // 0: single task, score = rescale; 1: fmaf chain over tasks
    float w[8];
    // filter groups: queries that share one set of signature rows
    int32_t n_groups;
    const int32_t* grp_row_off;  // [F+1]
    const int32_t* grp_rows;
    const int32_t* grp_q_off;    // [F+1]
    const int32_t* grp_q;        // query indices, grouped
    // level
    int64_t item_begin, item_end;
    int32_t seg_items;
    int32_t seg_per_visit;       // consecutive segments a workgroup takes before striding on
    int32_t use_tau;
    const uint64_t* tau;         // [B]
    // output regions
    uint64_t* cand;              // [B][G][cap]
    uint32_t* cnt;               // [B][G]
    uint32_t* ovf;               // [B]
    int32_t cap;
    int32_t groups;              // G (== gridDim.x)
    int32_t debug_stop;          // TEMP profiling aid
    uint64_t* debug_ts;          // TEMP profiling aid: [level][workgroup][8] timestamps
};

// Score of one (query, item) pair from the item row held by this lane.
__device__ inline float pair_score(const ScanParams& p, int q, const int8_t* item_row, float s_i)
{
    if (!p.weighted)
        return rescale(dot_rows(item_row, p.queries + (int64_t)q * p.d, p.d), p.qscale[q], s_i);
    float agg = 0.0f;
    for (int t = 0; t < p.n_tasks; ++t) {
        const int64_t row = (int64_t)q * p.n_tasks + t;
        const float st = rescale(dot_rows(item_row, p.queries + row * p.d, p.d), p.qscale[row], s_i);
        agg = __fmaf_rn(p.w[t], st, agg);
    }
    return agg;
}

// Admission of a candidate into this workgroup's region for query q.
__device__ inline void admit(const ScanParams& p, uint32_t* cnt_l, int q, uint64_t key)
{
    const uint32_t slot = atomicAdd(&cnt_l[q], 1u);
    if (slot < (uint32_t)p.cap)
        p.cand[((int64_t)q * p.groups + blockIdx.x) * p.cap + slot] = key;
}

// Scan with the wavefront dot-product scorer: one lane per passing item, v_dot4 over the row.
__global__ __launch_bounds__(kScanThreads) void scan_wavedot_kernel(ScanParams p)
{
    extern __shared__ uint32_t cnt_l[];  // [batch] candidates admitted by this workgroup
    __shared__ uint64_t s_mask[kFilterBatch][kTileWords];
    __shared__ uint16_t s_list[kFilterBatch][kTileItems];
    __shared__ int s_listcnt[kFilterBatch];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int q = tid; q < p.batch; q += kScanThreads) cnt_l[q] = 0;
    __syncthreads();

    const int seg_words = p.seg_items >> 6;
    const int64_t n_seg = (p.item_end - p.item_begin + p.seg_items - 1) / p.seg_items;
    const int64_t n_visit = (n_seg + p.seg_per_visit - 1) / p.seg_per_visit;
    const int64_t item_lim = p.item_end < p.n_items ? p.item_end : p.n_items;
    for (int64_t vs = blockIdx.x; vs < n_visit; vs += gridDim.x)
      for (int64_t seg = vs * p.seg_per_visit; seg < (vs + 1) * p.seg_per_visit && seg < n_seg; ++seg) {
        const int64_t item0 = p.item_begin + seg * p.seg_items;
        const int64_t word0 = item0 >> 6;
        for (int g0 = 0; g0 < p.n_groups; g0 += kFilterBatch) {
            const int nf = min(kFilterBatch, p.n_groups - g0);
            // (1) Bloom test: one mask word per (filter, word)
            for (int idx = tid; idx < nf * seg_words; idx += kScanThreads) {
                const int gi = idx / seg_words, w = idx - gi * seg_words;
                const int g = g0 + gi;
                const int r0 = p.grp_row_off[g], r1 = p.grp_row_off[g + 1];
                s_mask[gi][w] = bloom_mask_word(p.bloom, p.m_bits, word0 + w, item_lim,
                                                p.grp_rows + r0, r1 - r0);
            }
            __syncthreads();
            // (2) compaction: the passing items of each filter as a dense list of local indices
            for (int gi = wave; gi < nf; gi += kScanThreads / 64) {
                uint64_t mask = lane < seg_words ? s_mask[gi][lane] : 0ULL;
                const int c = __popcll(mask);
                int incl = c;
                for (int o = 1; o < kTileWords; o <<= 1) {
                    const int v = __shfl_up(incl, o);
                    if (lane >= o) incl += v;
                }
                int pos = incl - c;
                while (mask) {
                    const int b = __ffsll((long long)mask) - 1;
                    mask &= mask - 1;
                    s_list[gi][pos++] = (uint16_t)(lane * 64 + b);
                }
                const int total = __shfl(incl, kTileWords - 1);
                if (lane == 0) s_listcnt[gi] = total;
            }
            __syncthreads();
            // (3) score the passing items against the queries of the filter's group
            for (int gi = 0; gi < nf; ++gi) {
                const int n = s_listcnt[gi];
                const int g = g0 + gi;
                const int qb = p.grp_q_off[g], qe = p.grp_q_off[g + 1];
                for (int b0 = ((wave + gi) & 3) * 64; b0 < n; b0 += kScanThreads) {
                    const int li = b0 + lane;
                    const bool active = li < n;
                    const int64_t item = item0 + (active ? (int)s_list[gi][li] : (int)s_list[gi][0]);
                    const int8_t* row = p.items + item * p.d;
                    const float s_i = p.iscale[item];
                    for (int qi = qb; qi < qe; ++qi) {
                        const int q = p.grp_q[qi];
                        const float s = pair_score(p, q, row, s_i);
                        if (active) {
                            const uint64_t key = make_key(s, (uint32_t)item);
                            if (!p.use_tau || key >= p.tau[q]) admit(p, cnt_l, q, key);
                        }
                    }
                }
            }
            __syncthreads();
        }
    }
    __syncthreads();
    // region fill counts of the queries this launch owns
    const int n_q = p.grp_q_off[p.n_groups];
    for (int i = tid; i < n_q; i += kScanThreads) {
        const int q = p.grp_q[i];
        const uint32_t c = cnt_l[q];
        p.cnt[(int64_t)q * p.groups + blockIdx.x] = c < (uint32_t)p.cap ? c : (uint32_t)p.cap;
        if (c > (uint32_t)p.cap) p.ovf[q] = 1u;
    }
}

// ------------------------------------------------------------------------------------------
// Workgroup-wide exact top-K of n distinct 64-bit keys in buf (LDS or global memory), K >= 1.
// On return sorted[0 .. min(n,K)) holds the best keys in descending order (sorted may be LDS or
// global, k_pad = power of two >= K entries).  A radix select finds the K-th largest key eight
// bits at a time -- starting below the bits all keys share, stopping as soon as a whole bucket is
// needed -- then the keys at or above it are collected and a bitonic network orders them.
// All threads of the workgroup must call it; uses s_hist (256 words), s_misc (8 words) and
// s_red (2 x 8 64-bit words) of LDS.
__device__ inline int wg_topk(const uint64_t* buf, int64_t n, int K, uint64_t* sorted, int k_pad,
                              uint32_t* s_hist, uint32_t* s_misc, uint64_t* s_red)
{
    const int tid = threadIdx.x, nt = blockDim.x;
    const int n_out = n < (int64_t)K ? (int)n : K;
    // power-of-two size the sorting network runs on
    int P = 1;
    while (P < n_out) P <<= 1;
    if (P > k_pad) P = k_pad;
    if (n <= (int64_t)K) {
        for (int i = tid; i < P; i += nt) sorted[i] = i < n_out ? buf[i] : 0ULL;
    } else {
        // bits shared by every key need no pass: find the highest byte in which two keys differ
        uint64_t lo = ~0ULL, hi = 0ULL;
        for (int64_t i = tid; i < n; i += nt) {
            const uint64_t key = buf[i];
            lo = key < lo ? key : lo;
            hi = key > hi ? key : hi;
        }
        for (int o = 32; o > 0; o >>= 1) {
            const uint64_t l2 = __shfl_xor((unsigned long long)lo, o), h2 = __shfl_xor((unsigned long long)hi, o);
            lo = l2 < lo ? l2 : lo;
            hi = h2 > hi ? h2 : hi;
        }
        if ((tid & 63) == 0) { s_red[(tid >> 6) * 2] = lo; s_red[(tid >> 6) * 2 + 1] = hi; }
        __syncthreads();
        for (int w = 0; w < (nt >> 6); ++w) {
            const uint64_t l2 = s_red[2 * w], h2 = s_red[2 * w + 1];
            lo = l2 < lo ? l2 : lo;
            hi = h2 > hi ? h2 : hi;
        }
        const int top_shift = 56 - (__clzll((long long)(lo ^ hi)) >> 3) * 8;  // n > K >= 1: lo != hi
        uint64_t prefix_mask = top_shift == 56 ? 0ULL : ~((1ULL << (top_shift + 8)) - 1ULL);
        uint64_t prefix = hi & prefix_mask;
        uint32_t want = (uint32_t)K;  // rank (1-based, from the top) still to locate inside the prefix bucket
        for (int shift = top_shift; shift >= 0; shift -= 8) {
            for (int i = tid; i < 256; i += nt) s_hist[i] = 0;
            __syncthreads();
            for (int64_t i = tid; i < n; i += nt) {
                const uint64_t key = buf[i];
                if ((key & prefix_mask) == prefix) atomicAdd(&s_hist[(key >> shift) & 255], 1u);
            }
            __syncthreads();
            if (tid < 64) {
                // lane l owns digits 255-4l .. 252-4l (descending); find the digit where the
                // running count from the top reaches `want`
                const int l = tid;
                uint32_t h[4], sum = 0;
                for (int j = 0; j < 4; ++j) { h[j] = s_hist[255 - 4 * l - j]; sum += h[j]; }
                uint32_t incl = sum;
                for (int o = 1; o < 64; o <<= 1) {
                    const uint32_t v = __shfl_up(incl, o);
                    if (l >= o) incl += v;
                }
                uint32_t before = incl - sum;  // keys in digits above this lane's four
                if (before < want && want <= incl) {
                    for (int j = 0; j < 4; ++j) {
                        if (want <= before + h[j]) {
                            s_misc[0] = (uint32_t)(255 - 4 * l - j);
                            s_misc[1] = want - before;
                            s_misc[3] = (want - before == h[j]) ? 1u : 0u;  // the whole bucket is needed
                            break;
                        }
                        before += h[j];
                    }
                }
            }
            __syncthreads();
            prefix |= (uint64_t)s_misc[0] << shift;
            prefix_mask |= 0xFFULL << shift;
            want = s_misc[1];
            const bool done = s_misc[3] != 0u;
            __syncthreads();
            if (done) break;
        }
        const uint64_t kth = prefix;  // keys are distinct: exactly K of them are >= kth
        if (tid == 0) s_misc[2] = 0;
        __syncthreads();
        for (int64_t i = tid; i < n; i += nt) {
            const uint64_t key = buf[i];
            if (key >= kth) {
                const uint32_t slot = atomicAdd(&s_misc[2], 1u);
                if (slot < (uint32_t)P) sorted[slot] = key;
            }
        }
        for (int i = K + tid; i < P; i += nt) sorted[i] = 0ULL;
    }
    __syncthreads();
    if (P <= nt) {
        // few keys: every thread ranks its key against all the others (no barriers per stage);
        // padding zeros tie among themselves and are ordered by position
        uint64_t key = 0;
        int rank = 0;
        if (tid < P) {
            key = sorted[tid];
            for (int j = 0; j < P; ++j) {
                const uint64_t o = sorted[j];
                rank += (o > key || (o == key && j < tid)) ? 1 : 0;
            }
        }
        __syncthreads();
        if (tid < P) sorted[rank] = key;
        __syncthreads();
        return n_out;
    }
    for (int k2 = 2; k2 <= P; k2 <<= 1) {
        for (int j = k2 >> 1; j > 0; j >>= 1) {
            for (int i = tid; i < P; i += nt) {
                const int x = i ^ j;
                if (x > i) {
                    const uint64_t a = sorted[i], b = sorted[x];
                    const bool desc = (i & k2) == 0;
                    if (desc ? (a < b) : (a > b)) { sorted[i] = b; sorted[x] = a; }
                }
            }
            __syncthreads();
        }
    }
    return n_out;
}

// Writes one query's result row from sorted keys, padding with id -1 / score -inf.
__device__ inline void write_result(const uint64_t* sorted, int n_out, int K, int64_t* out_ids,
                                    float* out_scores, int32_t* out_count)
{
    for (int i = threadIdx.x; i < K; i += blockDim.x) {
        if (i < n_out) {
            out_ids[i] = (int64_t)key_item(sorted[i]);
            out_scores[i] = key_score(sorted[i]);
        } else {
            out_ids[i] = -1;
            out_scores[i] = -__builtin_inff();
        }
    }
    if (threadIdx.x == 0) *out_count = n_out;
}

struct SelectParams {
    const uint64_t* cand;   // [B][G][cap]
    const uint32_t* cnt;    // [B][G]
    int32_t cap, groups;
    int32_t regions;        // regions the scan launches of this level wrote (a prefix of the G)
    uint64_t* topk_keys;    // [B][K] running top-K (read when !first, always written)
    uint32_t* topk_cnt;     // [B]
    uint64_t* gath;         // [B][gath_cap]
    int64_t gath_cap;
    uint64_t* srt;          // [B][k_pad] or null (sort in LDS)
    int32_t K, k_pad;
    uint64_t* tau;          // [B] out
    uint64_t* tau_img;      // thresholds in the order of the scorer's resident query image, or null
    const int32_t* q_taupos;  // [B] position of each query in tau_img (-1: none)
    uint32_t* ovf;          // [B]
    int32_t first, last;
    int64_t* out_ids;       // [B][K]
    float* out_scores;
    int32_t* out_count;
    // slow exact path (last level only): corpus, queries, all filter groups
    ScanParams scan;
    const int32_t* q2grp;   // [B] group of each query
};

constexpr int kSelectThreads = 512;
constexpr int kLdsKeys = 4096;  // candidates per query gathered in LDS; more go through global memory

// Slow exact path for a query whose candidate region overflowed in some level: rescans the whole
// corpus for that query alone, keeping at most gath_cap keys and pruning to the best K whenever
// the buffer cannot take another tile.  Called by the whole workgroup.
__device__ inline void rescue_query(const SelectParams& r, int q, uint64_t* s_sorted, uint32_t* s_hist,
                                    uint32_t* s_misc, uint64_t* s_red, uint64_t* s_mask, uint32_t* s_n)
{
    const int tid = threadIdx.x, nt = blockDim.x;
    const ScanParams& p = r.scan;
    const int g = r.q2grp[q];
    const int r0 = p.grp_row_off[g], r1 = p.grp_row_off[g + 1];
    uint64_t* buf = r.gath + (int64_t)q * r.gath_cap;
    uint64_t* sorted = r.srt ? r.srt + (int64_t)q * r.k_pad : s_sorted;
    uint64_t tau = 0;
    if (tid == 0) *s_n = 0;
    __syncthreads();
    const int64_t n_tiles = (p.n_items + kTileItems - 1) / kTileItems;
    for (int64_t tile = 0; tile < n_tiles; ++tile) {
        if ((int64_t)*s_n + kTileItems > r.gath_cap) {  // uniform: *s_n is stable between barriers
            const int n_out = wg_topk(buf, (int64_t)*s_n, r.K, sorted, r.k_pad, s_hist, s_misc, s_red);
            for (int i = tid; i < n_out; i += nt) buf[i] = sorted[i];
            tau = n_out == r.K ? sorted[r.K - 1] : 0ULL;
            __syncthreads();
            if (tid == 0) *s_n = (uint32_t)n_out;
            __syncthreads();
        }
        if (tid < kTileWords)
            s_mask[tid] = bloom_mask_word(p.bloom, p.m_bits, tile * kTileWords + tid, p.n_items,
                                          p.grp_rows + r0, r1 - r0);
        __syncthreads();
        for (int loc = tid; loc < kTileItems; loc += nt) {
            if ((s_mask[loc >> 6] >> (loc & 63)) & 1ULL) {
                const int64_t item = tile * kTileItems + loc;
                const float sc = pair_score(p, q, p.items + item * p.d, p.iscale[item]);
                const uint64_t key = make_key(sc, (uint32_t)item);
                if (key >= tau) buf[atomicAdd(s_n, 1u)] = key;
            }
        }
        __syncthreads();
    }
    const int n_out = wg_topk(buf, (int64_t)*s_n, r.K, sorted, r.k_pad, s_hist, s_misc, s_red);
    write_result(sorted, n_out, r.K, r.out_ids + (int64_t)q * r.K, r.out_scores + (int64_t)q * r.K,
                 r.out_count + q);
}

// One workgroup per query: gather the regions (and the running top-K) into a contiguous array
// (LDS when it fits), select and sort the best K, publish the K-th key as the next admission
// threshold.  On the last level it writes the result rows, through the slow exact path if one
// of the query's regions overflowed.
__global__ __launch_bounds__(kSelectThreads) void select_kernel(SelectParams p)
{
    __shared__ uint64_t s_keys[kLdsKeys];
    __shared__ uint64_t s_sorted[kLdsSortMax];
    __shared__ uint64_t s_red[2 * kSelectThreads / 64];
    __shared__ uint64_t s_mask[kTileWords];
    __shared__ uint32_t s_hist[256];
    __shared__ uint32_t s_misc[8];
    __shared__ uint32_t s_scan[kSelectThreads];
    __shared__ uint32_t s_off[kMaxScanGroups + 1];
    const int q = blockIdx.x, tid = threadIdx.x;
    constexpr int NT = kSelectThreads;
    // counts are clamped to what the buffers can hold, whatever the memory says
    uint32_t n_prev = p.first ? 0u : p.topk_cnt[q];
    n_prev = n_prev < (uint32_t)p.K ? n_prev : (uint32_t)p.K;
    const bool overflowed = !p.first && p.ovf[q] != 0u;
    if (p.first && tid == 0) p.ovf[q] = 0u;
    if (p.last && overflowed) {  // uniform over the workgroup
        rescue_query(p, q, s_sorted, s_hist, s_misc, s_red, s_mask, &s_misc[4]);
        return;
    }

    // exclusive prefix sum of the region counts, NT threads x ceil(regions/NT) regions each
    const int R = p.regions;
    const int per = (R + NT - 1) / NT;
    const uint32_t* cq = p.cnt + (int64_t)q * p.groups;
    uint32_t mine = 0;
    for (int j = 0; j < per; ++j) {
        const int w = tid * per + j;
        if (w < R) mine += min(cq[w], (uint32_t)p.cap);
    }
    s_scan[tid] = mine;
    __syncthreads();
    for (int o = 1; o < NT; o <<= 1) {
        const uint32_t v = tid >= o ? s_scan[tid - o] : 0u;
        __syncthreads();
        s_scan[tid] += v;
        __syncthreads();
    }
    const uint32_t total = n_prev + s_scan[NT - 1];
    const bool in_lds = total <= (uint32_t)kLdsKeys;
    uint64_t* gkeys = p.gath + (int64_t)q * p.gath_cap;
    {
        // each thread copies the entries of its own regions (loads independent of each other)
        uint32_t off = n_prev + s_scan[tid] - mine;
        for (int j = 0; j < per; ++j) {
            const int w = tid * per + j;
            if (w < R) {
                const uint32_t c = min(cq[w], (uint32_t)p.cap);
                const uint64_t* src = p.cand + ((int64_t)q * p.groups + w) * p.cap;
                for (uint32_t i0 = 0; i0 < c; i0 += 4) {
                    uint64_t v[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (i0 + u < c) v[u] = src[i0 + u];
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (i0 + u < c) {
                            if (in_lds) s_keys[off + i0 + u] = v[u];
                            else gkeys[off + i0 + u] = v[u];
                        }
                }
                off += c;
            }
        }
    }
    for (int i = tid; i < (int)n_prev; i += NT) {
        const uint64_t v = p.topk_keys[(int64_t)q * p.K + i];
        if (in_lds) s_keys[i] = v;
        else gkeys[i] = v;
    }
    __syncthreads();

    const uint64_t* keys = in_lds ? s_keys : gkeys;
    uint64_t* sorted = p.srt ? p.srt + (int64_t)q * p.k_pad : s_sorted;
    const int n_out = wg_topk(keys, (int64_t)total, p.K, sorted, p.k_pad, s_hist, s_misc, s_red);
    if (!p.last) {
        for (int i = tid; i < n_out; i += NT) p.topk_keys[(int64_t)q * p.K + i] = sorted[i];
        if (tid == 0) {
            const uint64_t t64 = n_out == p.K ? sorted[p.K - 1] : 0ULL;
            p.topk_cnt[q] = (uint32_t)n_out;
            p.tau[q] = t64;
            if (p.tau_img) {
                const int pos = p.q_taupos[q];
                if (pos >= 0) p.tau_img[pos] = t64;
            }
        }
    } else {
        write_result(sorted, n_out, p.K, p.out_ids + (int64_t)q * p.K, p.out_scores + (int64_t)q * p.K,
                     p.out_count + q);
    }
}

// Parity export of the scoring arithmetic for chosen pairs.
__global__ __launch_bounds__(256) void score_pairs_kernel(const int8_t* __restrict__ items,
                                                          const float* __restrict__ iscale, int32_t d,
                                                          const int8_t* __restrict__ queries,
                                                          const float* __restrict__ qscale,
                                                          const int64_t* __restrict__ pair_item,
                                                          const int32_t* __restrict__ pair_query,
                                                          int64_t n_pairs, int32_t* out_dot,
                                                          float* out_score)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_pairs) return;
    const int64_t item = pair_item[i];
    const int q = pair_query[i];
    const int dot = dot_rows(items + item * d, queries + (int64_t)q * d, d);
    if (out_dot) out_dot[i] = dot;
    if (out_score) out_score[i] = rescale(dot, qscale[q], iscale[item]);
}

}  // namespace st
