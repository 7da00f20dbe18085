// Search kernels: fused Bloom test + compaction + int8 scoring + threshold admission (scan),
// per-query selection of the running top-K (select), and the slow exact path for queries whose
// candidate regions overflowed (rescue).  Paper: Sec. 4.1 (Eq. 4), Sec. 4.2, Sec. 4.3
// (Algorithm 1 phases 3-4), Sec. 5.2.
#pragma once
#include <atomic>

#include "st_bloom_kernels.h"
#include "st_device.h"
#include "st_plan.h"
#include "st_scan_params.h"

namespace st {

constexpr int kScanThreads = 256;
constexpr int kFilterBatch = 16;  // distinct filters handled per pass over a segment

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

// Dot products of the item row this lane holds with NR query rows whose addresses are the same in
// every lane: the item row is read once, the query chunks come through the scalar cache (the
// queries are read-only for the whole search, which the constant address space tells the compiler).
constexpr int kRowBlock = 8;
template <int NR>
__device__ inline void dot_block(const int4* item, const int8_t* queries, const int64_t (&qoff)[kRowBlock],
                                 int chunks, int (&acc)[kRowBlock])
{
    typedef int Int4 __attribute__((ext_vector_type(4)));
    typedef const Int4 __attribute__((address_space(4))) * ConstRow;
    constexpr int kUnroll = NR > 4 ? 2 : 4;  // chunks in flight: bounded by the scalar registers
#pragma unroll kUnroll
    for (int c = 0; c < chunks; ++c) {
        const int4 v = item[c];
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            const ConstRow qr = (ConstRow)(uintptr_t)(queries + qoff[r]);
            const Int4 qv = qr[c];
            acc[r] = dot16(v, make_int4(qv.x, qv.y, qv.z, qv.w), acc[r]);
        }
    }
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
    extern __shared__ uint32_t cnt_l[];  // [batch] candidates admitted by this workgroup, then [batch] 64-bit thresholds
    __shared__ uint64_t s_mask[kFilterBatch][kTileWords];
    __shared__ uint16_t s_list[kFilterBatch][kTileItems];
    __shared__ int s_listcnt[kFilterBatch];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint64_t* tau_l = reinterpret_cast<uint64_t*>(cnt_l + ((p.batch + 1) & ~1));
    for (int q = tid; q < p.batch; q += kScanThreads) {
        cnt_l[q] = 0;
        uint64_t t = 0;
        if (p.use_tau) {
            t = ~0ULL;
            for (int pp = 0; pp < p.tau_parts; ++pp) t = min(t, p.tau[(int64_t)q * kTauParts + pp]);
        }
        tau_l[q] = t;
    }
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
                // (the words of a tile sit in the first 16 lanes: one row, register moves)
                static_assert(kTileWords == 16, "the prefix sum below covers one row of 16 lanes");
                int incl = c;
                incl += (int)row_shr<1>((uint32_t)incl);
                incl += (int)row_shr<2>((uint32_t)incl);
                incl += (int)row_shr<4>((uint32_t)incl);
                incl += (int)row_shr<8>((uint32_t)incl);
                int pos = incl - c;
                while (mask) {
                    const int b = __ffsll((long long)mask) - 1;
                    mask &= mask - 1;
                    s_list[gi][pos++] = (uint16_t)(lane * 64 + b);
                }
                const int total = (int)lane_value((uint32_t)incl, kTileWords - 1);
                if (lane == 0) s_listcnt[gi] = total;
            }
            __syncthreads();
            // (3) score the passing items against the queries of the filter's group: a lane holds
            // one item row and takes up to eight query rows per pass over it
            const int qpp = p.n_tasks >= kRowBlock ? 1 : kRowBlock / p.n_tasks;  // queries per pass
            for (int gi = 0; gi < nf; ++gi) {
                const int n = s_listcnt[gi];
                const int g = g0 + gi;
                const int qb = p.grp_q_off[g], qe = p.grp_q_off[g + 1];
                for (int b0 = ((wave + gi) & 3) * 64; b0 < n; b0 += kScanThreads) {
                    const int li = b0 + lane;
                    const bool active = li < n;
                    const int64_t item = item0 + (active ? (int)s_list[gi][li] : (int)s_list[gi][0]);
                    const int4* row = reinterpret_cast<const int4*>(p.items + item * p.d);
                    const float s_i = p.iscale[item];
                    for (int q0 = qb; q0 < qe; q0 += qpp) {
                        const int nq = min(qpp, qe - q0);
                        const int nr = nq * p.n_tasks;
                        // rows past the pass's last one repeat row 0 (their sums are not used)
                        int64_t qoff[kRowBlock];
#pragma unroll
                        for (int r = 0; r < kRowBlock; ++r) {
                            const int rr = r < nr ? r : 0;
                            const int j = rr / p.n_tasks, t = rr - j * p.n_tasks;
                            qoff[r] = ((int64_t)p.grp_q[q0 + j] * p.n_tasks + t) * p.d;
                        }
                        int acc[kRowBlock];
#pragma unroll
                        for (int r = 0; r < kRowBlock; ++r) acc[r] = 0;
                        if (nr == 1) dot_block<1>(row, p.queries, qoff, p.d >> 4, acc);
                        else if (nr == 2) dot_block<2>(row, p.queries, qoff, p.d >> 4, acc);
                        else if (nr <= 4) dot_block<4>(row, p.queries, qoff, p.d >> 4, acc);
                        else dot_block<kRowBlock>(row, p.queries, qoff, p.d >> 4, acc);
                        // rows in order: the tasks of a query are consecutive, and its aggregate
                        // is complete after the last of them
                        float agg = 0.0f;
                        int t = 0, j = 0;
#pragma unroll
                        for (int r = 0; r < kRowBlock; ++r) {
                            if (r < nr) {
                                const int q = p.grp_q[q0 + j];
                                const float st = rescale(acc[r], p.qscale[(int64_t)q * p.n_tasks + t], s_i);
                                agg = p.weighted ? __fmaf_rn(p.w[t], st, agg) : st;
                                if (++t == p.n_tasks) {
                                    if (active) {
                                        const uint64_t key = make_key(agg, (uint32_t)item);
                                        if (key >= tau_l[q]) admit(p, cnt_l, q, key);
                                    }
                                    agg = 0.0f;
                                    t = 0;
                                    ++j;
                                }
                            }
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
// With want_sorted = false the bitonic network is skipped: sorted[0 .. min(n,K)) then holds the
// best keys in no particular order (a caller that only carries the set forward needs no order),
// and *kth_out, if given, receives the K-th best key (0 if n < K) in either mode.
__device__ inline int wg_topk(const uint64_t* buf, int64_t n, int K, uint64_t* sorted, int k_pad,
                              uint32_t* s_hist, uint32_t* s_misc, uint64_t* s_red, bool want_sorted = true,
                              uint64_t* kth_out = nullptr)
{
    const int tid = threadIdx.x, nt = blockDim.x;
    const int n_out = n < (int64_t)K ? (int)n : K;
    uint64_t low = ~0ULL;  // smallest key this thread put into sorted[]
    // f(key) for every key of buf, this thread's share: eight loads are requested before the first
    // is used (one memory round trip per eight keys instead of one per key)
    auto for_each = [&](auto&& f) {
        constexpr int U = 8;
        int64_t i = tid;
        for (; i + (int64_t)(U - 1) * nt < n; i += (int64_t)U * nt) {
            uint64_t v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = buf[i + (int64_t)u * nt];
#pragma unroll
            for (int u = 0; u < U; ++u) f(v[u]);
        }
        for (; i < n; i += nt) f(buf[i]);
    };
    // power-of-two size the sorting network runs on
    int P = 1;
    while (P < n_out) P <<= 1;
    if (P > k_pad) P = k_pad;
    if (n <= (int64_t)K) {
        for (int i = tid; i < P; i += nt) {
            const uint64_t key = i < n_out ? buf[i] : 0ULL;
            sorted[i] = key;
            if (i < n_out && key < low) low = key;
        }
    } else {
        // bits shared by every key need no pass: find the highest byte in which two keys differ
        uint64_t lo = ~0ULL, hi = 0ULL;
        for_each([&](uint64_t key) {
            lo = key < lo ? key : lo;
            hi = key > hi ? key : hi;
        });
        lo = ~wave_max_u64(~lo);  // (both in lane 63)
        hi = wave_max_u64(hi);
        if ((tid & 63) == 63) { s_red[(tid >> 6) * 2] = lo; s_red[(tid >> 6) * 2 + 1] = hi; }
        __syncthreads();
        for (int w = 0; w < (nt >> 6); ++w) {
            const uint64_t l2 = s_red[2 * w], h2 = s_red[2 * w + 1];
            lo = l2 < lo ? l2 : lo;
            hi = h2 > hi ? h2 : hi;
        }
        // The first digit starts at the highest bit in which two keys differ (not at a byte boundary:
        // a digit with a few distinct values sends all keys to a few counters, and updates of one
        // LDS word are served one after the other); the last one may overlap bits already fixed.
        const int top_bit = 63 - __clzll((long long)(lo ^ hi));  // n > K >= 1: lo != hi
        const int top_shift = top_bit >= 7 ? top_bit - 7 : 0;
        uint64_t prefix_mask = top_shift == 56 ? 0ULL : ~((1ULL << (top_shift + 8)) - 1ULL);
        uint64_t prefix = hi & prefix_mask;
        uint32_t want = (uint32_t)K;  // rank (1-based, from the top) still to locate inside the prefix bucket
        for (int shift = top_shift;; shift = shift >= 8 ? shift - 8 : 0) {
            for (int i = tid; i < 256; i += nt) s_hist[i] = 0;
            __syncthreads();
            for_each([&](uint64_t key) {
                if ((key & prefix_mask) == prefix) atomicAdd(&s_hist[(key >> shift) & 255], 1u);
            });
            __syncthreads();
            if (tid < 64) {
                // lane l owns digits 255-4l .. 252-4l (descending); find the digit where the
                // running count from the top reaches `want`
                const int l = tid;
                uint32_t h[4], sum = 0;
                for (int j = 0; j < 4; ++j) { h[j] = s_hist[255 - 4 * l - j]; sum += h[j]; }
                const uint32_t incl = wave_scan_add(sum);
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
            if (done || shift == 0) break;
        }
        const uint64_t kth = prefix;  // keys are distinct: exactly K of them are >= kth
        if (tid == 0) s_misc[2] = 0;
        __syncthreads();
        for_each([&](uint64_t key) {
            if (key >= kth) {
                const uint32_t slot = atomicAdd(&s_misc[2], 1u);
                if (slot < (uint32_t)P) sorted[slot] = key;
                if (key < low) low = key;
            }
        });
        for (int i = K + tid; i < P; i += nt) sorted[i] = 0ULL;
    }
    __syncthreads();
    if (kth_out) {
        // the K-th best key is the smallest one kept (keys are distinct), when there are K of them
        low = ~wave_max_u64(~low);  // (in lane 63)
        if ((tid & 63) == 63) s_red[tid >> 6] = low;
        __syncthreads();
        for (int w = 0; w < (nt >> 6); ++w) low = s_red[w] < low ? s_red[w] : low;
        *kth_out = n_out == K ? low : 0ULL;
        __syncthreads();
    }
    if (!want_sorted) return n_out;
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

// Descending bitonic sort of P keys in global memory (P a power of two above C) by one workgroup,
// blocked through an LDS buffer of C keys (C a power of two): every stage whose partner distance
// is below C runs on chunks held in LDS, only the log2(P / C) * (log2(P / C) + 1) / 2 stages at
// distance C and above touch global memory.  All threads of the workgroup must call it.
__device__ inline void blocked_bitonic_desc(uint64_t* g, int P, uint64_t* chunk, int C)
{
    const int tid = threadIdx.x, nt = blockDim.x;
    auto lds_stages = [&](int c0, int k2, int j_first) {  // stages j_first .. 1 of merge size k2 on the chunk at c0
        for (int j = j_first; j > 0; j >>= 1) {
            for (int i = tid; i < C; i += nt) {
                const int x = i ^ j;
                if (x > i) {
                    const uint64_t a = chunk[i], b = chunk[x];
                    const bool desc = ((c0 + i) & k2) == 0;
                    if (desc ? (a < b) : (a > b)) { chunk[i] = b; chunk[x] = a; }
                }
            }
            __syncthreads();
        }
    };
    for (int c0 = 0; c0 < P; c0 += C) {
        for (int i = tid; i < C; i += nt) chunk[i] = g[c0 + i];
        __syncthreads();
        for (int k2 = 2; k2 <= C; k2 <<= 1) lds_stages(c0, k2, k2 >> 1);
        for (int i = tid; i < C; i += nt) g[c0 + i] = chunk[i];
        __syncthreads();
    }
    for (int k2 = 2 * C; k2 <= P; k2 <<= 1) {
        for (int j = k2 >> 1; j >= C; j >>= 1) {
            for (int i = tid; i < P; i += nt) {
                const int x = i ^ j;
                if (x > i) {
                    const uint64_t a = g[i], b = g[x];
                    const bool desc = (i & k2) == 0;
                    if (desc ? (a < b) : (a > b)) { g[i] = b; g[x] = a; }
                }
            }
            __syncthreads();
        }
        for (int c0 = 0; c0 < P; c0 += C) {
            for (int i = tid; i < C; i += nt) chunk[i] = g[c0 + i];
            __syncthreads();
            lds_stages(c0, k2, C >> 1);
            for (int i = tid; i < C; i += nt) g[c0 + i] = chunk[i];
            __syncthreads();
        }
    }
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

// Faster variant for keys that sit in LDS and fit in registers: every thread keeps up to
// kTopkRegs keys in registers for all passes; a pass costs one barrier (three histograms rotate,
// every wavefront scans the histogram for itself).  Requires n <= kTopkRegs * blockDim.x,
// blockDim.x a multiple of 256 and at most 1024, k_pad <= room in sorted (LDS).  The key buffer
// is overwritten (it serves as scratch once the keys sit in registers).
//
// The key buffer must hold max(n, 1024) entries (the final ordering of 512 keys uses it as scratch).
//
// kth receives the K-th best key (0 if n < K).  With want_sorted the best min(n, K) keys end up
// in sorted[] in descending order; without, they are there in no particular order (callers that
// only carry the set forward and need the threshold skip the sort).
constexpr int kTopkRegs = 16;

__device__ inline int lds_topk(uint64_t* keys, int n, int K, uint64_t* sorted, int k_pad,
                               uint32_t* s_hist3 /*[3][256]*/, uint32_t* s_misc /*[8]*/, uint64_t* s_red /*[2*16]*/,
                               bool want_sorted, uint64_t& kth)
{
    const int tid = threadIdx.x, nt = blockDim.x, lane = tid & 63, wv = tid >> 6, nw = nt >> 6;
    const int n_out = n < K ? n : K;
    int P = 1;
    while (P < n_out) P <<= 1;
    if (P > k_pad) P = k_pad;
    kth = 0;
    if (n <= K) {
        for (int i = tid; i < P; i += nt) sorted[i] = i < n_out ? keys[i] : 0ULL;
        __syncthreads();
        if (n < K && !want_sorted) return n_out;
        want_sorted = true;  // n == K: the threshold is the smallest key, read off the sorted list
    } else {
        uint64_t kr[kTopkRegs];
        const uint64_t k0 = keys[0];
        uint64_t diff = 0;  // bits in which some key differs from the first
        const int ne = (n + nt - 1) / nt;  // register slots in use (uniform)
#pragma unroll
        for (int j = 0; j < kTopkRegs; ++j) {
            const int i = tid + j * nt;
            kr[j] = i < n ? keys[i] : 0ULL;  // 0 is below every real key
            if (i < n) diff |= kr[j] ^ k0;
        }
        const uint32_t dl = wave_or_u32((uint32_t)diff), dh = wave_or_u32((uint32_t)(diff >> 32));
        if (lane == 63) s_red[wv] = ((uint64_t)dh << 32) | dl;
        for (int i = tid; i < 3 * 256; i += nt) s_hist3[i] = 0;
        if (tid == 0) s_misc[2] = 0;
        __syncthreads();
        diff = 0;
        for (int w = 0; w < nw; ++w) diff |= s_red[w];
        // (first digit from the highest differing bit, last one overlapping, as in wg_topk)
        const int top_bit = 63 - __clzll((long long)diff);  // n > K >= 1 distinct keys: diff != 0
        const int top_shift = top_bit >= 7 ? top_bit - 7 : 0;
        uint64_t prefix_mask = top_shift == 56 ? 0ULL : ~((1ULL << (top_shift + 8)) - 1ULL);
        uint64_t prefix = k0 & prefix_mask;
        uint32_t want = (uint32_t)K;
        int pass = 0;
        for (int shift = top_shift;; shift = shift >= 8 ? shift - 8 : 0, ++pass) {
            uint32_t* hist = s_hist3 + (pass % 3) * 256;
#pragma unroll
            for (int j = 0; j < kTopkRegs; ++j)
                if (j < ne && kr[j] && (kr[j] & prefix_mask) == prefix) atomicAdd(&hist[(kr[j] >> shift) & 255], 1u);
            // clear the next pass's histogram: its last readers (two passes ago) were done before the
            // previous barrier, whereas the one scanned in the previous pass may still be being read
            uint32_t* stale = s_hist3 + ((pass + 1) % 3) * 256;
            if (tid < 256) stale[tid] = 0;
            __syncthreads();
            // every wavefront: lane l owns digits 255-4l .. 252-4l (descending)
            uint32_t h[4], sum = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) { h[j] = hist[255 - 4 * lane - j]; sum += h[j]; }
            const uint32_t incl = wave_scan_add(sum);
            uint32_t before = incl - sum;
            const bool mine = before < want && want <= incl;
            uint32_t digit = 0, rest = 0, whole = 0;
            if (mine) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (want > before && want <= before + h[j]) {
                        digit = (uint32_t)(255 - 4 * lane - j);
                        rest = want - before;
                        whole = rest == h[j] ? 1u : 0u;
                    }
                    before += h[j];
                }
            }
            const int src = __ffsll((long long)ballot(mine)) - 1;  // exactly one lane
            digit = lane_value(digit, src);
            rest = lane_value(rest, src);
            whole = lane_value(whole, src);
            prefix |= (uint64_t)digit << shift;
            prefix_mask |= 0xFFULL << shift;
            want = rest;
            if (whole || shift == 0) break;  // uniform: every wavefront computed the same
        }
        // keys are distinct: exactly K of them are >= prefix; when the search stopped on a whole
        // bucket the K-th key is the smallest of them
        const uint64_t bound = prefix;
        uint64_t low = ~0ULL;
#pragma unroll
        for (int j = 0; j < kTopkRegs; ++j)
            if (j < ne && kr[j] >= bound && kr[j]) {
                const uint32_t slot = atomicAdd(&s_misc[2], 1u);
                if (slot < (uint32_t)P) sorted[slot] = kr[j];
                low = kr[j] < low ? kr[j] : low;
            }
        for (int i = K + tid; i < P; i += nt) sorted[i] = 0ULL;
        if (!want_sorted) {
            // threshold = smallest collected key: wavefront minimum, then across wavefronts
            const uint64_t wave_low = ~wave_max_u64(~low);  // (lanes without a key hold ~0)
            if (lane == 63) s_red[16 + wv] = wave_low;
        }
        __syncthreads();
        if (!want_sorted) {
            uint64_t m = ~0ULL;
            for (int w = 0; w < nw; ++w) m = s_red[16 + w] < m ? s_red[16 + w] : m;
            kth = m;
            return n_out;
        }
    }
    if (P <= nt && P > 256) {
        // One key per thread, bitonic network (descending; the padding zeros sink to the end).  The
        // exchange partner sits in the same wavefront for distances below 64 (two 32-bit shuffles:
        // exchanges by register moves measured slower here, the independent shuffles of a stage overlap),
        // beyond that the keys go through LDS with one barrier per stage (two buffers alternate).
        // 45 stages for 512 keys, 6 of them through LDS: a rank sort reads every key in every
        // thread instead, 2 MB of LDS traffic for 512 keys.
        uint64_t* bufs[2] = {keys, keys + P};  // the key buffer is free once the keys sit in `sorted`
        uint64_t key = tid < P ? sorted[tid] : 0ULL;
        int flip = 0;
        for (int k2 = 2; k2 <= P; k2 <<= 1) {
            const bool desc = (tid & k2) == 0;
            for (int j = k2 >> 1; j > 0; j >>= 1) {
                uint64_t other;
                if (j >= 64) {
                    if (tid < P) bufs[flip][tid] = key;
                    __syncthreads();
                    other = tid < P ? bufs[flip][tid ^ j] : 0ULL;
                    flip ^= 1;
                } else {
                    const uint32_t ol = __shfl_xor((uint32_t)key, j), oh = __shfl_xor((uint32_t)(key >> 32), j);
                    other = ((uint64_t)oh << 32) | ol;
                }
                const bool lower = (tid & j) == 0;          // the lower index of the pair
                const bool want_max = lower == desc;        // descending run: the lower index keeps the larger key
                const bool take = want_max ? other > key : other < key;
                key = take ? other : key;
            }
        }
        __syncthreads();
        if (tid < P) sorted[tid] = key;
        __syncthreads();
        if (n_out == K) kth = sorted[K - 1];
        return n_out;
    }
    if (P <= nt) {
        // rank sort with every thread at work: thread (c, i) counts, among one share of the list,
        // the keys that precede key i; shares are summed in LDS (padding zeros tie among
        // themselves and are ordered by position)
        uint32_t* s_rank = reinterpret_cast<uint32_t*>(keys);
        int chunks = nt / P;
        if (chunks > P) chunks = P;
        const int seg = P / chunks;
        const int i = tid % P, c = tid / P;
        if (tid < P) s_rank[tid] = 0;
        __syncthreads();
        uint64_t key = 0;
        if (c < chunks) {
            key = sorted[i];
            int rank = 0;
            const int j0 = c * seg;
            if (seg >= 8) {
                for (int j = j0; j < j0 + seg; j += 8) {  // eight reads in flight at a time
                    uint64_t o[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) o[u] = sorted[j + u];
#pragma unroll
                    for (int u = 0; u < 8; ++u) rank += (o[u] > key || (o[u] == key && j + u < i)) ? 1 : 0;
                }
            } else {
                for (int j = j0; j < j0 + seg; ++j) {
                    const uint64_t o = sorted[j];
                    rank += (o > key || (o == key && j < i)) ? 1 : 0;
                }
            }
            if (rank) atomicAdd(&s_rank[i], (uint32_t)rank);
        }
        __syncthreads();
        if (tid < P) sorted[s_rank[tid]] = key;  // tid < P implies c == 0: key is sorted[tid]
        __syncthreads();
        if (n_out == K) kth = sorted[K - 1];
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
    if (n_out == K) kth = sorted[K - 1];
    return n_out;
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
    int32_t keep;           // keys this selection keeps (K on the last level; fewer: a tighter threshold for the next level)
    int32_t keep_prev;      // what the selection before this one kept (K: its threshold was safe by construction)
    int32_t tau_parts;      // entries of tau the scan of this level admitted by (the smallest counts; 0: no threshold)
    uint64_t* tau;          // [B][kTauParts] in/out (entry 0; the seed pass writes one per slice)
    uint64_t* tau_img;      // thresholds in the order of the scorer's resident query image, or null
    const int32_t* q_taupos;  // [B] position of each query in tau_img (-1: none)
    const int32_t* q_prow;    // [B][kSeedRows + 1] first signature rows of each query's filter (-1 padded), then their count
    uint32_t* ovf;          // [B]
    int32_t lds_keys;       // candidates per query the selection gathers in LDS (<= kLdsKeys; sizes its LDS)
    int32_t first, last;
    int32_t big_sort;       // K above the LDS sort size: the set is carried unordered; 1: the launch's LDS holds k_pad keys for the final order, 2: ordered in global memory
    int32_t may_overflow;   // 0: the level's regions cannot overflow (every pair admitted, one visit per region): the flag is reset
    int64_t* out_ids;       // [B][K]
    float* out_scores;
    int32_t* out_count;
    // slow exact path (last level only): corpus, queries, all filter groups
    ScanParams scan;
    const int32_t* q2grp;   // [B] group of each query
    unsigned long long* density_acc;  // first level only: receives the query's candidate count (null: none)
};

constexpr int kSelectThreads = 512;
constexpr int kLdsKeys = kSelectLdsKeys;  // candidates per query gathered in LDS; more go through global memory

// Slow exact path for a query whose candidate region overflowed in some level: rescans the whole
// corpus for that query alone, keeping at most gath_cap keys and pruning to the best K whenever
// the buffer cannot take another round.  Called by the whole workgroup.
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
    // A thread owns one 64-item word per round and scores the items it admits itself: rounds of up to
    // blockDim.x words, as many as the buffer is sure to hold beside the K keys kept (one tile at least).
    const int64_t n_words = (p.n_items + 63) >> 6;
    int64_t wpr = (r.gath_cap - r.K) / 64;
    wpr = wpr > nt ? nt : (wpr < kTileWords ? kTileWords : wpr);
    (void)s_mask;
    for (int64_t w0 = 0; w0 < n_words; w0 += wpr) {
        if ((int64_t)*s_n + wpr * 64 > r.gath_cap) {  // uniform: *s_n is stable between barriers
            const int n_out = wg_topk(buf, (int64_t)*s_n, r.K, sorted, r.k_pad, s_hist, s_misc, s_red);
            for (int i = tid; i < n_out; i += nt) buf[i] = sorted[i];
            tau = n_out == r.K ? sorted[r.K - 1] : 0ULL;
            __syncthreads();
            if (tid == 0) *s_n = (uint32_t)n_out;
            __syncthreads();
        }
        const int64_t gw = w0 + tid;
        uint64_t m = 0;
        if (tid < wpr && gw < n_words) m = bloom_mask_word(p.bloom, p.m_bits, gw, p.n_items, p.grp_rows + r0, r1 - r0);
        while (m) {
            const int bit = __ffsll((long long)m) - 1;
            m &= m - 1;
            const int64_t item = gw * 64 + bit;
            const float sc = pair_score(p, q, p.items + item * p.d, p.iscale[item]);
            const uint64_t key = make_key(sc, (uint32_t)item);
            if (key >= tau) buf[atomicAdd(s_n, 1u)] = key;
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
static_assert(kLdsSortMax * 8 >= kLdsKeys * 2, "the sort buffer doubles as the seed kernel's 16-bit item list");
constexpr int kSelectLdsBytes = kLdsKeys * 8 + kLdsSortMax * 8 + 3 * 256 * 4 + 64 * 8 + 64 * 4;
// Key capacity for batches that need more than one workgroup per compute unit: two selection
// workgroups then fit the 160 KB of LDS side by side.
constexpr int kLdsKeysDense = 7168;
inline int select_lds_bytes(int lds_keys) { return kSelectLdsBytes - (kLdsKeys - lds_keys) * 8; }

__global__ __launch_bounds__(kSelectThreads) void select_kernel(SelectParams p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char sel_lds[];
    const int lds_keys = p.lds_keys;
    uint64_t* s_keys = reinterpret_cast<uint64_t*>(sel_lds);                       // [lds_keys]
    uint64_t* s_sorted = s_keys + lds_keys;                                        // [kLdsSortMax]
    uint64_t* s_red = s_sorted + kLdsSortMax;                                      // [32]
    uint64_t* s_mask = s_red + 32;                                                 // [16]
    uint32_t* s_hist = reinterpret_cast<uint32_t*>(s_mask + 16);                   // [3][256]
    uint32_t* s_misc = s_hist + 3 * 256;                                           // [8]
    uint32_t* s_wsum = s_misc + 8;                                                 // [16]
    const int q = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    constexpr int NT = kSelectThreads;
    // counts are clamped to what the buffers can hold, whatever the memory says
    uint32_t n_prev = p.first ? 0u : p.topk_cnt[q];
    n_prev = n_prev < (uint32_t)p.K ? n_prev : (uint32_t)p.K;
    // (the level after a seed pass has no list from before but admits by threshold: its regions
    // can overflow like any later level's, and the seed pass has reset the flag)
    const bool overflowed = p.may_overflow && p.ovf[q] != 0u;
    if (!p.may_overflow && tid == 0) p.ovf[q] = 0u;
    if (p.last && overflowed) {  // uniform over the workgroup
        rescue_query(p, q, s_sorted, s_hist, s_misc, s_red, s_mask, &s_misc[4]);
        return;
    }

    // exclusive prefix sum of the region counts: NT threads x ceil(regions/NT) regions each,
    // shuffles inside a wavefront, one LDS exchange between the wavefronts
    const int R = p.regions;
    const int per = (R + NT - 1) / NT;
    const uint32_t* cq = p.cnt + (int64_t)q * p.groups;
    uint32_t mine = 0;
    // With at most two regions per thread (the usual layout) the first eight keys of each region
    // are requested together with its count, before the count is known: a region holds a handful
    // of keys as a rule, so this is one memory round trip instead of two (what lies beyond the
    // count is stale workspace and is dropped).
    constexpr int kHead = 8;
    const bool spec = per <= 2 && gridDim.x <= 512;  // (larger batches fill the chip several times over: latency is hidden, bytes are not)
    uint32_t hc[2] = {0u, 0u};
    int4 hv[2][kHead / 2];
    if (spec) {
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const int w = tid * per + jj;
            const bool live = jj < per && w < R;
            const int4* src = reinterpret_cast<const int4*>(p.cand + ((int64_t)q * p.groups + (live ? w : 0)) * p.cap);
            if (live) {
                hc[jj] = cq[w];
#pragma unroll
                for (int u = 0; u < kHead / 2; ++u) hv[jj][u] = src[u];  // (a region holds at least 64 entries)
            }
        }
        hc[0] = min(hc[0], (uint32_t)p.cap);
        hc[1] = min(hc[1], (uint32_t)p.cap);
        mine = hc[0] + hc[1];
    } else {
        for (int j = 0; j < per; ++j) {
            const int w = tid * per + j;
            if (w < R) mine += min(cq[w], (uint32_t)p.cap);
        }
    }
    const uint32_t incl = wave_scan_add(mine);
    if (lane == 63) s_wsum[wv] = incl;
    __syncthreads();
    uint32_t wbase = 0, all = 0;
    for (int w = 0; w < NT / 64; ++w) {
        const uint32_t v = s_wsum[w];
        if (w < wv) wbase += v;
        all += v;
    }
    const uint32_t total = n_prev + all;
    if (p.density_acc && tid == 0) atomicAdd(p.density_acc, (unsigned long long)all);
    // A threshold tighter than the K-th best so far has let through every key at or above it and
    // nothing else.  If those are fewer than K in the whole corpus the threshold was too tight for
    // this query (its best items crowd the head of the corpus): recompute the query exactly.
    uint64_t tau_prev = 0ULL;
    if (p.keep_prev < p.K && p.tau_parts > 0) {
        tau_prev = ~0ULL;
        for (int pp = 0; pp < p.tau_parts; ++pp) tau_prev = min(tau_prev, p.tau[(int64_t)q * kTauParts + pp]);
    }
    if (p.last && tau_prev != 0ULL && total < (uint32_t)p.K) {  // uniform over the workgroup
        if (tid == 0) p.ovf[q] = 1u;  // reported like an overflow: the query took the slow exact path
        __syncthreads();
        rescue_query(p, q, s_sorted, s_hist, s_misc, s_red, s_mask, &s_misc[4]);
        return;
    }
    const bool in_lds = total <= (uint32_t)lds_keys;
    // More candidates than LDS holds, result sorted in LDS: the candidates are narrowed down where
    // they lie (below), not copied.
    const bool narrow = !in_lds && !p.srt;
    uint64_t* gkeys = p.gath + (int64_t)q * p.gath_cap;
    // f(key) for every candidate of the query: each thread walks its own regions (loads independent
    // of each other), then the running top-K
    auto for_each_key = [&](auto&& f) {
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
                        if (i0 + u < c) f(v[u]);
                }
            }
        }
        for (int i = tid; i < (int)n_prev; i += NT) f(p.topk_keys[(int64_t)q * p.K + i]);
    };
    if (!narrow) {
        // contiguous copy: regions in order after the running top-K.  A thread's regions are taken
        // two at a time, the first eight keys of both requested before any is stored (a region
        // holds a handful of keys as a rule: one memory round trip instead of one per four keys).
        uint32_t off = n_prev + wbase + incl - mine;
        for (int j0 = 0; j0 < per; j0 += 2) {
            uint32_t c[2];
            const uint64_t* src[2];
            uint64_t v[2][kHead];
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) {
                const int w = tid * per + j0 + jj;
                const bool live = j0 + jj < per && w < R;
                c[jj] = spec ? hc[jj] : (live ? min(cq[w], (uint32_t)p.cap) : 0u);
                src[jj] = p.cand + ((int64_t)q * p.groups + (live ? w : 0)) * p.cap;
            }
            if (spec) {
#pragma unroll
                for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                    for (int u = 0; u < kHead / 2; ++u) {
                        v[jj][2 * u] = ((uint64_t)(uint32_t)hv[jj][u].y << 32) | (uint32_t)hv[jj][u].x;
                        v[jj][2 * u + 1] = ((uint64_t)(uint32_t)hv[jj][u].w << 32) | (uint32_t)hv[jj][u].z;
                    }
            } else {
#pragma unroll
                for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                    for (int u = 0; u < kHead; ++u)
                        if ((uint32_t)u < c[jj]) v[jj][u] = src[jj][u];
            }
#pragma unroll
            for (int jj = 0; jj < 2; ++jj) {
#pragma unroll
                for (int u = 0; u < kHead; ++u)
                    if ((uint32_t)u < c[jj]) {
                        if (in_lds) s_keys[off + u] = v[jj][u];
                        else gkeys[off + u] = v[jj][u];
                    }
                for (uint32_t i0 = kHead; i0 < c[jj]; i0 += 4) {
                    uint64_t t[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (i0 + u < c[jj]) t[u] = src[jj][i0 + u];
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (i0 + u < c[jj]) {
                            if (in_lds) s_keys[off + i0 + u] = t[u];
                            else gkeys[off + i0 + u] = t[u];
                        }
                }
                off += c[jj];
            }
        }
        for (int i = tid; i < (int)n_prev; i += NT) {
            const uint64_t v = p.topk_keys[(int64_t)q * p.K + i];
            if (in_lds) s_keys[i] = v;
            else gkeys[i] = v;
        }
    }
    __syncthreads();

    uint64_t* sorted = p.srt ? p.srt + (int64_t)q * p.k_pad : s_sorted;
    int n_out;
    uint64_t kth = 0;  // K-th best key so far (0: fewer than K candidates yet)
    if (narrow) {
        // Radix passes from the top, 12 bits each, over the candidates where they lie, until the
        // keys at or above the bucket that holds the K-th fit in LDS; those are collected and the
        // selection finishes there.  Scores of one query share most of their leading bits only up
        // to the exponent, so one pass is the rule.
        constexpr int kBins = 4096;
        static_assert(kBins * 4 <= kLdsSortMax * 8, "histogram borrows the sort buffer");
        uint32_t* hist = reinterpret_cast<uint32_t*>(s_sorted);
        uint64_t prefix = 0, pmask = 0;
        uint32_t want = (uint32_t)p.keep, above = 0;  // above: keys over the prefix bucket (all kept)
        uint64_t bound = 0;
        uint32_t keep = 0;
        for (int shift = 52;;) {
            for (int i = tid; i < kBins; i += NT) hist[i] = 0;
            __syncthreads();
            for_each_key([&](uint64_t key) {
                if ((key & pmask) == prefix) atomicAdd(&hist[(uint32_t)(key >> shift) & (kBins - 1)], 1u);
            });
            __syncthreads();
            // thread t owns bins 4095-8t .. 4088-8t (descending); running count from the top
            constexpr int kPer = kBins / NT;
            uint32_t h[kPer], sum = 0;
#pragma unroll
            for (int j = 0; j < kPer; ++j) { h[j] = hist[kBins - 1 - kPer * tid - j]; sum += h[j]; }
            const uint32_t inc = wave_scan_add(sum);
            if (lane == 63) s_wsum[wv] = inc;
            __syncthreads();
            uint32_t base = 0;
            for (int w = 0; w < wv; ++w) base += s_wsum[w];
            uint32_t before = base + inc - sum;  // keys of the bucket in bins above mine
            if (before < want && want <= before + sum) {  // exactly one thread
#pragma unroll
                for (int j = 0; j < kPer; ++j) {
                    if (want > before && want <= before + h[j]) {
                        s_misc[0] = (uint32_t)(kBins - 1 - kPer * tid - j);
                        s_misc[1] = want - before;   // rank inside that bin
                        s_misc[3] = before;          // keys of the bucket in the bins above it
                        s_misc[5] = before + h[j];   // ... and including it
                    }
                    before += h[j];
                }
            }
            __syncthreads();
            const uint32_t digit = s_misc[0], rest = s_misc[1], gt = s_misc[3], ge = s_misc[5];
            __syncthreads();
            if (above + ge <= (uint32_t)lds_keys || shift == 0) {
                bound = prefix | ((uint64_t)digit << shift);
                keep = above + ge;
                break;
            }
            above += gt;
            prefix |= (uint64_t)digit << shift;
            pmask |= (uint64_t)(kBins - 1) << shift;
            want = rest;
            shift = shift >= 12 ? shift - 12 : 0;  // the last window overlaps bits already fixed
        }
        if (tid == 0) s_misc[2] = 0;
        __syncthreads();
        for_each_key([&](uint64_t key) {
            if (key >= bound) {
                const uint32_t slot = atomicAdd(&s_misc[2], 1u);
                if (slot < (uint32_t)lds_keys) s_keys[slot] = key;
            }
        });
        __syncthreads();
        keep = keep < (uint32_t)lds_keys ? keep : (uint32_t)lds_keys;  // keys are distinct: never cut
        n_out = lds_topk(s_keys, (int)keep, p.keep, s_sorted, p.k_pad, s_hist, s_misc, s_red, p.last != 0, kth);
    } else if (in_lds && !p.srt) {
        n_out = lds_topk(s_keys, (int)total, p.keep, s_sorted, p.k_pad, s_hist, s_misc, s_red, p.last != 0, kth);
    } else if (p.big_sort) {
        // Large K: the set is carried from level to level unordered (only its K-th key is needed);
        // the last level orders it in LDS, which holds all k_pad keys once the selection's own
        // buffers are no longer in use.
        // (big_sort 2: more keys than LDS holds; the last level then orders them where they lie)
        const bool lds_final = p.big_sort == 1;
        n_out = wg_topk(in_lds ? s_keys : gkeys, (int64_t)total, p.keep, sorted, p.k_pad, s_hist, s_misc, s_red,
                        false, &kth);
        if (p.last && !lds_final) {
            // more keys than LDS holds: ordered in global memory, chunk by chunk through LDS
            constexpr int kChunk = 16384;  // (the launch sized the LDS for it)
            int P = 1;
            while (P < n_out) P <<= 1;
            __syncthreads();
            for (int i = n_out + tid; i < P; i += NT) sorted[i] = 0ULL;
            __syncthreads();
            if (P > kChunk)
                blocked_bitonic_desc(sorted, P, reinterpret_cast<uint64_t*>(sel_lds), kChunk);
            else
                (void)wg_topk(sorted, (int64_t)n_out, n_out, sorted, P, s_hist, s_misc, s_red);
        }
        if (p.last && lds_final) {
            uint64_t* big = reinterpret_cast<uint64_t*>(sel_lds);  // [k_pad]: the launch sized the LDS for it
            int P = 1;
            while (P < n_out) P <<= 1;
            __syncthreads();
            for (int i = tid; i < P; i += NT) big[i] = i < n_out ? sorted[i] : 0ULL;
            __syncthreads();
            for (int k2 = 2; k2 <= P; k2 <<= 1) {
                for (int j = k2 >> 1; j > 0; j >>= 1) {
                    for (int i = tid; i < P; i += NT) {
                        const int x = i ^ j;
                        if (x > i) {
                            const uint64_t a = big[i], b = big[x];
                            const bool desc = (i & k2) == 0;
                            if (desc ? (a < b) : (a > b)) { big[i] = b; big[x] = a; }
                        }
                    }
                    __syncthreads();
                }
            }
            sorted = big;
        }
    } else {
        n_out = wg_topk(in_lds ? s_keys : gkeys, (int64_t)total, p.keep, sorted, p.k_pad, s_hist, s_misc, s_red);
        kth = n_out == p.keep ? sorted[p.keep - 1] : 0ULL;
    }
    if (!p.last) {
        for (int i = tid; i < n_out; i += NT) p.topk_keys[(int64_t)q * p.K + i] = sorted[i];
        if (tid == 0) {
            // fewer keys than this level keeps: what is there is every key at or above the
            // threshold in force, which therefore stays (0: none yet, everything passing is kept)
            const uint64_t t64 = kth ? kth : tau_prev;
            p.topk_cnt[q] = (uint32_t)n_out;
            p.tau[(int64_t)q * kTauParts] = t64;
            if (p.tau_img) {
                const int pos = p.q_taupos[q];
                if (pos >= 0) p.tau_img[(int64_t)pos * kTauParts] = t64;
            }
        }
    } else {
        write_result(sorted, n_out, p.K, p.out_ids + (int64_t)q * p.K, p.out_scores + (int64_t)q * p.K,
                     p.out_count + q);
    }
}

// Seed pass for small batches: the prefix [0, seed_items) of the corpus is scanned per query by
// `parts` workgroups, each on its own slice -- Bloom test of every word at once, compaction, one
// lane per passing item for the int8 dot products (Sec. 4.2), radix select of the slice's keys
// (Algorithm 1 phase 4 on the prefix).  Its only product is an admission threshold per query for
// the first cooperative level, which then scans the whole range from item 0.
constexpr int kSeedThreads = 512;
constexpr int kSeedRows = 8;       // signature rows per query in the seed kernel's row table
constexpr int kSeedMaxParts = kTauParts;
static_assert(kSeedItems / 64 <= kSeedThreads, "one Bloom word per thread");

// A threshold from the rank-th best of n keys in LDS, for a small rank, computed in registers
// (one barrier, no histogram passes: the radix selection costs about 5 us whatever the rank).
// It works on the keys' score halves.  A round takes the largest score below that of the round
// before, so after `rank` rounds at least `rank` keys lie at or above the score found.  Every
// wavefront runs the rounds over its share of the keys and leaves its `rank` best distinct
// scores in LDS; the first wavefront then runs them once more over those, and returns the
// smallest key with the score it ends on -- at or below the rank-th best key, equal to it up to
// the item id unless scores tie among the best.  Fewer distinct scores than `rank` (fewer keys, or
// many ties): 0, and the caller takes the exact selection.  For workgroups of at most 8 wavefronts
// and n <= 1024 keys per wavefront; the result is valid in the first wavefront.
constexpr int kSmallRank = 8;
constexpr int kSmallRankPerLane = 16;

__device__ inline uint64_t wg_threshold_small(const uint64_t* keys, int n, int rank, uint32_t* s_best /*[8][kSmallRank]*/)
{
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, nw = blockDim.x >> 6;
    // rounds over the values in kr[0 .. nj): the distinct maxima in falling order, `found` of them
    auto rounds = [&](const uint32_t (&kr)[kSmallRankPerLane], int nj, uint32_t (&best)[kSmallRank]) -> int {
        uint32_t bound = 0xFFFFFFFFu;  // exclusive; above every score half
        int found = 0;
#pragma unroll
        for (int r = 0; r < kSmallRank; ++r) best[r] = 0u;
#pragma unroll
        for (int r = 0; r < kSmallRank; ++r) {
            if (r >= rank) break;
            uint32_t m = 0;
#pragma unroll
            for (int j = 0; j < kSmallRankPerLane; ++j) {
                if (j >= nj) break;  // (the same in every lane)
                const uint32_t c = kr[j] < bound ? kr[j] : 0u;
                m = c > m ? c : m;
            }
            m = lane_value(wave_max_u32(m), 63);
            if (m == 0) break;
            best[r] = m;
            bound = m;
            ++found;
        }
        return found;
    };
    uint32_t kr[kSmallRankPerLane], best[kSmallRank];
    const int nj = (n + 64 * nw - 1) / (64 * nw);  // keys per lane, at most kSmallRankPerLane
#pragma unroll
    for (int j = 0; j < kSmallRankPerLane; ++j) {
        const int i = lane + 64 * (wv + nw * j);
        kr[j] = (j < nj && i < n) ? (uint32_t)(keys[i] >> 32) : 0u;  // (score halves are never 0)
    }
    (void)rounds(kr, nj, best);
#pragma unroll
    for (int r = 0; r < kSmallRank; ++r)
        if (lane == r) s_best[wv * kSmallRank + r] = best[r];
    __syncthreads();
    uint64_t kth = 0;
    if (wv == 0) {
        kr[0] = lane < nw * kSmallRank ? s_best[lane] : 0u;
        const int found = rounds(kr, 1, best);
        uint32_t last = 0;
#pragma unroll
        for (int r = 0; r < kSmallRank; ++r)
            if (r < found) last = best[r];
        if (found == rank) kth = (uint64_t)last << 32;
    }
    return kth;
}

// Slices per query: enough workgroups to occupy the chip, whole 1024-item tiles per slice.
inline int seed_parts(int batch, int k_pad)
{
    int parts = 1;
    (void)k_pad;
    while (parts < kSeedMaxParts && batch * parts < 256 && kSeedItems / (2 * parts) >= kTileItems)
        parts *= 2;
    return parts;
}

// The seed pass is the first kernel of a search, so it also brings the call's table blob to the
// device: its own tables are read from the caller-side pinned copy (the table pointers in p that it
// uses point there), and the workgroups copy the blob, a share each, to where the later kernels
// expect it.
struct SeedUpload {
    const int32_t* src;  // pinned host memory, device-visible
    int32_t* dst;        // table area of the workspace
    int32_t words;
    // Resident-query image of the MFMA scorer (null: none).  The seed pass also writes it, in the
    // layout that scorer keeps in LDS, so that the scan that follows stages its queries with one
    // memory round trip instead of two (row table, then rows).
    int8_t* img_q;             // [q_split][rows_local][d], 16-byte chunks swizzled as in LDS
    float* img_sq;             // [q_split][rows_local]
    int32_t* img_qrow;         // [q_split][rows_local]  global query row or -1 (padding)
    const int32_t* blk_row;    // [n_blocks * 16] query row of every block row, pinned host memory
    int32_t n_blocks, q_split, rows_local;
    // The 64-item words of the seed pass are spread evenly over the corpus: word i of the pass is
    // word i * word_stride of the corpus (1: a prefix), and the slices take the pass's words in
    // turn.  What the pass learns about a query's scores then does not depend on trends along the
    // item order, and every slice sees what the others see.
    int32_t word_stride;
};

// D16 = d / 16 for d in {64, 128, 256} (item rows staged in registers, two items per thread in
// flight), 0 = any other d (plain loop).  Grid (batch, parts).
template <int D16>
__global__ __launch_bounds__(kSeedThreads) void seed_kernel(SelectParams p, int64_t seed_items, SeedUpload up)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char sel_lds[];
    uint64_t* s_keys = reinterpret_cast<uint64_t*>(sel_lds);                       // [kLdsKeys]
    uint64_t* s_sorted = s_keys + kLdsKeys;                                        // [kLdsSortMax]
    uint64_t* s_red = s_sorted + kLdsSortMax;                                      // [32]
    uint64_t* s_mask = s_red + 32;                                                 // [16]
    uint32_t* s_hist = reinterpret_cast<uint32_t*>(s_mask + 16);                   // [3][256]
    uint32_t* s_misc = s_hist + 3 * 256;                                           // [8]
    uint32_t* s_wsum = s_misc + 8;                                                 // [16]
    const int q = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int parts = (int)gridDim.y, part = (int)blockIdx.y;
    constexpr int NT = kSeedThreads;
    const ScanParams& sp = p.scan;
    const int slot = q * parts + part;
    {  // this workgroup's share of the table blob
        const int n_wg = (int)(gridDim.x * gridDim.y);
        const int share = (up.words + n_wg - 1) / n_wg;
        const int w0 = slot * share;
        for (int i = tid; i < share && w0 + i < up.words; i += NT) up.dst[w0 + i] = up.src[w0 + i];
    }
    if (up.img_q && wv == NT / 64 - 1) {  // the last wavefront: the first ones hold the Bloom words of the slice
        const int l = lane, T = sp.n_tasks, d = sp.d, nch = d >> 4;
        const int sh = nch >= 16 ? 0 : (nch == 8 ? 1 : 2), smask = (nch < 16 ? nch : 16) - 1;  // the scorer's chunk swizzle
        const int rows_q = up.rows_local / T;  // queries per row of scan workgroups
        if (part == 0) {
            const int pos = p.q_taupos[q];
            if (pos >= 0) {
                const int yy = pos / rows_q, lr0 = (pos - yy * rows_q) * T;
                for (int i = l; i < T * nch; i += 64) {
                    const int t = i / nch, c = i - t * nch, lr = lr0 + t;
                    const int64_t grow = (int64_t)q * T + t;
                    const int64_t ir = (int64_t)yy * up.rows_local + lr;
                    const int4 v = reinterpret_cast<const int4*>(sp.queries + grow * d)[c];
                    *reinterpret_cast<int4*>(up.img_q + ir * d + ((c ^ ((lr >> sh) & smask)) << 4)) = v;
                    if (c == 0) {
                        up.img_sq[ir] = sp.qscale[grow];
                        up.img_qrow[ir] = (int)grow;
                    }
                }
            }
        }
        // padding rows of the image, dealt out over the workgroups
        const int n_rows = up.rows_local * up.q_split, n_wg = (int)(gridDim.x * gridDim.y);
        for (int ir = slot; ir < n_rows; ir += n_wg) {
            const int yy = ir / up.rows_local, lr = ir - yy * up.rows_local;
            const int b = (lr >> 4) * up.q_split + yy;
            const int grow = b < up.n_blocks ? up.blk_row[b * 16 + (lr & 15)] : -1;
            if (grow < 0) {
                for (int c = l; c < nch; c += 64)
                    *reinterpret_cast<int4*>(up.img_q + (int64_t)ir * d + (c << 4)) = make_int4(0, 0, 0, 0);
                if (l == 0) {
                    up.img_sq[ir] = 0.0f;
                    up.img_qrow[ir] = -1;
                }
            }
        }
    }
    const int64_t ws = up.word_stride > 1 ? up.word_stride : 1;
    // Place in the corpus of position l of this slice.  The pass's words are dealt out to the slices
    // in turn (word j of slice `part` is word j * parts + part of the pass), so that every slice is
    // itself spread over the whole corpus.
    auto corpus_word = [&](int64_t slice_word) -> int64_t { return (slice_word * parts + part) * ws; };
    auto corpus_item = [&](int64_t l) -> int64_t { return (corpus_word(l >> 6) << 6) | (l & 63); };
    const int64_t n_all = seed_items < sp.n_items ? seed_items : sp.n_items;
    const int64_t part_items = seed_items / parts;  // whole tiles
    const int64_t begin = part * part_items;
    const int64_t n = n_all - begin < part_items ? (n_all - begin > 0 ? n_all - begin : 0) : part_items;  // items of this slice
    const int n_words = (int)((n + 63) >> 6);  // <= NT: one word per thread
    // per query: [parts][pstride] scratch for the selection of slices too large for LDS, then room
    // for their keys
    const int pshare = kLdsKeys / parts;
    const int pstride = p.K > pshare ? p.K : pshare;
    uint64_t* gpart = p.gath + (int64_t)q * p.gath_cap;
    uint64_t* gkeys = gpart + (int64_t)parts * pstride + begin;
    // the query's candidate regions are free at this point: scratch for the list of passing items
    uint32_t* glist = reinterpret_cast<uint32_t*>(const_cast<uint64_t*>(p.cand) + (int64_t)q * p.groups * p.cap) + begin;

    // Bloom test: thread w owns word w of the slice.  The first signature rows of the query's filter
    // come from a per-query table (one round trip), longer filters fetch the rest through the group tables.
    uint64_t mword = 0;
    if (tid < n_words) {
        const int64_t left = n - (int64_t)tid * 64;
        mword = left >= 64 ? ~0ULL : ((1ULL << left) - 1ULL);
        const int64_t gw = corpus_word(tid);
        const uint64_t* base = sp.bloom + ((gw >> 4) * (int64_t)sp.m_bits) * kTileWords + (gw & 15);
        const int* qr = p.q_prow + q * (kSeedRows + 1);
        const int nr = qr[kSeedRows];
#pragma unroll
        for (int r = 0; r < kSeedRows; ++r) {
            const int row = qr[r];
            if (row >= 0) mword &= base[(int64_t)row * kTileWords];
        }
        if (nr > kSeedRows) {
            const int g = p.q2grp[q];
            const int r0 = sp.grp_row_off[g];
            for (int r = kSeedRows; r < nr; ++r) mword &= base[(int64_t)sp.grp_rows[r0 + r] * kTileWords];
        }
    }
    const uint32_t mine = (uint32_t)__popcll(mword);
    const uint32_t incl = wave_scan_add(mine);
    if (lane == 63) s_wsum[wv] = incl;
    __syncthreads();
    uint32_t wbase = 0, total = 0;
    for (int w = 0; w < NT / 64; ++w) {
        const uint32_t v = s_wsum[w];
        if (w < wv) wbase += v;
        total += v;
    }
    const bool in_lds = total <= (uint32_t)kLdsKeys;
    // list of passing items (relative to the slice): 16-bit entries in the (still unused) sort
    // buffer when the keys fit LDS, else 32-bit entries in the query's candidate regions
    uint16_t* slist = reinterpret_cast<uint16_t*>(s_sorted);  // kLdsSortMax * 8 bytes = kLdsKeys * 2
    {
        uint32_t off = wbase + incl - mine;
        uint64_t m = mword;
        while (m) {
            const int b = __ffsll((long long)m) - 1;
            m &= m - 1;
            if (in_lds) slist[off] = (uint16_t)(tid * 64 + b);
            else glist[off] = (uint32_t)(tid * 64 + b);
            ++off;
        }
    }
    __syncthreads();
    // scores: one lane per passing item
    if (D16 == 0) {
        for (uint32_t e = tid; e < total; e += NT) {
            const int64_t item = corpus_item(in_lds ? (int64_t)slist[e] : (int64_t)glist[e]);
            const float sc = pair_score(sp, q, sp.items + item * sp.d, sp.iscale[item]);
            const uint64_t key = make_key(sc, (uint32_t)item);
            if (in_lds) s_keys[e] = key;
            else gkeys[e] = key;
        }
    } else {
        constexpr int DD = D16 > 0 ? D16 : 1;
        // two items per thread and round: all of their row loads are in flight together
        for (uint32_t e0 = tid; e0 < total; e0 += 2 * NT) {
            int4 ra[2][DD];
            float si[2];
            int64_t item[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const uint32_t e = e0 + u * NT;
                const uint32_t ec = e < total ? e : e0;
                item[u] = corpus_item(in_lds ? (int64_t)slist[ec] : (int64_t)glist[ec]);
                const int4* rp = reinterpret_cast<const int4*>(sp.items + item[u] * (DD * 16));
#pragma unroll
                for (int c = 0; c < DD; ++c) ra[u][c] = rp[c];
                si[u] = sp.iscale[item[u]];
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const uint32_t e = e0 + u * NT;
                float sc = 0.0f;
                const int nt_ = sp.weighted ? sp.n_tasks : 1;
                for (int t = 0; t < nt_; ++t) {
                    const int64_t qr = (int64_t)q * nt_ + t;
                    const int4* qp = reinterpret_cast<const int4*>(sp.queries + qr * (DD * 16));
                    int acc = 0;
#pragma unroll
                    for (int c = 0; c < DD; ++c) acc = dot16(ra[u][c], qp[c], acc);
                    const float st = rescale(acc, sp.qscale[qr], si[u]);
                    sc = sp.weighted ? __fmaf_rn(sp.w[t], st, sc) : st;
                }
                if (e < total) {
                    const uint64_t key = make_key(sc, (uint32_t)item[u]);
                    if (in_lds) s_keys[e] = key;
                    else gkeys[e] = key;
                }
            }
        }
    }
    __syncthreads();

    // This slice's share of the threshold: its ceil(keep / parts)-th best key.  With every slice
    // holding that many keys at or above its own value, the prefix holds at least `keep` keys at or
    // above the smallest of them, so the minimum over the slices lies at or below the keep-th best
    // key of the prefix: a valid admission threshold for keep = K, and for a smaller keep the
    // tighter one the schedule counts on (0 = this slice has too few passing items: no threshold).
    // Nothing else is carried over: the level after the seed pass scans the prefix again.
    // (Small ranks -- the usual case -- are taken in registers; that value may lie below the rank-th
    // best key by the ties in its score, which a threshold may.  A slice with fewer distinct scores
    // than the rank goes to the exact selection.)
    const int rank = (p.keep + parts - 1) / parts;
    int rank_pad = 1;
    while (rank_pad < rank) rank_pad <<= 1;
    uint64_t kth = 0;
    static_assert(NT / 64 * kSmallRankPerLane * 64 >= kLdsKeys, "every count of keys that fits LDS fits the registers of the small form");
    bool small_done = false;
    if (in_lds && rank <= kSmallRank && total >= (uint32_t)rank) {
        kth = wg_threshold_small(s_keys, (int)total, rank, reinterpret_cast<uint32_t*>(s_red));
        if (tid == 0) s_misc[6] = kth != 0ULL ? 1u : 0u;  // (a tie-heavy slice: the exact selection below)
        __syncthreads();
        small_done = s_misc[6] != 0u;  // (word 6 serves nothing else in this kernel)
    }
    if (small_done) {
        // (thread 0 holds the value and publishes it)
    } else if (in_lds) {
        (void)lds_topk(s_keys, (int)total, rank, s_sorted, rank_pad, s_hist, s_misc, s_red, false, kth);
    } else {
        uint64_t* sorted = gpart + (int64_t)part * pstride;  // K <= pstride entries of scratch
        const int n_out = wg_topk(gkeys, (int64_t)total, rank, sorted, rank_pad, s_hist, s_misc, s_red);
        kth = n_out == rank ? sorted[rank - 1] : 0ULL;
    }
    if (tid == 0) {
        p.tau[(int64_t)q * kTauParts + part] = kth;
        if (p.tau_img) {
            const int pos = p.q_taupos[q];
            if (pos >= 0) p.tau_img[(int64_t)pos * kTauParts + part] = kth;
        }
        if (part == 0) {
            p.ovf[q] = 0u;
            p.topk_cnt[q] = 0u;
        }
    }
}

template <int D16>
inline hipError_t launch_seed_t(const SelectParams& se, int64_t seed_items, int batch, int parts, const SeedUpload& up,
                                hipStream_t stream)
{
    static std::atomic<bool> lds_set{false};
    if (!lds_set.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&seed_kernel<D16>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kSelectLdsBytes);
        if (e != hipSuccess) return e;
        lds_set.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(seed_kernel<D16>, dim3(batch, parts), dim3(kSeedThreads), kSelectLdsBytes, stream, se, seed_items,
                       up);
    return hipGetLastError();
}

inline hipError_t launch_seed(const SelectParams& se, int64_t seed_items, int batch, int parts, const SeedUpload& up,
                              hipStream_t stream)
{
    switch (se.scan.d) {
        case 64: return launch_seed_t<4>(se, seed_items, batch, parts, up, stream);
        case 128: return launch_seed_t<8>(se, seed_items, batch, parts, up, stream);
        case 256: return launch_seed_t<16>(se, seed_items, batch, parts, up, stream);
        default: return launch_seed_t<0>(se, seed_items, batch, parts, up, stream);
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
