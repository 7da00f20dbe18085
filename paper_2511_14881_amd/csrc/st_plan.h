// Host-side scheduling of one search: how the corpus is cut into levels, how large the
// candidate regions are, and where everything sits in the caller's workspace.
//
// The corpus is scanned exactly once, in consecutive chunks ("levels").  Level 0 admits every
// passing (query, item) pair; after each level a selection kernel reduces the candidates to the
// best `keep` keys seen so far and publishes the keep-th as the admission threshold of the next
// level.  With keep = K that threshold is safe by construction (any item of the final top-K is at
// least as good as the K-th best of a prefix of the corpus).  A smaller keep gives a tighter
// threshold that is right unless the prefix holds at least `keep` of the final top-K items; the
// last selection notices that case (fewer than K keys at or above the threshold in the whole
// corpus) and recomputes the query exactly, so the result is exact either way (optimistic_keep).
// Levels grow geometrically so that the expected number of admitted candidates per
// (workgroup, query) region stays at a quarter of the region's capacity.  (The plan gives sizes;
// whether the first level's items are a prefix or segments spread over the corpus is the
// launcher's choice.)
#pragma once
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include <math.h>

namespace st {

constexpr int kComputeUnits = 256;   // MI355X
constexpr int kScanGroups = 1024;    // candidate regions per query (one per scan workgroup at 4 workgroups per CU)
constexpr int kMaxScanGroups = 2048;
constexpr int kMaxLevels = 32;
constexpr int kMaxSegItems = 512;    // items one workgroup takes per step, at most
constexpr int kLdsSortMax = 2048;    // top-K lists up to this (padded) size are sorted in LDS
constexpr int kSelectLdsKeys = 8192; // candidates per query the selection kernel handles in LDS

struct Level {
    int64_t begin, end;      // item range [begin, end)
    int32_t seg_items;       // items one workgroup stages per step (multiple of 64, divides 1024)
    int32_t seg_per_visit;   // consecutive segments a workgroup takes before striding on
    int32_t seed;            // 1: this prefix is handled by the per-query seed kernel
    int32_t keep;            // keys per query the selection after this level keeps (K on the last level)
};

struct Plan {
    int32_t groups;  // scan workgroups
    int32_t cap;     // entries per (workgroup, query) candidate region
    int32_t n_levels;
    Level level[kMaxLevels];
};

inline int64_t round_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

inline int32_t pow2_ceil(int32_t v)
{
    int32_t p = 1;
    while (p < v) p <<= 1;
    return p;
}

// Workgroups the scan kernels are launched with (fixes the candidate-region layout).
inline int scan_groups() { return kScanGroups; }

// Levels for a given region capacity.  g_eff = workgroups that share one query's candidates
// (all of them, unless the query rows are split over several workgroup rows).
constexpr int kSeedItems = 32768;      // prefix the seed kernel scans (one workgroup per query)
constexpr int kSeedMaxRows = 128;      // query rows (batch x tasks) up to which the seed kernel is used

// Small batches start with a seed pass: one workgroup per query scans a short prefix on its own
// and selects its top-K there, which replaces the first cooperative level and its selection.
inline int64_t seed_items_for(int64_t n_items, int32_t batch_rows)
{
    return (batch_rows <= kSeedMaxRows && n_items >= 8 * (int64_t)kSeedItems) ? kSeedItems : 0;
}

// Keys of a prefix of `prefix` items out of n_items worth keeping when the K best of the whole
// corpus are wanted.  The K best items sit at K of the n_items positions; if positions carry no
// information about scores (the order of the corpus is arbitrary with respect to a query), the
// number X of them inside the prefix is hypergeometric with mean m = K * prefix / n_items, and
// P(X >= r) <= exp(-m * ((r/m) * ln(r/m) - (r/m - 1))) (Chernoff bound, valid for sampling without
// replacement).  The smallest r that brings the bound under 1e-12 is returned: the r-th best key
// of the prefix is then below the K-th best of the corpus except with that probability, and the
// exact fallback of the last selection covers the exception (and corpora whose order does carry
// information).  Never more than K, which is always safe.
inline int32_t optimistic_keep(int32_t K, int64_t prefix, int64_t n_items)
{
    if (prefix >= n_items || K < 1) return K;
    const double m = (double)K * (double)prefix / (double)n_items;
    const double need = 27.631;  // ln(1e12)
    double lo = m > 1.0 ? m : 1.0, hi = (double)K;
    auto bound = [&](double r) { const double x = r / m; return m * (x * log(x) - (x - 1.0)); };
    if (bound(hi) < need) return K;
    for (int it = 0; it < 64 && hi - lo > 0.5; ++it) {
        const double mid = 0.5 * (lo + hi);
        if (bound(mid) >= need) hi = mid; else lo = mid;
    }
    const int64_t r = (int64_t)ceil(hi) + 1;
    return r < (int64_t)K ? (int32_t)r : K;
}

// `waves` = wavefronts that scan one level side by side (per row of workgroups): it sizes the
// segments of a level.
// optimistic = false: every selection keeps K keys (thresholds safe by construction); for searches
// whose passing items sit in a few item ranges, where a prefix says nothing about the rest.
// first_div: the first level takes 1 / first_div of the items it could.
inline int make_levels_sized(int64_t n_items, int32_t K, int32_t cap, int32_t g_eff, int32_t seg_cap, int64_t seed_items,
                             int32_t waves, Plan* out, bool optimistic, int32_t first_div)
{
    Plan p;
    p.groups = scan_groups();
    p.cap = cap;
    p.n_levels = 0;
    if (cap > kMaxSegItems || g_eff < 1 || seg_cap < 64 || seg_cap > kMaxSegItems || (seg_cap & (seg_cap - 1)))
        return -1;
    // level 0 hands each workgroup at most `cap` consecutive items (one visit), so no region can
    // overflow
    int64_t n0 = (int64_t)g_eff * cap / first_div;
    if (n0 > n_items) n0 = n_items;
    const int32_t seg0 = cap < seg_cap ? cap : seg_cap;
    if (seed_items > 0) {
        n0 = seed_items < n_items ? seed_items : n_items;
        p.level[p.n_levels++] = Level{0, n0, 0, 0, 1, K};
    } else {
        p.level[p.n_levels++] = Level{0, n0, seg0, cap / seg0, 0, K};
    }
    // keys kept after the level just planned = what the next level's threshold admits per growth
    auto keep_after = [&](int64_t prefix) -> int32_t {
        if (prefix >= n_items || !optimistic) return K;
        return optimistic_keep(K, prefix, n_items);
    };
    int32_t keep = keep_after(n0);
    p.level[0].keep = keep;
    // (the seed pass takes the smallest of its slices' ceil(keep / slices)-th best keys, which lies
    // at or below the keep-th best of the prefix: count on twice as many admissions)
    if (seed_items > 0 && keep < K) keep = 2 * keep < K ? 2 * keep : K;
    int64_t cur = n0;
    // The seed pass only leaves a threshold behind (no candidate list): the level after it starts
    // over at item 0, with the growth still counted from the prefix the threshold comes from.
    int64_t next_begin = seed_items > 0 ? 0 : n0;
    while (cur < n_items) {
        if (p.n_levels >= kMaxLevels) return -1;
        // expected admissions per region in a level that grows the scanned prefix by `grow` are
        // keep*(grow-1)/g_eff; aim at cap/4.  Never grow by less than 2x (extreme K with few sharing
        // workgroups): regions may then overflow and the slow exact path takes those queries.
        double grow = 1.0 + (double)cap * (double)g_eff / (4.0 * (double)keep);
        // a level should not admit more candidates per query (about keep * (grow - 1)) than the
        // selection kernel handles in LDS together with the running list; the estimate from `keep`
        // keys has a relative spread of keep^-1/2, hence the wider margin below K
        if (K <= kLdsSortMax) {
            const double fit = 1.0 + (keep < K ? 0.6 : 0.8) * (double)(kSelectLdsKeys - K) / (double)keep;
            if (grow > fit) grow = fit;
        }
        if (grow < 2.0) grow = 2.0;
        double want = (double)cur * grow;
        int64_t nxt = want >= (double)n_items ? n_items : (int64_t)want;
        if (nxt < n_items) nxt = nxt / 1024 * 1024;
        if (nxt <= cur) nxt = cur + 1024 < n_items ? cur + 1024 : n_items;
        // Segment size: a wavefront's share of the level is ceil(segments / waves) segments, each
        // costing a fixed part (the memory round trips of a stage, worth about 256 items of
        // streaming) plus its items; the size with the smallest product wins, larger on ties
        // (large segments also fill the 16-item MFMA tiles best).
        // A segment's candidates go to one region, and about K * (grow - 1) candidates per query are
        // expected in the level: sizes that leave fewer segments than four times that many over
        // the region capacity are passed over (down to the smallest size).
        int32_t seg = seg_cap;
        {
            const int64_t span = nxt - next_begin;
            const double admitted = (double)keep * ((double)nxt / (double)(cur > 0 ? cur : 1) - 1.0);
            const int64_t min_seg_count = (int64_t)(4.0 * admitted / (double)cap) + 1;
            int64_t best = -1;
            for (int32_t c = seg_cap; c >= 64; c >>= 1) {
                const int64_t n_seg = (span + c - 1) / c;
                if (n_seg < min_seg_count && c > 64) continue;
                const int64_t cost = ((n_seg + waves - 1) / waves) * (256 + c);
                if (best < 0 || cost < best) {
                    best = cost;
                    seg = c;
                }
            }
        }
        keep = keep_after(nxt);
        p.level[p.n_levels++] = Level{next_begin, nxt, seg, 4, 0, keep};  // one segment per wavefront of the workgroup
        cur = nxt;
        next_begin = nxt;
    }
    *out = p;
    return 0;
}

// A first level of half the size costs less itself (fewer candidates for its selection to read, a
// shorter admit-everything pass) and leaves a looser threshold, i.e. more admissions in the level
// that follows.  Measured: it pays where the two-level schedule stays and the keys that level
// then hands to the final selection stay below this many (Multi, K = 200: step -3 %; Large, K = 500,
// would go from 4300 to 6000 keys per query: +15 %).
constexpr int kSmallFirstLevelKeys = 3500;

// small_first: the caller will take the first level's items as segments spread over the corpus (not
// as a prefix), and wants the smaller first level where it pays.  (With a prefix, a smaller first level
// widens the set of corpora -- best items at the head -- whose queries end on the slow exact path.)
inline int make_levels(int64_t n_items, int32_t K, int32_t cap, int32_t g_eff, int32_t seg_cap, int64_t seed_items,
                       int32_t waves, Plan* out, bool optimistic = true, bool small_first = false)
{
    Plan full;
    const int rc = make_levels_sized(n_items, K, cap, g_eff, seg_cap, seed_items, waves, &full, optimistic, 1);
    if (rc != 0) return rc;
    if (small_first && seed_items == 0 && optimistic && full.n_levels == 2 && full.level[0].end < n_items) {
        Plan half;
        if (make_levels_sized(n_items, K, cap, g_eff, seg_cap, seed_items, waves, &half, optimistic, 2) == 0 &&
            half.n_levels == 2 && half.level[0].end >= 1024) {
            const double grow = (double)n_items / (double)half.level[0].end;
            if ((double)K + (double)half.level[0].keep * (grow - 1.0) <= (double)kSmallFirstLevelKeys) {
                *out = half;
                return 0;
            }
        }
    }
    *out = full;
    return 0;
}

// Region capacity from the sizes alone (it fixes the workspace layout).  The first level admits
// every passing pair of groups * cap items, so its cost grows with the capacity; later levels
// grow by at most cap * groups / (4K).  The smallest capacity that keeps the schedule at six
// levels or fewer (every workgroup sharing every query) is taken, else the largest.
inline int choose_cap(int64_t n_items, int32_t K, int32_t min_cap = 64)
{
    static const int32_t caps[] = {64, 128, 256, 512};
    int best = -1;
    for (int32_t cap : caps) {
        if (cap < min_cap) continue;
        // the slow exact path appends into a buffer of K + groups*cap keys, a tile at a time
        if ((int64_t)scan_groups() * cap < 2 * (int64_t)K + 2048) continue;
        Plan p;
        if (make_levels(n_items, K, cap, scan_groups(), kMaxSegItems, 0, 2048, &p) != 0) continue;
        best = cap;
        if (p.n_levels <= 6) break;
    }
    return best;
}

// min_cap: smallest region capacity to consider.  Searches whose passing items sit in a few dense
// item ranges (cluster probing) ask for the largest: a long first level that admits everything
// then gives every query a threshold, and a dense range cannot overflow a region.
inline int make_plan(int64_t n_items, int32_t K, int32_t q_split, int32_t seg_cap, int32_t batch_rows, Plan* out,
                     int32_t waves = 2048, int32_t min_cap = 64, bool optimistic = true, bool small_first = false)
{
    const int cap = choose_cap(n_items, K, min_cap);
    if (cap < 0 || q_split < 1 || scan_groups() % q_split) return -1;
    // the seed pass borrows the candidate regions and the gather buffer of a query as scratch
    const bool seed_fits = K <= kLdsSortMax && (int64_t)scan_groups() * cap >= 2 * (int64_t)kSeedItems;
    const int64_t seed = seed_fits ? seed_items_for(n_items, batch_rows) : 0;
    return make_levels(n_items, K, cap, scan_groups() / q_split, seg_cap, seed, waves < 1 ? 1 : waves, out, optimistic, small_first);
}

// Byte offsets of the pieces of the device workspace.
struct Layout {
    size_t meta, meta_bytes;  // uploaded group tables
    size_t density;           // uint64           passing pairs of the first level, summed over the batch
    size_t tau;               // uint64 [B][8]    admission threshold per query (seed pass: one per slice, the minimum counts)
    size_t ovf;               // uint32 [B]       1 = a candidate region overflowed
    size_t topk_keys;         // uint64 [B][K]    running top-K, sorted
    size_t topk_cnt;          // uint32 [B]
    size_t cnt;               // uint32 [B][G]    entries used in each region
    size_t cand;              // uint64 [B][G][cap]
    size_t gath;              // uint64 [B][K + G*cap]  contiguous copy for selection
    size_t srt;               // uint64 [B][Kpad]       only when Kpad > kLdsSortMax
    size_t img_q, img_sq, img_qrow, img_tau;  // resident-query image of the MFMA scorer
    size_t img_rows;          // rows the image has room for
    size_t total;
    int64_t gath_cap;
    int32_t k_pad;
};

inline size_t meta_bound_bytes(int32_t batch)
{
    // group tables (rows: at most 64 per query, twice: all groups and the per-scorer copies),
    // query lists, offsets, MFMA block tables (at most 16*(T/16 + 1) rows per query), slack
    return (size_t)round_up(4096 + (size_t)batch * 840, 256);
}

inline Layout make_layout(const Plan& p, int32_t batch, int32_t K, int32_t d = 16, int32_t n_tasks = 1)
{
    Layout L;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = (size_t)round_up((int64_t)(off + bytes), 256); return o; };
    L.meta_bytes = meta_bound_bytes(batch);
    L.meta = take(L.meta_bytes);
    L.density = take(8);
    L.tau = take((size_t)batch * 8 * 8);
    L.ovf = take((size_t)batch * 4);
    L.topk_keys = take((size_t)batch * K * 8);
    L.topk_cnt = take((size_t)batch * 4);
    L.cnt = take((size_t)batch * p.groups * 4);
    L.cand = take((size_t)batch * p.groups * p.cap * 8);
    L.gath_cap = (int64_t)K + (int64_t)p.groups * p.cap;
    L.gath = take((size_t)batch * L.gath_cap * 8);
    L.k_pad = pow2_ceil(K);
    L.srt = take(L.k_pad > kLdsSortMax ? (size_t)batch * L.k_pad * 8 : 0);
    // query rows padded to 16-row blocks per filter group (at most 128 groups use the image),
    // and again to whole blocks per row of workgroups (at most 32 rows)
    L.img_rows = (size_t)batch * n_tasks + 16 * 128 + 16 * 32;
    L.img_q = take(L.img_rows * d);
    L.img_sq = take(L.img_rows * 4);
    L.img_qrow = take(L.img_rows * 4);
    L.img_tau = take(L.img_rows * 8 * 8);
    L.total = off;
    return L;
}

}  // namespace st
