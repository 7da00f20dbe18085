// Scan with the int8 MFMA scorer (v_mfma_i32_16x16x64_i8), for filter groups that carry enough
// query rows to make scoring a dense contraction (Sec. 4.2: item rows are streamed from the
// embedding table and multiplied with the batched queries on the fly, nothing is gathered into
// a temporary in HBM).  Queries stay resident in LDS for the whole launch and are the only thing
// the four wavefronts of a workgroup share; in the main loop every wavefront works alone, on
// its own segments of the corpus, without barriers:
//   1. lane (filter, word) ANDs the Bloom rows of its filter for its 64-item word (the words of
//      the next segment are fetched while the current one is scored),
//   2. the set bits of each filter's words become a dense list of passing items (wave-private
//      LDS),
//   3. 16 passing items of one filter at a time go straight from HBM into the B operand (a ring
//      of register slots keeps the loads of the next units in flight while the current one is
//      multiplied) and are contracted with the filter group's query blocks; scores that reach
//      the query's threshold are admitted to the workgroup's candidate region.
//
// Contraction layout per MFMA (M = 16 query rows, N = 16 items, K = 64 bytes of the embedding):
//   A (queries): lane l supplies row (l % 16), bytes [16*(l/16), +16) of the 64-byte k-step
//   B (items)  : lane l supplies item (l % 16), the same byte range
//   D          : lane l receives D[4*(l/16) + r][l % 16], r = 0..3  -> one item, four query rows
// so with T in {1, 2, 4} tasks the rows one lane holds are whole queries and the Value-Model
// sum needs no cross-lane traffic.
#pragma once
#include <atomic>
#include <type_traits>

#include "st_device.h"
#include "st_plan.h"
#include "st_scan_params.h"

namespace st {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kMfmaFilterBatch = 8;        // distinct filters handled per pass over a segment
constexpr int kPrefetchRows = 8;           // signature rows per filter prefetched by 4-wavefront workgroups, and resident in the kernel arguments
constexpr int kPrefetchStride = 16;        // rows per filter in the prefetch table; 8-wavefront workgroups prefetch all of them
constexpr int kMfmaQueryLds = 64 * 1024;   // LDS bytes for resident query rows per workgroup
constexpr int kMfmaMinRows = 4;            // a group needs this many query rows to go to MFMA
constexpr int kMfmaMaxGroups = 128;        // groups one MFMA launch takes (the rest go to the dot scorer)
constexpr int kMfmaSegItems = 512;         // items per wavefront segment, at most (8 mask words x 8 filters = 64 lanes)
constexpr int kQueueSlots = 128;           // (size of the accumulator part of the queue, in 8-byte words)
constexpr int kQueueLanes = 64;            // queued lanes per wavefront: four accumulator values and a code each
constexpr int kQueueBytes = kQueueSlots * 8 + kQueueLanes * 4;
// queue bytes per wavefront: kernels that contract two units at once (8 wavefronts, d <= 128) queue
// pair by pair and need no code array
constexpr int mfma_queue_bytes(int d, int waves) { return (waves == 8 && d <= 128) ? kQueueSlots * 8 : kQueueBytes; }
constexpr int kMaxRegionSlots = 8;         // candidate regions one workgroup may fill in a launch
constexpr int kDenseItems = 12;            // passing items per filter and 512-item segment from which full units are the rule


struct MfmaParams {
    const int32_t* grp_blk_off;  // [F+1] first 16-row block of each group
    const int32_t* blk_row;      // [n_blocks*16] global query row (q*T + t) or -1 for padding
    int32_t n_blocks;            // all groups
    int32_t q_split;             // S: gridDim.y; block b belongs to y = b % S, local index b / S
    int32_t rows_local;          // 16 * blocks per y (max over y)
    const int32_t* prow;         // [groups][kPrefetchStride] first signature rows of each filter, -1 padded
    // The same rows for the first batch of filters, resident in the kernel arguments so that the
    // very first Bloom words can be requested before anything has been read from memory:
    // row r of filter g is bits [16*(r%4), +16) of prow_pack[g][r/4]; prow_n holds the row counts.
    // (4-wavefront workgroups take the first kPrefetchRows of them, 8-wavefront ones all.)
    uint64_t prow_pack[kMfmaFilterBatch][kPrefetchStride / 4];
    uint64_t prow_n;             // byte g = min(rows of filter g, kPrefetchStride)
    // Resident-query image in the workspace: written by workgroup x = 0 of each row of the grid
    // on the first level, read by every workgroup afterwards (one round trip instead of two).
    int8_t* img_q;               // [S][rows_local][d]   swizzled as in LDS
    float* img_sq;               // [S][rows_local]
    int32_t* img_qrow;           // [S][rows_local]
    uint64_t* img_tau;           // [S][rows_local / T][kTauParts]  written by the selection kernel (entry 0) or the seed pass
    int32_t first_level;         // 1: build the resident state from the tables and write the image
    int32_t multi_block;         // 1: some filter group holds more than one query block in a row of workgroups
    int32_t waves;               // wavefronts per workgroup: 4 or 8
    // A launch holds only as many workgroups as the device keeps resident; each owns region_slots
    // candidate regions (x + j * gridDim.x within its row of the grid) and rotates through them
    // visit by visit, so that the regions fill as evenly as with one workgroup per region.
    int32_t region_slots;
    int32_t seg_stride;          // items the per-wavefront LDS lists are laid out for (256 or 512, >= seg_items)
    // Passing (query, item) pairs of the first level, summed over the batch by its selection: the
    // first-level scan clears it, the selection adds each query's count, the later levels compare
    // it with density_limit to choose between the two forms of the scan (null: none of this).
    unsigned long long* density_acc;
    unsigned long long density_limit;
    // dynamic LDS layout (byte offsets)
    int32_t lds_sq, lds_tauf, lds_tau64, lds_qrow, lds_cnt, lds_list, lds_queue, lds_prow, lds_blkoff, lds_rowoff, lds_tq, lds_thr, lds_scl, lds_total;
};

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every
// outstanding global load; the set-up barrier of the scan would then sit out the HBM latency of
// the first Bloom words, which are requested before it and needed only after.
__device__ inline void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// chunk swizzle: keeps 16 consecutive rows of d bytes on distinct LDS banks when the 16 lanes
// of a quarter-wave read the same 16-byte chunk of each
template <int KS>
__device__ inline int swz(int row)
{
    constexpr int nch = KS * 4;                       // 16-byte chunks per row
    constexpr int sh = nch >= 16 ? 0 : (nch == 8 ? 1 : 2);
    return (row >> sh) & ((nch < 16 ? nch : 16) - 1);
}

// Item rows of one unit (up to 16 passing items of one filter group) in MFMA B layout.
template <int KS>
struct UnitRegs {
    v4i b[KS];
    float si;    // scale of the lane's item
    int si_fix;  // the same as a fixed-point factor for the integer cull (plain search)
    int si_fix2;  // second form of the scan: the lane's item as the 10-bit code a queued pair carries
    int item;    // lane's item (l % 16), relative to the segment start; -1 = padding lane
    int gi;      // filter within the batch (uniform)
};

// MULTI = some filter group holds more than one 16-row query block in a row of workgroups.
// NW = wavefronts per workgroup: 4, or 8 when the resident queries leave room for one workgroup
// per compute unit only (twice the wavefronts then share one query image).
// ADMIT = first level with one segment per region (8-wavefront workgroups only): no threshold
// exists yet, every passing pair is a candidate and goes straight to its region.
template <int KS, int TT, bool WEIGHTED, bool MULTI, int NW, bool ADMIT = false>
__device__ __forceinline__ void scan_mfma_body(const ScanParams& p, const MfmaParams& mp)
{
    static_assert(!ADMIT || NW == 8, "the first-level variant exists for 8-wavefront workgroups");
    constexpr int kThreads = NW * 64;
    // The variant for small batches (one query block per filter, four wavefronts) is only launched
    // with one region per workgroup and 256-item segments: both are compile-time facts there.
    constexpr bool LEAN = !MULTI && NW == 4;
    const int seg_stride = LEAN ? 256 : mp.seg_stride;
    constexpr int PR = NW == 8 ? kPrefetchStride : kPrefetchRows;  // rows prefetched per filter (register budget)
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int D = KS * 64;
    constexpr int CH = D / 16;  // 16-byte chunks per row
    constexpr int FB = kMfmaFilterBatch;
    // ring slots (units with rows in flight)
    // 8-wavefront workgroups contract two units at a time with each query block (the A operand and
    // the per-row constants are read from LDS once for both: LDS bandwidth, not the matrix cores,
    // bounds the loop when a filter group holds many query blocks); their ring holds two pairs.
    constexpr bool PAIRS = NW == 8 && KS <= 2;
    // (the small-batch variant at d = 128 measures best with two slots: its wavefronts wait on other things than rows,
    // and the registers of a third slot cost more than its loads in flight bring)
    // (the admit-everything first level at d = 256 has one short segment per wavefront: four slots halve its round trips)
    constexpr int NB = PAIRS ? 4 : (KS == 1 ? 4 : (KS == 2 ? (LEAN ? 2 : 3) : ((ADMIT && KS == 4) ? 4 : 2)));
    int8_t* s_q = reinterpret_cast<int8_t*>(lds);
    float* s_sq = reinterpret_cast<float*>(lds + mp.lds_sq);
    float* s_tauf = reinterpret_cast<float*>(lds + mp.lds_tauf);
    uint64_t* s_tau64 = reinterpret_cast<uint64_t*>(lds + mp.lds_tau64);    // [rows_local / TT]
    int* s_qrow = reinterpret_cast<int*>(lds + mp.lds_qrow);
    uint32_t* s_cnt = reinterpret_cast<uint32_t*>(lds + mp.lds_cnt);
    int* s_prow = reinterpret_cast<int*>(lds + mp.lds_prow);                // [groups][kPrefetchStride]
    int* s_glrow = reinterpret_cast<int*>(lds + mp.lds_blkoff);             // [groups] first local query row of the group
    int* s_gnblk = s_glrow + p.n_groups;                                    // [groups] local 16-row blocks of the group
    int* s_rowoff = reinterpret_cast<int*>(lds + mp.lds_rowoff);            // [groups + 1]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int S = mp.q_split, y = blockIdx.y;
    const int l16 = lane & 15, kg = lane >> 4;
    // Plain search: tau / s_q per row, so that a pair can only be admitted if dot * s_i reaches it.
    // +inf marks padding rows (never admitted), -inf rows that cannot be culled (no threshold yet,
    // tau <= 0, or a quotient outside the range the bound is valid for).
    auto tq_of = [](float tf, float sq) -> float {
        const float inf = __builtin_inff();
        if (tf == inf) return inf;
        if (!(tf > 0.0f)) return -inf;
        const float tq = tf / sq;
        return (tq > 0.0f && tq < inf) ? tq : -inf;
    };
    // Passing items of each filter, in item order, as the low 8 bits of their place in the segment:
    // entries of the upper half of a 512-item segment follow those of the lower half, so the
    // number of lower-half entries per filter restores the ninth bit.
    uint8_t* s_list = reinterpret_cast<uint8_t*>(lds + mp.lds_list) + wave * FB * seg_stride;  // wave-private [FB][seg]
    constexpr int QB = mfma_queue_bytes(KS * 64, NW);
    int4* q_acc = reinterpret_cast<int4*>(lds + mp.lds_queue + wave * QB);                        // wave-private
    uint64_t* s_queue = reinterpret_cast<uint64_t*>(q_acc);                                       // (the pair form of the queue)
    uint32_t* q_code = reinterpret_cast<uint32_t*>(lds + mp.lds_queue + wave * QB + kQueueSlots * 8);  // (lane form only)
    float* s_tq = reinterpret_cast<float*>(lds + mp.lds_tq);                                    // [rows_local] tau / s_q per row
    int* s_thr = reinterpret_cast<int*>(lds + mp.lds_thr) + wave * mp.rows_local;               // wave-private [rows_local]
    float* s_scl = reinterpret_cast<float*>(lds + mp.lds_scl) + wave * seg_stride;              // wave-private [seg] item scales

    // ---- schedule.  A visit is seg_per_visit consecutive segments; workgroup x owns visits x,
    // x + gridDim.x, ...  Its segments, in that order, are numbered 0, 1, ...; wavefront w starts on
    // number w and draws every further one from a counter in LDS, so that no wavefront of the
    // workgroup idles while another still has segments queued.  A stage is one (segment, filter
    // batch) of a wavefront.
    const int seg_items = p.seg_items;
    const int SW = seg_items >> 6;  // mask words per segment (1, 2, 4 or 8)
    const int spv = p.seg_per_visit;
    const int64_t item_lim = p.samp_role == 1 ? p.n_items : (p.item_end < p.n_items ? p.item_end : p.n_items);
    const int n_seg = (int)((p.item_end - p.item_begin + seg_items - 1) / seg_items);
    const int n_visit = (n_seg + spv - 1) / spv;
    const int n_batches = (p.n_groups + FB - 1) / FB;
    const int wg_visits = (int)blockIdx.x < n_visit ? (n_visit - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x : 0;
    const int wg_segs = wg_visits * spv;  // the last visit of the level may hold fewer: those have no items
    const int R = LEAN ? 1 : mp.region_slots;
    const int nq_pad = mp.rows_local / TT + 1;  // counters per region slot
    uint32_t* s_work = s_cnt + R * nq_pad;      // next segment number of the workgroup
    struct Stage {
        int num;    // segment number within the workgroup (>= wg_segs: none, the work has run out)
        int batch;  // filter batch
    };
    auto stage_ok = [&](const Stage& st) { return st.num < wg_segs; };
    auto stage_visit = [&](const Stage& st) { return st.num / spv; };  // among the workgroup's visits
    auto stage_seg = [&](const Stage& st) {  // segment index in the level (may lie past its end: no items there)
        const int i = st.num / spv;
        return ((int)blockIdx.x + i * (int)gridDim.x) * spv + (st.num - i * spv);
    };
    auto seg_first = [&](const Stage& st) -> int64_t {  // first item of the stage's segment
        const int64_t sg = stage_seg(st);
        return p.samp_role == 1 ? sg * p.samp_stride_items : p.item_begin + sg * seg_items;
    };
    auto in_sample = [&](int64_t first) -> bool {  // role 2: the 64-item word at `first` belongs to the sample
        if (p.samp_role != 2) return false;
        const uint32_t fw = (uint32_t)(first >> 6), sw = (uint32_t)(p.samp_stride_items >> 6);  // in words: 32 bits do
        const uint32_t j = fw / sw;
        return j < (uint32_t)p.samp_segs && fw - j * sw < (uint32_t)(p.samp_seg_items >> 6);
    };
    auto stage_next = [&](const Stage& st) -> Stage {
        if (!stage_ok(st)) return st;
        if (st.batch + 1 < n_batches) return Stage{st.num, st.batch + 1};
        uint32_t v = 0;
        if (lane == 0) v = atomicAdd(s_work, 1u);
        return Stage{__builtin_amdgcn_readfirstlane((int)v), 0};
    };
    Stage cur{wave, 0};

    // Bloom words: lane (gi * SW + w) owns word w of filter gi of the stage's batch.
    const bool pair_lane = lane < FB * SW;
    const int pr_gi = lane / SW, pr_w = lane - pr_gi * SW;
    uint64_t pre[PR];
    int pre_valid = 0;  // rows of the current stage that were prefetched
#pragma unroll
    for (int r = 0; r < PR; ++r) pre[r] = ~0ULL;
    auto prefetch_issue = [&](const Stage& st) {
        if (!pair_lane || !stage_ok(st)) return;
        const int g = st.batch * FB + pr_gi;
        if (g >= p.n_groups) return;
        const int64_t gw = (seg_first(st) >> 6) + pr_w;
        if (gw * 64 >= item_lim) return;
        const uint64_t* base = p.bloom + ((gw >> 4) * (int64_t)p.m_bits) * kTileWords + (gw & 15);
#pragma unroll
        for (int r = 0; r < PR; ++r) {
            const int row = s_prow[g * kPrefetchStride + r];
            pre[r] = row >= 0 ? base[(int64_t)row * kTileWords] : ~0ULL;
        }
    };
    // item scales of a stage's segment: lane l fetches items 4l .. 4l+3 and, in a 512-item
    // segment, 256+4l .. 256+4l+3 (zero past the end)
    float4 pre_sc = make_float4(0.f, 0.f, 0.f, 0.f), pre_sc2 = pre_sc;
    auto scale_fetch = [&](int64_t i0) -> float4 {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (i0 + 3 < item_lim) {
            v = *reinterpret_cast<const float4*>(p.iscale + i0);
        } else {
            if (i0 < item_lim) v.x = p.iscale[i0];
            if (i0 + 1 < item_lim) v.y = p.iscale[i0 + 1];
            if (i0 + 2 < item_lim) v.z = p.iscale[i0 + 2];
        }
        return v;
    };
    auto scale_issue = [&](const Stage& st) {
        pre_sc = pre_sc2 = make_float4(0.f, 0.f, 0.f, 0.f);
        if (!stage_ok(st) || 4 * lane >= seg_items) return;
        const int64_t i0 = seg_first(st) + 4 * lane;
        pre_sc = scale_fetch(i0);
        if (!LEAN && seg_items > 256) pre_sc2 = scale_fetch(i0 + 256);
    };
    auto prefetch_mask = [&](const Stage& st) -> uint64_t {  // mask word of my (filter, word) pair for the stage
        if (!pair_lane) return 0ULL;
        const int g = st.batch * FB + pr_gi;
        if (g >= p.n_groups) return 0ULL;
        const int64_t gw = (seg_first(st) >> 6) + pr_w;
        const int64_t first = gw * 64;
        if (first >= item_lim || in_sample(first)) return 0ULL;
        const int64_t left = item_lim - first;
        uint64_t mask = left >= 64 ? ~0ULL : ((1ULL << left) - 1ULL);
#pragma unroll
        for (int r = 0; r < PR; ++r) mask &= pre[r];
        const int r0 = s_rowoff[g], nr = s_rowoff[g + 1] - r0;
        if (nr > pre_valid) {  // long filters: the remaining rows, not prefetched
            const uint64_t* base = p.bloom + ((gw >> 4) * (int64_t)p.m_bits) * kTileWords + (gw & 15);
            for (int r = pre_valid; r < nr; ++r) mask &= base[(int64_t)p.grp_rows[r0 + r] * kTileWords];
        }
        return mask;
    };
    // ---- first Bloom words: rows from the kernel arguments, requested before any table is read
    if (pair_lane && stage_ok(cur)) {
        uint64_t pk[4] = {0, 0, 0, 0};
        int nr = 0;
#pragma unroll
        for (int g = 0; g < FB; ++g)
            if (pr_gi == g) {
#pragma unroll
                for (int c = 0; c < PR / 4; ++c) pk[c] = mp.prow_pack[g][c];
                nr = (int)((mp.prow_n >> (8 * g)) & 255);
            }
        const int64_t gw = (seg_first(cur) >> 6) + pr_w;
        if (pr_gi < p.n_groups && gw * 64 < item_lim) {
            const uint64_t* base = p.bloom + ((gw >> 4) * (int64_t)p.m_bits) * kTileWords + (gw & 15);
#pragma unroll
            for (int r = 0; r < PR; ++r) {
                const int row = (int)((pk[r >> 2] >> (16 * (r & 3))) & 0xFFFF);
                if (r < nr) pre[r] = base[(int64_t)row * kTileWords];
            }
        }
    }
    scale_issue(cur);

    // ---- workgroup-wide set-up: tables and resident queries into LDS.  The compiler keeps a
    // global load behind the LDS stores that precede it, so a copy loop per table would pay one
    // memory round trip each.  The first share of every table (all of it for ordinary sizes) is
    // therefore requested up front, into registers, and stored afterwards; loops take what is left.
    const int n_prow = p.n_groups * kPrefetchStride;
    const int n_piece = mp.first_level ? 0 : mp.rows_local * CH;   // 16-byte pieces of the query image
    const int n_imgrow = mp.first_level ? 0 : mp.rows_local;
    const int4* gq = reinterpret_cast<const int4*>(mp.img_q + (int64_t)y * mp.rows_local * D);
    {
        const int v_prow = mp.prow[tid < n_prow ? tid : 0];
        const int gc = tid <= p.n_groups ? tid : 0;
        const int v_rowoff = p.grp_row_off[gc];
        const int v_b0 = mp.grp_blk_off[gc < p.n_groups ? gc : 0], v_b1 = mp.grp_blk_off[gc < p.n_groups ? gc + 1 : 0];
        int4 v_img[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = tid + u * kThreads;
            v_img[u] = i < n_piece ? gq[i] : make_int4(0, 0, 0, 0);
        }
        int v_qrow = -1;
        float v_sq = 0.0f;
        uint64_t v_tau = 0;
        if (tid < n_imgrow) {
            v_qrow = mp.img_qrow[y * mp.rows_local + tid];
            v_sq = mp.img_sq[y * mp.rows_local + tid];
            v_tau = ~0ULL;
            for (int pp = 0; pp < p.tau_parts; ++pp)
                v_tau = min(v_tau, mp.img_tau[(int64_t)(y * (mp.rows_local / TT) + tid / TT) * kTauParts + pp]);
        }
        if (tid < n_prow) s_prow[tid] = v_prow;
        if (tid <= p.n_groups) {
            s_rowoff[tid] = v_rowoff;
            if (tid < p.n_groups) {  // the group's 16-row blocks that live in this row of workgroups
                const int bf = v_b0 + ((y - v_b0) % S + S) % S;
                s_gnblk[tid] = bf < v_b1 ? (v_b1 - bf + S - 1) / S : 0;
                s_glrow[tid] = (bf / S) * 16;
            }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = tid + u * kThreads;
            if (i < n_piece) reinterpret_cast<int4*>(s_q)[i] = v_img[u];
        }
        if (tid < n_imgrow) {
            s_qrow[tid] = v_qrow;
            s_sq[tid] = v_sq;
            const float tf = v_qrow >= 0 ? (v_tau ? key_score(v_tau) : -__builtin_inff()) : __builtin_inff();
            s_tauf[tid] = tf;
            if (!WEIGHTED) s_tq[tid] = tq_of(tf, v_sq);
            if ((tid % TT) == 0) s_tau64[tid / TT] = v_tau;
        }
    }
    for (int i = tid; i < R * nq_pad; i += kThreads) s_cnt[i] = 0;
    if (tid == 0) *s_work = (uint32_t)NW;  // numbers 0 .. NW-1 are the wavefronts' first segments
    for (int i = tid + kThreads; i < n_prow; i += kThreads) s_prow[i] = mp.prow[i];
    for (int g = tid + kThreads; g <= p.n_groups; g += kThreads) {
        s_rowoff[g] = p.grp_row_off[g];
        if (g < p.n_groups) {
            const int b0 = mp.grp_blk_off[g], b1 = mp.grp_blk_off[g + 1];
            const int bf = b0 + ((y - b0) % S + S) % S;
            s_gnblk[g] = bf < b1 ? (b1 - bf + S - 1) / S : 0;
            s_glrow[g] = (bf / S) * 16;
        }
    }
    if (mp.first_level) {
        // Resident state straight from the tables.  Two dependent reads per entry (row index, then
        // the row's data); as above, all reads of one stage are issued before anything is stored.
        auto row_of = [&](int lr) -> int {
            const int b = (lr >> 4) * S + y;
            return (lr < mp.rows_local && b < mp.n_blocks) ? mp.blk_row[b * 16 + (lr & 15)] : -1;
        };
        const int n_piece_t = mp.rows_local * CH;
        for (int lr0 = 0, i0 = 0; lr0 < mp.rows_local || i0 < n_piece_t; lr0 += kThreads, i0 += 8 * kThreads) {
            const int lr = lr0 + tid;
            const int grow = row_of(lr);
            int grow_p[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = i0 + tid + u * kThreads;
                grow_p[u] = i < n_piece_t ? row_of(i / CH) : -1;
            }
            const float sq = grow >= 0 ? p.qscale[grow] : 0.0f;
            uint64_t t64 = 0ULL;
            if (grow >= 0 && p.use_tau) {
                t64 = ~0ULL;
                for (int pp = 0; pp < p.tau_parts; ++pp) t64 = min(t64, p.tau[(int64_t)(grow / TT) * kTauParts + pp]);
            }
            int4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = i0 + tid + u * kThreads;
                v[u] = make_int4(0, 0, 0, 0);
                if (grow_p[u] >= 0) v[u] = reinterpret_cast<const int4*>(p.queries + (int64_t)grow_p[u] * D)[i % CH];
            }
            if (lr < mp.rows_local) {
                s_qrow[lr] = grow;
                s_sq[lr] = sq;
                const float tf = grow >= 0 ? (t64 ? key_score(t64) : -__builtin_inff()) : __builtin_inff();
                s_tauf[lr] = tf;
                if (!WEIGHTED) s_tq[lr] = tq_of(tf, sq);
                if ((lr % TT) == 0) s_tau64[lr / TT] = t64;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int i = i0 + tid + u * kThreads;
                if (i < n_piece_t) {
                    const int r = i / CH, c = i % CH;
                    *reinterpret_cast<int4*>(s_q + r * D + ((c ^ swz<KS>(r)) << 4)) = v[u];
                }
            }
        }
        lds_barrier();
        if (blockIdx.x == 0) {  // publish the image for the later levels
            int4* gq = reinterpret_cast<int4*>(mp.img_q + (int64_t)y * mp.rows_local * D);
            for (int i = tid; i < mp.rows_local * CH; i += kThreads) gq[i] = reinterpret_cast<const int4*>(s_q)[i];
            for (int lr = tid; lr < mp.rows_local; lr += kThreads) {
                mp.img_sq[y * mp.rows_local + lr] = s_sq[lr];
                mp.img_qrow[y * mp.rows_local + lr] = s_qrow[lr];
            }
        }
    } else {
        // what the first share above did not cover
        for (int i = tid + 8 * kThreads; i < n_piece; i += kThreads) reinterpret_cast<int4*>(s_q)[i] = gq[i];
        for (int lr = tid + kThreads; lr < mp.rows_local; lr += kThreads) {
            const int grow = mp.img_qrow[y * mp.rows_local + lr];
            s_qrow[lr] = grow;
            const float sq = mp.img_sq[y * mp.rows_local + lr];
            s_sq[lr] = sq;
            uint64_t t64 = ~0ULL;
            for (int pp = 0; pp < p.tau_parts; ++pp)
                t64 = min(t64, mp.img_tau[(int64_t)(y * (mp.rows_local / TT) + lr / TT) * kTauParts + pp]);
            const float tf = grow >= 0 ? (t64 ? key_score(t64) : -__builtin_inff()) : __builtin_inff();
            s_tauf[lr] = tf;
            if (!WEIGHTED) s_tq[lr] = tq_of(tf, sq);
            if ((lr % TT) == 0) s_tau64[lr / TT] = t64;
        }
        lds_barrier();
    }

    // lane constants of the MFMA operand reads: byte offset of this lane's chunk k inside a
    // 16-row query block (the swizzle of row lrow + l16 depends on l16 only: lrow is a multiple
    // of 16), and of its four rows in the per-row tables
    int a_off[KS];
#pragma unroll
    for (int k = 0; k < KS; ++k) a_off[k] = l16 * D + (((kg + 4 * k) ^ swz<KS>(l16)) << 4);

    int thr_E = -1000;  // exponent the wavefront's integer bounds were built for (none yet)
    for (bool first = true; stage_ok(cur); first = false) {
        const int64_t item0 = seg_first(cur);
        const int g0 = cur.batch * FB;
        const int nf = min(FB, p.n_groups - g0);
        // candidate region: one per visit on the first level (a region then holds the candidates of
        // at most `cap` items and cannot overflow), afterwards the workgroup's regions take turns
        // segment by segment, which spreads the load over all of them even in a short level
        const int slot = R == 1 ? 0 : (p.use_tau ? cur.num : stage_visit(cur)) % R;
        const int region = (int)blockIdx.x + slot * (int)gridDim.x + y * (int)gridDim.x * R;
        uint32_t* cnt_s = s_cnt + slot * nq_pad;

        // (1) + (2): mask word of my pair, then the set bits of each filter's words, in item
        // order, into the filter's list
        pre_valid = PR;  // (the first stage's rows came from the kernel arguments, as many)
        uint64_t mask = prefetch_mask(cur);
        const Stage nxt = stage_next(cur);
#pragma unroll
        for (int r = 0; r < PR; ++r) pre[r] = ~0ULL;
        prefetch_issue(nxt);
        const int c = __popcll(mask);
        int incl = c;  // running count over the words of my filter
        // (the words of a filter sit in neighbouring lanes of one 16-lane row: register moves, no shuffles)
        if (SW > 1) { const int v = (int)row_shr<1>((uint32_t)incl); if (pr_w >= 1) incl += v; }
        if (SW > 2) { const int v = (int)row_shr<2>((uint32_t)incl); if (pr_w >= 2) incl += v; }
        if (SW > 4) { const int v = (int)row_shr<4>((uint32_t)incl); if (pr_w >= 4) incl += v; }
        {
            int pos = incl - c;
            uint8_t* list = s_list + pr_gi * seg_stride;
            while (mask) {
                const int b = __ffsll((long long)mask) - 1;
                mask &= mask - 1;
                list[pos++] = (uint8_t)(pr_w * 64 + b);
            }
        }
        // list size of filter gi -> lane gi; 16-item units per filter and their running sum
        // (the shuffle runs in every lane: a lane switched off would read as 0 for the others)
        const int last_word = __shfl(incl, (lane * SW + SW - 1) & 63);
        const int low_words = LEAN ? last_word : __shfl(incl, (lane * SW + (SW > 4 ? 3 : SW - 1)) & 63);  // entries of the lower 256 items
        const int gcount = lane < nf ? last_word : 0;
        const int glow = lane < nf ? low_words : 0;
        const int gunits = (gcount + 15) >> 4;
        int ucum = gunits;  // inclusive over filters
        static_assert(FB == 8, "three steps cover the filters of a batch");
        { const int v = (int)row_shr<1>((uint32_t)ucum); if (lane >= 1) ucum += v; }
        { const int v = (int)row_shr<2>((uint32_t)ucum); if (lane >= 2) ucum += v; }
        { const int v = (int)row_shr<4>((uint32_t)ucum); if (lane >= 4) ucum += v; }
        const int n_units = __builtin_amdgcn_readlane(ucum, FB - 1);
        // first local query row and local block count of filter gi -> lane gi
        const int glrow = lane < nf ? s_glrow[g0 + lane] : 0;
        const int gnblk = lane < nf ? s_gnblk[g0 + lane] : 0;

        // Item scales of the segment into LDS.  Plain search: their maximum fixes a power of two
        // 2^E above every scale of the segment; the lane's scale becomes the fixed-point factor
        // ceil(s_i * 2^(31-E)) and every row gets the integer bound floor(tau / s_q * 2^-(E+1)),
        // shaved by more than all roundings involved.  A pair can only be admitted if
        // mulhi(dot, factor) reaches the bound of its row, which costs two integer instructions per
        // pair; the exact fp32 arithmetic runs when an entry is drained from the queue.  The bounds
        // depend on the segment through E only and are rebuilt when E changes (rarely: scales of
        // neighbouring segments are of one magnitude).
        float fix_scale = 0.0f;  // 2^(31-E); 0: no cull in this segment
        {
            const float4 sc4 = pre_sc, sc4b = pre_sc2;
            scale_issue(nxt);
            if (4 * lane < seg_items) *reinterpret_cast<float4*>(s_scl + 4 * lane) = sc4;
            if (!LEAN && seg_items > 256) *reinterpret_cast<float4*>(s_scl + 256 + 4 * lane) = sc4b;
            if (!WEIGHTED && n_units > 0) {
                float smax = fmaxf(fmaxf(sc4.x, sc4.y), fmaxf(sc4.z, sc4.w));
                smax = fmaxf(smax, fmaxf(fmaxf(sc4b.x, sc4b.y), fmaxf(sc4b.z, sc4b.w)));
                // the largest of the wavefront: scales are positive, so their bit patterns order as they
                // do (a negative or non-finite scale comes out on top and switches the cull off below)
                smax = __uint_as_float(lane_value(wave_max_u32(__float_as_uint(smax)), 63));
                int E = 0;
                bool cull = smax > 0.0f && smax < __builtin_inff();
                if (cull) {
                    E = ilogbf(smax) + 1;  // 2^E > smax
                    cull = E > -90 && E < 90;
                }
                fix_scale = cull ? ldexpf(1.0f, 31 - E) : 0.0f;
                const float thr_scale = ldexpf(0.99999618530273f, -(E + 1));  // (1 - 2^-18) * 2^-(E+1)
                const int e_code = cull ? E : 1000;
                const bool rebuild = e_code != thr_E;
                thr_E = e_code;
                for (int row = lane; rebuild && row < mp.rows_local; row += 64) {
                    const float tq = s_tq[row];
                    int thr = (int)0x80000000;  // no bound
                    if (tq == __builtin_inff())
                        thr = 0x7FFFFFFF;       // padding row
                    else if (cull && tq > 0.0f)
                        thr = __float2int_rd(fminf(tq * thr_scale, 2.0e9f));
                    s_thr[row] = thr;
                }
            }
        }

        // (3) units = (filter gi, 16 passing items from b0), in filter order.  A ring of NB
        // register slots keeps the item rows of the next NB units in flight while one is
        // contracted: uniform bases + 32-bit lane offsets (the segment spans at most 512 * D bytes)
        const char* seg_rows = reinterpret_cast<const char*>(p.items + item0 * D) + kg * 16;
        int qn = 0;          // queued admissions (uniform)
        int cur_lrow = -1;   // query block whose A operand (and per-row constants) sit in registers
        float4 cur_sq = make_float4(0.f, 0.f, 0.f, 0.f), cur_tf = cur_sq;  // weighted search
        int4 cur_thr = make_int4(0, 0, 0, 0);                              // plain search
        v4i areg[KS];

        // unit generator: (gen_gi, gen_b0) is the next unit to request; it stays on the last unit
        // once all have been produced, so that requests past the end are harmless repeats
        int gen_gi = 0, gen_b0 = 0, gen_n = 0, gen_low = 0, gen_left = 0;
        auto gen_seek = [&](int u) {  // position on unit u (cold)
            gen_gi = __popcll(ballot(lane < nf && ucum <= u));
            gen_b0 = (u - (__builtin_amdgcn_readlane(ucum, gen_gi) - __builtin_amdgcn_readlane(gunits, gen_gi))) << 4;
            gen_n = __builtin_amdgcn_readlane(gcount, gen_gi);
            gen_low = __builtin_amdgcn_readlane(glow, gen_gi);
            gen_left = n_units - 1 - u;
        };
        auto unit_load = [&](UnitRegs<KS>& w) {
            const int li = gen_b0 + l16;
            const int at = min(li, gen_n - 1);
            const int idx = (int)s_list[gen_gi * seg_stride + at] + (!LEAN && at >= gen_low ? 256 : 0);
            w.item = li < gen_n ? idx : -1;
            w.gi = gen_gi;
            const uint32_t off = (uint32_t)(idx * D);
#pragma unroll
            for (int k = 0; k < KS; ++k) {
                const int4 v = *reinterpret_cast<const int4*>(seg_rows + (off + 64u * k));
                w.b[k] = v4i{v.x, v.y, v.z, v.w};
            }
            w.si = s_scl[idx];
            w.si_fix = 0;
            if (!WEIGHTED) w.si_fix = __float2int_ru(w.si * fix_scale);  // < 2^31: s_i < 2^E
            if (gen_left > 0) {  // advance (scalar)
                --gen_left;
                gen_b0 += 16;
                while (gen_b0 >= gen_n) {
                    ++gen_gi;
                    gen_b0 = 0;
                    gen_n = __builtin_amdgcn_readlane(gcount, gen_gi);
                    gen_low = __builtin_amdgcn_readlane(glow, gen_gi);
                }
            }
        };
        // A lane whose block test leaves an admission possible is queued as it is (wave-private LDS,
        // positions from a ballot: no waiting): its four values -- the int32 dot products (plain
        // search, rescaled when drained) or the aggregated scores (weighted search) -- and a code
        // with the first of its four local rows and the item's place in the segment.  The queue is
        // drained 64 lanes at a time, so that keys, the comparisons with the queries' threshold
        // keys and the LDS round trips of the counter updates are paid with every lane at work.
        //
        // The store of a drained candidate is written in assembly.  On this target loads and stores
        // share one outstanding-operation counter; a store the compiler knows of, possibly pending,
        // turns every later wait for a unit's rows into a wait for all younger loads as well, which
        // would flatten the row pipeline.  This way the compiler keeps counting loads only.  A store
        // it does not know of can only make one of its waits last longer, never end early: a wait
        // for "at most n operations outstanding" is met once enough operations have completed, the
        // loads complete in the order they were issued, so the load waited for is among them with
        // or without the store.  (Nothing in the kernel reads the stored keys back.)
        auto drain_lanes = [&]() {  // empties the queue: one queued lane (an item and four query rows) per lane
            if (lane < qn) {
                const int4 a4 = q_acc[lane];
                const uint32_t code = q_code[lane];
                const int lrow4 = (int)(code >> 9);  // first of the lane's four local rows
                const int it = (int)(code & 511u);
                const float si = s_scl[it];
                const float4 sq4 = *reinterpret_cast<const float4*>(s_sq + lrow4);
                const int4 qr4 = *reinterpret_cast<const int4*>(s_qrow + lrow4);
                const int accv[4] = {a4.x, a4.y, a4.z, a4.w};
                const float sqv[4] = {sq4.x, sq4.y, sq4.z, sq4.w};
                const int qrv[4] = {qr4.x, qr4.y, qr4.z, qr4.w};
#pragma unroll
                for (int q0 = 0; q0 < 4; q0 += TT) {
                    // weighted search: the aggregate of query q0 was queued; plain: its int32 dot product
                    const float score = WEIGHTED ? __uint_as_float((uint32_t)accv[q0]) : rescale(accv[q0], sqv[q0], si);
                    const uint64_t key = make_key(score, (uint32_t)(item0 + it));
                    const int srow = lrow4 + q0, grow = qrv[q0];
                    if (grow >= 0 && key >= s_tau64[srow / TT]) {
                        const uint32_t at = atomicAdd(&cnt_s[srow / TT], 1u);
                        if (at < (uint32_t)p.cap) {
                            uint64_t* dst = p.cand + ((int64_t)(grow / TT) * p.groups + region) * p.cap + at;
                            asm volatile("global_store_dwordx2 %0, %1, off" : : "v"(dst), "v"(key) : "memory");
                        }
                    }
                }
            }
            qn = 0;
        };
        // The queue pair by pair: an entry holds the local row, the item's place in the segment and
        // the aggregated score (weighted search) or the int32 dot product (plain search).
        auto drain_pairs = [&]() {  // takes the last (up to) 64 queued entries; the order inside a region is free
            const int base = qn > 64 ? qn - 64 : 0;
            if (base + lane < qn) {
                const uint64_t e = s_queue[base + lane];
                const int srow = (int)((uint32_t)e >> 9);  // local row of the query's first task
                const int it = (int)(e & 511u);
                float score;
                if (WEIGHTED)
                    score = __uint_as_float((uint32_t)(e >> 32));
                else
                    score = rescale((int)(uint32_t)(e >> 32), s_sq[srow], s_scl[it]);
                const uint64_t key = make_key(score, (uint32_t)(item0 + it));
                const int grow = s_qrow[srow];
                if (grow >= 0 && key >= s_tau64[srow / TT]) {
                    const uint32_t at = atomicAdd(&cnt_s[srow / TT], 1u);
                    if (at < (uint32_t)p.cap) {
                        uint64_t* dst = p.cand + ((int64_t)(grow / TT) * p.groups + region) * p.cap + at;
                        asm volatile("global_store_dwordx2 %0, %1, off" : : "v"(dst), "v"(key) : "memory");
                    }
                }
            }
            qn = base;
        };
        // Weighted search: scores of one block's accumulators (this lane: one item, four query
        // rows; the aggregate of query q0 is left in sc[q0]) and the lanes with an admission.
        auto block_scores = [&](const float4& sq4, const float4& tf4, const v4i& acc, const UnitRegs<KS>& w, uint64_t valid,
                                uint32_t (&val)[4], uint64_t (&hits)[4]) -> bool {
            const float sqv[4] = {sq4.x, sq4.y, sq4.z, sq4.w};
            const float tfv[4] = {tf4.x, tf4.y, tf4.z, tf4.w};
            float sc[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) sc[r] = rescale(acc[r], sqv[r], w.si);
            // Value-Model sum over the TT tasks of each query this lane holds
#pragma unroll
            for (int q0 = 0; q0 < 4; q0 += TT) {
                float agg = 0.0f;
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) agg = __fmaf_rn(p.w[tt], sc[q0 + tt], agg);
                sc[q0] = agg;
            }
            uint64_t any = 0;
#pragma unroll
            for (int r = 0; r < 4; r += TT) {
                hits[r] = ballot(sc[r] >= tfv[r]);
                val[r] = __float_as_uint(sc[r]);
                any |= hits[r];
            }
            return (any & valid) != 0;
        };
        // Plain search: the integer cull; candidates carry their int32 dot product.
        auto block_cull = [&](const int4& thr, const v4i& acc, const UnitRegs<KS>& w, uint64_t valid, uint32_t (&val)[4],
                              uint64_t (&hits)[4]) -> bool {
            const int thv[4] = {thr.x, thr.y, thr.z, thr.w};
            uint64_t any = 0;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                hits[r] = ballot(__mulhi(acc[r], w.si_fix) >= thv[r]);
                val[r] = (uint32_t)acc[r];
                any |= hits[r];
            }
            return (any & valid) != 0;
        };
        // Queues the lanes of a block that hold a possible admission, as they are: the four values
        // of the lane and where its rows and its item are.  The exact test of each of the four
        // pairs runs when the queue is drained, with every lane at work.
        auto push_lanes = [&](int lrow, const UnitRegs<KS>& w, uint64_t valid, const uint32_t (&val)[4],
                              const uint64_t (&hits)[4]) {
            uint64_t m = 0;
#pragma unroll
            for (int r = 0; r < 4; r += TT) m |= hits[r];
            m &= valid;  // (non-zero: the caller has tested it)
            const int n = __popcll(m);
            if (qn + n > kQueueLanes) drain_lanes();
            if ((m >> lane) & 1ULL) {
                const int pos = qn + __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
                q_acc[pos] = make_int4((int)val[0], TT == 1 ? (int)val[1] : 0, TT <= 2 ? (int)val[2] : 0, TT == 1 ? (int)val[3] : 0);
                q_code[pos] = (uint32_t)(((lrow + 4 * kg) << 9) | w.item);
            }
            qn += n;
        };
        // Queues the candidates of a block (rare path).
        auto push_pairs = [&](int lrow, const UnitRegs<KS>& w, uint64_t valid, const uint32_t (&val)[4],
                              const uint64_t (&hits)[4]) {
#pragma unroll
            for (int r = 0; r < 4; r += TT) {
                const uint64_t m = hits[r] & valid;
                if (m) {  // uniform
                    if ((m >> lane) & 1ULL) {
                        const int pos = qn + __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32),
                                                                    __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
                        s_queue[pos] = ((uint64_t)val[r] << 32) | (uint32_t)(((lrow + 4 * kg + r) << 9) | w.item);
                    }
                    qn += __popcll(m);
                    if (qn >= 64) drain_pairs();
                }
            }
        };
        // Which form of the queue: whole lanes where a unit meets few query blocks (the exact test
        // of four pairs per queued lane is then cheaper than queueing pair by pair); pairs where two
        // units share every block's operands (dense batches: few lanes hold an admission, and the
        // pair form keeps fewer values alive across the blocks of a round).
        constexpr bool LANEQ = !PAIRS;
        auto block_push = [&](int lrow, const UnitRegs<KS>& w, uint64_t valid, const uint32_t (&val)[4],
                              const uint64_t (&hits)[4]) {
            if (LANEQ)
                push_lanes(lrow, w, valid, val, hits);
            else
                push_pairs(lrow, w, valid, val, hits);
        };
        auto drain_all = [&]() {
            if (LANEQ) {
                if (qn > 0) drain_lanes();
            } else {
                while (qn > 0) drain_pairs();
            }
        };
        auto block_a = [&](int lrow, v4i (&a)[KS]) {
            const int8_t* qp = s_q + lrow * D;
#pragma unroll
            for (int k = 0; k < KS; ++k) {
                const int4 v = *reinterpret_cast<const int4*>(qp + a_off[k]);
                a[k] = v4i{v.x, v.y, v.z, v.w};
            }
        };
        auto block_mfma = [&](const v4i (&a)[KS], const UnitRegs<KS>& w) -> v4i {
            v4i acc = {0, 0, 0, 0};
#pragma unroll
            for (int k = 0; k < KS; ++k) acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[k], w.b[k], acc, 0, 0, 0);
            return acc;
        };
        auto row_sq = [&](int lrow) { return *reinterpret_cast<const float4*>(s_sq + lrow + 4 * kg); };
        auto row_tf = [&](int lrow) { return *reinterpret_cast<const float4*>(s_tauf + lrow + 4 * kg); };
        auto row_thr = [&](int lrow) { return *reinterpret_cast<const int4*>(s_thr + lrow + 4 * kg); };
        // the per-row constants of one block (read from LDS together with its A operand, well before
        // the accumulators they are compared with exist) and the test that uses them
        struct RowK {
            float4 sq, tf;  // weighted search
            int4 thr;       // plain search
        };
        auto row_k = [&](int lrow) -> RowK {
            RowK k;
            k.sq = k.tf = make_float4(0.f, 0.f, 0.f, 0.f);
            k.thr = make_int4(0, 0, 0, 0);
            if (WEIGHTED) {
                k.sq = row_sq(lrow);
                k.tf = row_tf(lrow);
            } else {
                k.thr = row_thr(lrow);
            }
            return k;
        };
        auto block_test = [&](const RowK& k, const v4i& acc, const UnitRegs<KS>& w, uint64_t valid, uint32_t (&val)[4],
                              uint64_t (&hits)[4]) -> bool {
            if (WEIGHTED) return block_scores(k.sq, k.tf, acc, w, valid, val, hits);
            return block_cull(k.thr, acc, w, valid, val, hits);
        };
        // Contracts one unit with the query blocks of its filter group, two blocks per round (the
        // operands of both are read before either is used).  A group of a single block keeps its
        // A operand and per-row constants in registers from one unit to the next.
        // First level with one segment per region: there is no threshold and every pair is a
        // candidate, so the queue and its counters are bypassed.  An item's place in its filter's
        // list is its place in the region of each of the filter's queries (the 16 lanes of a quarter
        // wavefront write 16 consecutive keys of one query), and the list length is the fill count.
        auto unit_admit_all = [&](const UnitRegs<KS>& w, int u) {
            const int lrow0 = __builtin_amdgcn_readlane(glrow, w.gi);
            const int nblk = __builtin_amdgcn_readlane(gnblk, w.gi);
            const int n = __builtin_amdgcn_readlane(gcount, w.gi);
            const int pos = ((u - (__builtin_amdgcn_readlane(ucum, w.gi) - __builtin_amdgcn_readlane(gunits, w.gi))) << 4) + l16;
            for (int j = 0; j < nblk; ++j) {
                const int lrow = lrow0 + 16 * j;
                v4i a[KS];
                block_a(lrow, a);
                const v4i acc = block_mfma(a, w);
                const float4 sq4 = row_sq(lrow);
                const float sqv[4] = {sq4.x, sq4.y, sq4.z, sq4.w};
                float sc[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) sc[r] = rescale(acc[r], sqv[r], w.si);
                if (WEIGHTED) {
#pragma unroll
                    for (int q0 = 0; q0 < 4; q0 += TT) {
                        float agg = 0.0f;
#pragma unroll
                        for (int tt = 0; tt < TT; ++tt) agg = __fmaf_rn(p.w[tt], sc[q0 + tt], agg);
                        sc[q0] = agg;
                    }
                }
#pragma unroll
                for (int r = 0; r < 4; r += TT) {
                    const int row = lrow + 4 * kg + r;
                    const int grow = s_qrow[row];
                    if (w.item >= 0 && grow >= 0) {
                        const uint64_t key = make_key(sc[r], (uint32_t)(item0 + w.item));
                        uint64_t* dst = p.cand + ((int64_t)(grow / TT) * p.groups + region) * p.cap + pos;
                        asm volatile("global_store_dwordx2 %0, %1, off" : : "v"(dst), "v"(key) : "memory");  // as in drain()
                        if (pos == n - 1) cnt_s[row / TT] = (uint32_t)n;
                    }
                }
            }
        };
        auto unit_compute = [&](const UnitRegs<KS>& w) {
            const int lrow0 = __builtin_amdgcn_readlane(glrow, w.gi);
            const int nblk = __builtin_amdgcn_readlane(gnblk, w.gi);
            uint32_t val[4];
            uint64_t hits[4];
            const uint64_t valid = ballot(w.item >= 0);  // lanes that hold a real item
            if (!MULTI || nblk == 1) {
                if (cur_lrow != lrow0) {
                    block_a(lrow0, areg);
                    if (WEIGHTED) {
                        cur_sq = row_sq(lrow0);
                        cur_tf = row_tf(lrow0);
                    } else {
                        cur_thr = row_thr(lrow0);
                    }
                    cur_lrow = lrow0;
                }
                const v4i acc = block_mfma(areg, w);
                const bool any = WEIGHTED ? block_scores(cur_sq, cur_tf, acc, w, valid, val, hits)
                                          : block_cull(cur_thr, acc, w, valid, val, hits);
                if (any) block_push(lrow0, w, valid, val, hits);
                return;
            }
            if (!MULTI) return;
            int j = 0;
            if (NW == 8 && KS <= 2) {  // four blocks per round: independent chains, where the registers allow it
                for (; j + 4 <= nblk; j += 4) {
                    const int l0 = lrow0 + 16 * j;
                    v4i a0[KS], a1[KS], a2[KS], a3[KS];
                    uint32_t v0[4], v1[4], v2[4], v3[4];
                    uint64_t h0[4], h1[4], h2[4], h3[4];
                    block_a(l0, a0);
                    block_a(l0 + 16, a1);
                    block_a(l0 + 32, a2);
                    block_a(l0 + 48, a3);
                    const RowK k0 = row_k(l0), k1 = row_k(l0 + 16), k2 = row_k(l0 + 32), k3 = row_k(l0 + 48);
                    const v4i c0 = block_mfma(a0, w), c1 = block_mfma(a1, w), c2 = block_mfma(a2, w), c3 = block_mfma(a3, w);
                    const bool y0 = block_test(k0, c0, w, valid, v0, h0);
                    const bool y1 = block_test(k1, c1, w, valid, v1, h1);
                    const bool y2 = block_test(k2, c2, w, valid, v2, h2);
                    const bool y3 = block_test(k3, c3, w, valid, v3, h3);
                    if (y0) block_push(l0, w, valid, v0, h0);
                    if (y1) block_push(l0 + 16, w, valid, v1, h1);
                    if (y2) block_push(l0 + 32, w, valid, v2, h2);
                    if (y3) block_push(l0 + 48, w, valid, v3, h3);
                }
            }
            for (; j + 2 <= nblk; j += 2) {
                const int l0 = lrow0 + 16 * j;
                v4i a0[KS], a1[KS];
                uint32_t v0[4], v1[4];
                uint64_t h0[4], h1[4];
                block_a(l0, a0);
                block_a(l0 + 16, a1);
                const RowK k0 = row_k(l0), k1 = row_k(l0 + 16);
                const v4i c0 = block_mfma(a0, w), c1 = block_mfma(a1, w);
                const bool y0 = block_test(k0, c0, w, valid, v0, h0);
                const bool y1 = block_test(k1, c1, w, valid, v1, h1);
                if (y0) block_push(l0, w, valid, v0, h0);
                if (y1) block_push(l0 + 16, w, valid, v1, h1);
            }
            for (; j < nblk; ++j) {
                v4i a[KS];
                uint32_t val[4];
                uint64_t hits[4];
                block_a(lrow0 + 16 * j, a);
                const RowK k = row_k(lrow0 + 16 * j);
                const v4i acc = block_mfma(a, w);
                if (block_test(k, acc, w, valid, val, hits)) block_push(lrow0 + 16 * j, w, valid, val, hits);
            }
        };
        // Two units of one filter group at once: every block's operands serve both.
        auto unit_compute2 = [&](const UnitRegs<KS>& w0, const UnitRegs<KS>& w1) {
            const int lrow0 = __builtin_amdgcn_readlane(glrow, w0.gi);
            const int nblk = __builtin_amdgcn_readlane(gnblk, w0.gi);
            const uint64_t valid0 = ballot(w0.item >= 0), valid1 = ballot(w1.item >= 0);
            int j = 0;
            for (; j + 2 <= nblk; j += 2) {
                const int l0 = lrow0 + 16 * j;
                v4i a0[KS], a1[KS];
                uint32_t v00[4], v01[4], v10[4], v11[4];
                uint64_t h00[4], h01[4], h10[4], h11[4];
                block_a(l0, a0);
                block_a(l0 + 16, a1);
                const RowK k0 = row_k(l0), k1 = row_k(l0 + 16);
                const v4i c00 = block_mfma(a0, w0), c01 = block_mfma(a0, w1), c10 = block_mfma(a1, w0), c11 = block_mfma(a1, w1);
                const bool y00 = block_test(k0, c00, w0, valid0, v00, h00);
                const bool y01 = block_test(k0, c01, w1, valid1, v01, h01);
                const bool y10 = block_test(k1, c10, w0, valid0, v10, h10);
                const bool y11 = block_test(k1, c11, w1, valid1, v11, h11);
                if (y00) block_push(l0, w0, valid0, v00, h00);
                if (y01) block_push(l0, w1, valid1, v01, h01);
                if (y10) block_push(l0 + 16, w0, valid0, v10, h10);
                if (y11) block_push(l0 + 16, w1, valid1, v11, h11);
            }
            for (; j < nblk; ++j) {
                const int l0 = lrow0 + 16 * j;
                v4i a[KS];
                uint32_t v0[4], v1[4];
                uint64_t h0[4], h1[4];
                block_a(l0, a);
                const RowK k = row_k(l0);
                const v4i c0 = block_mfma(a, w0), c1 = block_mfma(a, w1);
                const bool y0 = block_test(k, c0, w0, valid0, v0, h0);
                const bool y1 = block_test(k, c1, w1, valid1, v1, h1);
                if (y0) block_push(l0, w0, valid0, v0, h0);
                if (y1) block_push(l0, w1, valid1, v1, h1);
            }
        };
        // Every load in the loop is unconditional (requests past the end repeat the last unit):
        // only then is the number of loads between a unit's request and its use a constant the
        // compiler can wait on.
        if (n_units > 0) {
            UnitRegs<KS> r0, r1, r2, r3;  // the ring, as separate variables (an array would be indexed through memory)
            auto step = [&](UnitRegs<KS>& r, int u) {
                if (u < n_units) {
                    if (ADMIT)
                        unit_admit_all(r, u);
                    else
                        unit_compute(r);
                }
                unit_load(r);
            };
            auto step2 = [&](UnitRegs<KS>& ra, UnitRegs<KS>& rb, int u) {
                if (u + 1 < n_units && ra.gi == rb.gi && __builtin_amdgcn_readlane(gnblk, ra.gi) > 1) {
                    unit_compute2(ra, rb);
                } else {
                    if (u < n_units) unit_compute(ra);
                    if (u + 1 < n_units) unit_compute(rb);
                }
                unit_load(ra);
                unit_load(rb);
            };
            gen_seek(0);
            unit_load(r0);
            unit_load(r1);
            if (NB > 2) unit_load(r2);
            if (NB > 3) unit_load(r3);
            for (int base = 0; base < n_units; base += NB) {
                if (PAIRS && !ADMIT) {
                    step2(r0, r1, base);
                    step2(r2, r3, base + 2);
                } else {
                    step(r0, base);
                    step(r1, base + 1);
                    if (NB > 2) step(r2, base + 2);
                    if (NB > 3) step(r3, base + 3);
                }
            }
            drain_all();
        }
        cur = nxt;
    }
    __syncthreads();
    // region fill counts: real ones for the queries this workgroup row owns, zero for the others
    for (int i = tid * TT; i < mp.n_blocks * 16; i += kThreads * TT) {
        const int grow = mp.blk_row[i];
        if (grow < 0) continue;
        const int q = grow / TT;
        const int b = i >> 4;
        for (int j = 0; j < R; ++j) {
            uint32_t c = 0;
            if (b % S == y) c = s_cnt[j * nq_pad + ((b / S) * 16 + (i & 15)) / TT];
            const int region = (int)blockIdx.x + j * (int)gridDim.x + y * (int)gridDim.x * R;
            p.cnt[(int64_t)q * p.groups + region] = c < (uint32_t)p.cap ? c : (uint32_t)p.cap;
            if (c > (uint32_t)p.cap) p.ovf[q] = 1u;
        }
    }
}

template <int KS, int TT, bool WEIGHTED, bool MULTI, int NW, bool ADMIT = false>
__global__ __launch_bounds__(NW * 64, (NW == 8 ? 2 : (KS <= 2 ? 4 : 2))) void scan_mfma_kernel(ScanParams p, MfmaParams mp)
{
    if (ADMIT && mp.density_acc && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *mp.density_acc = 0ULL;
    scan_mfma_body<KS, TT, WEIGHTED, MULTI, NW, ADMIT>(p, mp);
}

inline bool mfma_shape_ok(int d, int n_tasks)
{
    return (d == 64 || d == 128 || d == 256 || d == 512) && (n_tasks == 1 || n_tasks == 2 || n_tasks == 4);
}

// LDS one workgroup needs with the resident queries split S ways, `waves` wavefronts and
// `slots` candidate regions.
inline int mfma_lds_bytes(int n_blocks, int S, int d, int n_tasks, int n_groups, int waves, int slots, int seg_stride = 256);

// Candidate regions per workgroup when a compute unit holds `wgs` workgroups: all regions are
// shared out among the workgroups that are resident at once.
inline int mfma_region_slots(int wgs)
{
    const int resident = kComputeUnits * wgs;
    int r = (scan_groups() + resident - 1) / resident;
    return r < 1 ? 1 : (r > kMaxRegionSlots ? kMaxRegionSlots : r);
}

// Chooses the split S of the resident queries over rows of workgroups (every row scans the
// corpus for its share of the queries) and the wavefronts per workgroup.  Cost model: passes
// over the corpus divided by the wavefronts a compute unit holds at once (160 KB of LDS; at most
// 16 wavefronts for d <= 128 and 8 above, from the register budget).  Ties go to fewer passes.
inline void mfma_choose_config(int n_blocks, int d, int n_tasks, int n_groups, int max_split, int* out_S, int* out_waves,
                               int* out_wgs)
{
    const int wave_cap = d <= 128 ? 16 : 8;
    double best = 1e30;
    int best_S = 0, best_w = 4, best_wgs = 1;
    for (int S = 1; S <= max_split; S <<= 1) {
        for (int waves = 4; waves <= 8; waves += 4) {
            // workgroups per compute unit; fewer of them means more region slots each, which
            // takes a little more LDS: settle from the pessimistic side
            int wgs = 0;
            for (int slots = kMaxRegionSlots; slots >= 1; --slots) {
                const int lds = mfma_lds_bytes(n_blocks, S, d, n_tasks, n_groups, waves, slots);
                if (lds > 160 * 1024) continue;
                int w = (160 * 1024) / lds;
                if (w * waves > wave_cap) w = wave_cap / waves;
                if (w >= 1 && mfma_region_slots(w) <= slots) wgs = w;
            }
            if (wgs < 1) continue;
            const double cost = (double)S / (double)(wgs * waves);
            if (cost < best * 0.999) {
                best = cost;
                best_S = S;
                best_w = waves;
                best_wgs = wgs;
            }
        }
    }
    *out_S = best_S;  // 0: not even the largest split fits
    *out_waves = best_w;
    *out_wgs = best_wgs;
}

inline void mfma_lds_layout(MfmaParams* mp, int d, int n_tasks, int n_groups, int waves)
{
    const int blocks_local = (mp->n_blocks + mp->q_split - 1) / mp->q_split;
    mp->rows_local = blocks_local * 16;
    int off = 0;
    auto take = [&](int bytes) { int o = off; off = (off + bytes + 15) / 16 * 16; return o; };
    take(mp->rows_local * d);  // resident queries at offset 0
    mp->lds_sq = take(mp->rows_local * 4);
    mp->lds_tauf = take(mp->rows_local * 4);
    mp->lds_tau64 = take((mp->rows_local / n_tasks + 1) * 8);
    mp->lds_qrow = take(mp->rows_local * 4);
    mp->lds_cnt = take((mp->region_slots * (mp->rows_local / n_tasks + 1) + 1) * 4);  // + the segment counter
    mp->lds_list = take(waves * kMfmaFilterBatch * mp->seg_stride);
    mp->lds_queue = take(waves * mfma_queue_bytes(d, waves));
    mp->lds_prow = take(n_groups * kPrefetchStride * 4);
    mp->lds_blkoff = take((2 * n_groups + 2) * 4);
    mp->lds_rowoff = take((n_groups + 1) * 4);
    mp->lds_tq = take(mp->rows_local * 4);
    mp->lds_thr = take(waves * mp->rows_local * 4);
    mp->lds_scl = take(waves * mp->seg_stride * 4);
    mp->lds_total = off;
}

inline int mfma_lds_bytes(int n_blocks, int S, int d, int n_tasks, int n_groups, int waves, int slots, int seg_stride)
{
    MfmaParams t;
    t.n_blocks = n_blocks;
    t.q_split = S;
    t.region_slots = slots;
    t.seg_stride = seg_stride;
    mfma_lds_layout(&t, d, n_tasks, n_groups, waves);
    return t.lds_total;
}

template <int KS, int TT, bool WEIGHTED, bool MULTI, int NW, bool ADMIT = false>
inline hipError_t launch_scan_mfma_t(const ScanParams& sp, const MfmaParams& mp, int gx, hipStream_t stream)
{
    static std::atomic<int> max_set{0};  // largest dynamic LDS size this instantiation has been allowed
    if (mp.lds_total > max_set.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&scan_mfma_kernel<KS, TT, WEIGHTED, MULTI, NW, ADMIT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, mp.lds_total);
        if (e != hipSuccess) return e;
        max_set.store(mp.lds_total, std::memory_order_release);
    }
    const dim3 grid((unsigned)gx, (unsigned)mp.q_split);
    hipLaunchKernelGGL((scan_mfma_kernel<KS, TT, WEIGHTED, MULTI, NW, ADMIT>), grid, dim3(NW * 64), (size_t)mp.lds_total, stream, sp, mp);
    return hipGetLastError();
}

// The instantiations are compiled in one translation unit per embedding width (st_mfma_ks*.hip),
// so that the library builds in parallel; each defines its launcher through this template.
// gx = workgroups per row of the grid (at most groups / q_split); region index = x + y * gx
template <int KS>
inline hipError_t launch_scan_mfma_ks(const ScanParams& sp, const MfmaParams& mp, int gx, hipStream_t stream)
{
    const int tt = sp.n_tasks;
    // first level, one segment per region: every pair is a candidate and is stored directly
    const bool admit = !sp.use_tau && sp.seg_per_visit == 1 && sp.seg_items <= sp.cap;
// plain search has one task per query (several tasks always come with weights)
#define ST_ARM(T_, W_, M_, N_, A_)                                                                               \
    ((W_ || T_ == 1) ? launch_scan_mfma_t<KS, (W_ || T_ == 1) ? T_ : 1, W_, M_, N_, A_>(sp, mp, gx, stream)       \
                     : hipErrorInvalidValue)
#define ST_CASE(T_)                                                                                              \
    if (tt == T_) {                                                                                              \
        if (mp.waves == 8 && admit)                                                                              \
            return sp.weighted ? ST_ARM(T_, true, true, 8, true) : ST_ARM(T_, false, true, 8, true);             \
        if (mp.waves == 8)                                                                                       \
            return sp.weighted ? ST_ARM(T_, true, true, 8, false) : ST_ARM(T_, false, true, 8, false);           \
        if (mp.multi_block || mp.region_slots != 1 || mp.seg_stride != 256)                                      \
            return sp.weighted ? ST_ARM(T_, true, true, 4, false) : ST_ARM(T_, false, true, 4, false);           \
        return sp.weighted ? ST_ARM(T_, true, false, 4, false) : ST_ARM(T_, false, false, 4, false);             \
    }
    ST_CASE(1) ST_CASE(2) ST_CASE(4)
#undef ST_ARM
#undef ST_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_scan_mfma_ks1(const ScanParams& sp, const MfmaParams& mp, int gx, hipStream_t stream);
hipError_t launch_scan_mfma_ks2(const ScanParams& sp, const MfmaParams& mp, int gx, hipStream_t stream);
hipError_t launch_scan_mfma_ks4(const ScanParams& sp, const MfmaParams& mp, int gx, hipStream_t stream);
hipError_t launch_scan_mfma_ks8(const ScanParams& sp, const MfmaParams& mp, int gx, hipStream_t stream);

inline hipError_t launch_scan_mfma(const ScanParams& sp, const MfmaParams& mp, int gx, hipStream_t stream)
{
    if (sp.seg_items > mp.seg_stride || mp.seg_stride > kMfmaSegItems || sp.n_groups > kMfmaMaxGroups) return hipErrorInvalidValue;
    switch (sp.d) {
        case 64: return launch_scan_mfma_ks1(sp, mp, gx, stream);
        case 128: return launch_scan_mfma_ks2(sp, mp, gx, stream);
        case 256: return launch_scan_mfma_ks4(sp, mp, gx, stream);
        case 512: return launch_scan_mfma_ks8(sp, mp, gx, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace st
