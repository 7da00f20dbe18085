// Second form of the int8 MFMA scan, for the levels that admit by threshold with 8-wavefront
// workgroups (d <= 256): the same Bloom test, compaction and contraction as scan_mfma_kernel
// (Sec. 4.1 Eq. 4, Sec. 4.2, Algorithm 1 phase 3), with three changes that remove work per item:
//
//   * Passing items are contracted in full 16-item units only.  What a filter's list holds beyond
//     a multiple of 16 is carried, as absolute item numbers, to the wavefront's next segment, and
//     flushed as one partial unit when the wavefront runs out of segments.  At 0.1 % selectivity a
//     filter passes an item every other segment; without the carry each of them would cost a
//     whole unit of its own.
//   * The admission bound is one 24-bit multiply-add per (query row, item) pair and one compare
//     per four pairs: t = dot * F + NEG with F = ceil(s_i * 2^(P-E)) (a small integer: the item's
//     scale against a power of two 2^E above the scales seen so far) and NEG = -floor(tau / s_q *
//     2^(P-E) * (1 - 2^-18)) per row.  A pair can only be admitted if t >= 0; the exact fp32
//     score, key and threshold test run for those pairs alone.  |dot| <= 2^(14 + log2 d) and
//     F <= 2^P with P = 16 - log2 d keep dot * F within 2^30.
//   * An item's scale is loaded with its row (one 4-byte load per lane and unit), so nothing is
//     staged or reduced per segment.
#pragma once
#include "st_mfma_kernels.h"

namespace st {

constexpr int kCarry = 16;  // entries per filter a wavefront can carry to its next segment

template <int KS, int TT, bool WEIGHTED>
__device__ __forceinline__ void scan_mfma2_body(const ScanParams& p, const MfmaParams& mp)
{
    static_assert(KS == 1 || KS == 2 || KS == 4, "dot products must fit 23 bits for the 24-bit multiply");
    constexpr int NW = 8;
    constexpr int kThreads = NW * 64;
    constexpr int PR = kPrefetchStride;
    constexpr int D = KS * 64;
    constexpr int CH = D / 16;
    constexpr int FB = kMfmaFilterBatch;
    constexpr bool PAIRS = KS <= 2;
    constexpr int NB = PAIRS ? 4 : 2;
    constexpr int P = KS == 1 ? 10 : (KS == 2 ? 9 : 8);  // fixed-point bits of the item scale
    constexpr int kPass = (1 << 30) - 1;                 // NEG of a row without a bound: t >= 0 always (dot * F > -2^30)
    constexpr int kNever = -(1 << 30) - 1;               // NEG of a padding row: t < 0 always
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int seg_stride = mp.seg_stride;
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
    auto tq_of = [](float tf, float sq) -> float {  // tau / s_q; +inf: padding row, -inf: no bound
        const float inf = __builtin_inff();
        if (tf == inf) return inf;
        if (!(tf > 0.0f)) return -inf;
        const float tq = tf / sq;
        return (tq > 0.0f && tq < inf) ? tq : -inf;
    };
    // wave-private state
    uint8_t* s_list = reinterpret_cast<uint8_t*>(lds + mp.lds_list) + wave * FB * seg_stride;     // [FB][seg] this segment's passing items
    uint32_t* s_carry = reinterpret_cast<uint32_t*>(lds + mp.lds_scl) + wave * FB * kCarry;       // [FB][kCarry] absolute items carried over
    // queued lanes (one item x four query rows each) with a possible admission: the four
    // accumulators, and item scale << 32 | first local query row << 10 | item code (bit 9 clear:
    // place in the current segment; set: index into the carry area).  64 entries per wavefront.
    static_assert(kQueueSlots * 8 >= 64 * 16, "the accumulators of 64 queued lanes take the queue area");
    int4* q_acc = reinterpret_cast<int4*>(lds + mp.lds_queue + wave * mfma_queue_bytes(KS * 64, NW));
    uint64_t* q_meta = reinterpret_cast<uint64_t*>(lds + mp.lds_scl + NW * FB * kCarry * 4) + wave * 64;
    float* s_tq = reinterpret_cast<float*>(lds + mp.lds_tq);                                      // [rows_local] tau / s_q per row
    int* s_neg = reinterpret_cast<int*>(lds + mp.lds_thr) + wave * mp.rows_local;                 // [rows_local] NEG per row for the current E

    // ---- schedule: as in scan_mfma_kernel (visits dealt to workgroups, segments drawn by the
    // wavefronts from a counter in LDS)
    const int seg_items = p.seg_items;
    const int SW = seg_items >> 6;
    const int spv = p.seg_per_visit;
    const int64_t item_lim = p.item_end < p.n_items ? p.item_end : p.n_items;
    const int n_seg = (int)((p.item_end - p.item_begin + seg_items - 1) / seg_items);
    const int n_visit = (n_seg + spv - 1) / spv;
    const int n_batches = (p.n_groups + FB - 1) / FB;
    const int wg_visits = (int)blockIdx.x < n_visit ? (n_visit - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x : 0;
    const int wg_segs = wg_visits * spv;
    const int R = mp.region_slots;
    const int nq_pad = mp.rows_local / TT + 1;
    uint32_t* s_work = s_cnt + R * nq_pad;
    struct Stage {
        int num;
        int batch;
    };
    auto stage_ok = [&](const Stage& st) { return st.num < wg_segs; };
    auto stage_seg = [&](const Stage& st) {
        const int i = st.num / spv;
        return ((int)blockIdx.x + i * (int)gridDim.x) * spv + (st.num - i * spv);
    };
    auto seg_first = [&](const Stage& st) -> int64_t { return p.item_begin + (int64_t)stage_seg(st) * seg_items; };
    auto in_sample = [&](int64_t first) -> bool {  // the 64-item word at `first` belongs to the first level's sample
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
    int pre_valid = 0;
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
    auto prefetch_mask = [&](const Stage& st) -> uint64_t {
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
        if (nr > pre_valid) {
            const uint64_t* base = p.bloom + ((gw >> 4) * (int64_t)p.m_bits) * kTileWords + (gw & 15);
            for (int r = pre_valid; r < nr; ++r) mask &= base[(int64_t)p.grp_rows[r0 + r] * kTileWords];
        }
        return mask;
    };
    // first Bloom words: rows from the kernel arguments, requested before any table is read
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

    // ---- workgroup-wide set-up: tables and the resident-query image (written by an earlier
    // launch of the search) into LDS; all reads of a share are issued before anything is stored
    const int n_prow = p.n_groups * kPrefetchStride;
    const int n_piece = mp.rows_local * CH;
    const int n_imgrow = mp.rows_local;
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
            if (tid < p.n_groups) {
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
            s_tq[tid] = tq_of(tf, v_sq);
            if ((tid % TT) == 0) s_tau64[tid / TT] = v_tau;
        }
    }
    for (int i = tid; i < R * nq_pad; i += kThreads) s_cnt[i] = 0;
    if (tid == 0) *s_work = (uint32_t)NW;
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
        s_tq[lr] = tq_of(tf, sq);
        if ((lr % TT) == 0) s_tau64[lr / TT] = t64;
    }
    lds_barrier();

    int a_off[KS];
#pragma unroll
    for (int k = 0; k < KS; ++k) a_off[k] = l16 * D + (((kg + 4 * k) ^ swz<KS>(l16)) << 4);

    // scale exponent of the wavefront (plain search): every scale met so far is below 2^E
    int cur_E = -1000;
    float two_E = 0.0f;      // 2^E; 0 until the first unit sets it
    float fix_scale = 0.0f;  // 2^(P-E)
    auto set_exponent = [&](int E) {  // rebuilds the per-row NEG table for E (all lanes take part)
        cur_E = E;
        two_E = ldexpf(1.0f, E);
        fix_scale = ldexpf(1.0f, P - E);
        const float thr_scale = ldexpf(0.99999618530273f, P - E);  // (1 - 2^-18) * 2^(P-E)
        for (int row = lane; row < mp.rows_local; row += 64) {
            const float tq = s_tq[row];
            int neg = kPass;
            if (tq == __builtin_inff())
                neg = kNever;
            else if (tq > 0.0f)
                neg = -min(__float2int_rd(fminf(tq * thr_scale, 1.2e9f)), (1 << 30) + 1);  // bounds above 2^30 can never be met
            s_neg[row] = neg;
        }
    };
    if (WEIGHTED) {
        for (int row = lane; row < mp.rows_local; row += 64) s_neg[row] = 0;  // (not used)
    }

    int n_carry = 0;  // lane f < FB: entries of filter f in the carry area
    const bool can_carry = n_batches == 1;
    for (bool first = true; stage_ok(cur); first = false) {
        const int64_t item0 = seg_first(cur);
        const int g0 = cur.batch * FB;
        const int nf = min(FB, p.n_groups - g0);
        const int slot = R == 1 ? 0 : cur.num % R;
        const int region = (int)blockIdx.x + slot * (int)gridDim.x + y * (int)gridDim.x * R;
        uint32_t* cnt_s = s_cnt + slot * nq_pad;

        // (1) + (2): mask word of my (filter, word) pair, set bits into the filter's list
        pre_valid = PR;  // (the first stage's rows came from the kernel arguments, as many)
        uint64_t mask = prefetch_mask(cur);
        const Stage nxt = stage_next(cur);
#pragma unroll
        for (int r = 0; r < PR; ++r) pre[r] = ~0ULL;
        prefetch_issue(nxt);
        // the wavefront's last stage (or several filter batches per segment): partial units too
        const bool flush = !can_carry || !stage_ok(nxt);
        const int c = __popcll(mask);
        int incl = c;
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
        const int last_word = __shfl(incl, (lane * SW + SW - 1) & 63);
        const int low_words = __shfl(incl, (lane * SW + (SW > 4 ? 3 : SW - 1)) & 63);
        const int gcur = lane < nf ? last_word : 0;   // this segment's entries of filter `lane`
        const int glow = lane < nf ? low_words : 0;   // ... of its lower 256 items
        const int gnc = lane < nf ? n_carry : 0;      // carried entries in front of them
        const int gtot = gnc + gcur;
        const int gunits = flush ? (gtot + 15) >> 4 : gtot >> 4;
        int ucum = gunits;
        static_assert(FB == 8, "three steps cover the filters of a batch");
        { const int v = (int)row_shr<1>((uint32_t)ucum); if (lane >= 1) ucum += v; }
        { const int v = (int)row_shr<2>((uint32_t)ucum); if (lane >= 2) ucum += v; }
        { const int v = (int)row_shr<4>((uint32_t)ucum); if (lane >= 4) ucum += v; }
        const int n_units = __builtin_amdgcn_readlane(ucum, FB - 1);
        const int glrow = lane < nf ? s_glrow[g0 + lane] : 0;
        const int gnblk = lane < nf ? s_gnblk[g0 + lane] : 0;

        int qn = 0;          // queued candidates (uniform)
        int cur_lrow = -1;   // query block whose A operand (and per-row constants) sit in registers
        float4 cur_sq = make_float4(0.f, 0.f, 0.f, 0.f), cur_tf = cur_sq;
        int4 cur_neg = make_int4(0, 0, 0, 0);
        v4i areg[KS];

        // unit generator over the concatenation (carried entries, then this segment's) of each filter
        int gen_gi = 0, gen_b0 = 0, gen_tot = 0, gen_nc = 0, gen_low = 0, gen_units = 0, gen_left = 0;
        auto gen_fetch = [&]() {
            gen_tot = __builtin_amdgcn_readlane(gtot, gen_gi);
            gen_nc = __builtin_amdgcn_readlane(gnc, gen_gi);
            gen_low = __builtin_amdgcn_readlane(glow, gen_gi);
            gen_units = __builtin_amdgcn_readlane(gunits, gen_gi);
        };
        auto gen_seek0 = [&]() {  // position on unit 0 (n_units > 0)
            gen_gi = __popcll(ballot(lane < nf && ucum <= 0));
            gen_b0 = 0;
            gen_fetch();
            gen_left = n_units - 1;
        };
        // Entry `at` of the concatenation (carried entries, then this segment's) of filter f as an
        // absolute item number.  One 4-byte LDS read either way (a carried item number, or the
        // aligned word that holds the segment list's byte), so that no second read depends on the
        // first: the read sits in the chain between one unit's contraction and the next one's loads.
        auto entry_item = [&](int f, int at, int nc, int low) -> uint32_t {
            const int cj = at - nc;  // place in this segment's list (negative: a carried entry)
            const unsigned char* src = cj < 0 ? reinterpret_cast<const unsigned char*>(s_carry + f * kCarry + at)
                                              : s_list + f * seg_stride + (cj & ~3);
            const uint32_t v = *reinterpret_cast<const uint32_t*>(src);
            const uint32_t here = (uint32_t)item0 + ((v >> ((cj & 3) * 8)) & 255u) + (cj >= low ? 256u : 0u);
            return cj < 0 ? v : here;
        };
        auto unit_load = [&](UnitRegs<KS>& w) {
            const int li = gen_b0 + l16;
            const int at = min(li, gen_tot - 1);
            const uint32_t item = entry_item(gen_gi, at, gen_nc, gen_low);
            w.item = li < gen_tot ? (int)item : -1;
            // what a queued pair carries instead of the item number
            w.si_fix2 = at < gen_nc ? (512 | (gen_gi * kCarry + at)) : (int)(item - (uint32_t)item0);
            w.gi = gen_gi;
            // the scale first: loads complete in issue order, and the scale is what a unit's
            // contraction looks at first
            w.si = p.iscale[item];
            const char* rowp = reinterpret_cast<const char*>(p.items) + (uint64_t)item * D + kg * 16;
#pragma unroll
            for (int k = 0; k < KS; ++k) {
                const int4 v = *reinterpret_cast<const int4*>(rowp + 64 * k);
                w.b[k] = v4i{v.x, v.y, v.z, v.w};
            }
            w.si_fix = 0;
            if (gen_left > 0) {  // advance (scalar)
                --gen_left;
                gen_b0 += 16;
                if (gen_b0 >= gen_units * 16) {
                    do {
                        ++gen_gi;
                    } while (__builtin_amdgcn_readlane(gunits, gen_gi) == 0);
                    gen_b0 = 0;
                    gen_fetch();
                }
            }
        };
        // A lane whose block test leaves an admission possible is queued as it is -- its four
        // accumulators, its scale, where its rows and its item are -- and the queue is emptied 64
        // lanes at a time: exact fp32 scores, keys, comparison with each query's threshold key and
        // counter updates then run with every lane at work, for the four rows of a queued lane.
        // The store is issued in assembly so that the compiler keeps counting loads only when it
        // waits for a unit's rows (see scan_mfma_kernel).
        auto drain = [&]() {
            if (lane < qn) {
                const int4 a4 = q_acc[lane];
                const uint64_t e = q_meta[lane];
                const float si = __uint_as_float((uint32_t)(e >> 32));
                const int lrow4 = (int)((uint32_t)e >> 10);
                const uint32_t code = (uint32_t)e & 1023u;
                const uint32_t carried = s_carry[code & (FB * kCarry - 1)];
                const uint32_t item = (code & 512u) ? carried : (uint32_t)item0 + code;
                const float4 sq4 = *reinterpret_cast<const float4*>(s_sq + lrow4);
                const int4 qr4 = *reinterpret_cast<const int4*>(s_qrow + lrow4);
                const int accv[4] = {a4.x, a4.y, a4.z, a4.w};
                const float sqv[4] = {sq4.x, sq4.y, sq4.z, sq4.w};
                const int qrv[4] = {qr4.x, qr4.y, qr4.z, qr4.w};
                float sc[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) sc[r] = rescale(accv[r], sqv[r], si);
#pragma unroll
                for (int q0 = 0; q0 < 4; q0 += TT) {
                    float v = sc[q0];
                    if (WEIGHTED) {
                        v = 0.0f;
#pragma unroll
                        for (int tt = 0; tt < TT; ++tt) v = __fmaf_rn(p.w[tt], sc[q0 + tt], v);
                    }
                    const uint64_t key = make_key(v, item);
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
        // Queues the lanes m (uniform, non-zero) of the block that starts at local row lrow.
        auto block_push = [&](int lrow, const v4i& acc, const UnitRegs<KS>& w, uint64_t m) {
            const int n = __popcll(m);
            if (qn + n > 64) drain();
            if ((m >> lane) & 1ULL) {
                const int pos = qn + __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
                q_acc[pos] = make_int4(acc[0], acc[1], acc[2], acc[3]);
                q_meta[pos] = ((uint64_t)__float_as_uint(w.si) << 32) | (uint32_t)(((lrow + 4 * kg) << 10) | w.si_fix2);
            }
            qn += n;
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
        auto row_neg = [&](int lrow) { return *reinterpret_cast<const int4*>(s_neg + lrow + 4 * kg); };
        struct RowK {
            float4 sq, tf;  // weighted search
            int4 neg;       // plain search
        };
        auto row_k = [&](int lrow) -> RowK {
            RowK k;
            k.sq = k.tf = make_float4(0.f, 0.f, 0.f, 0.f);
            k.neg = make_int4(0, 0, 0, 0);
            if (WEIGHTED) {
                k.sq = row_sq(lrow);
                k.tf = row_tf(lrow);
            } else {
                k.neg = row_neg(lrow);
            }
            return k;
        };
        // Test of one block's accumulators (this lane: one item, four query rows): the lanes with a
        // possible admission.  `force` are lanes whose scale the bound does not cover.
        auto block_test = [&](const RowK& k, const v4i& acc, const UnitRegs<KS>& w, uint64_t valid, uint64_t force) -> uint64_t {
            if (WEIGHTED) {
                const float sqv[4] = {k.sq.x, k.sq.y, k.sq.z, k.sq.w};
                const float tfv[4] = {k.tf.x, k.tf.y, k.tf.z, k.tf.w};
                float sc[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) sc[r] = rescale(acc[r], sqv[r], w.si);
                bool hit = false;
#pragma unroll
                for (int q0 = 0; q0 < 4; q0 += TT) {
                    float agg = 0.0f;
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt) agg = __fmaf_rn(p.w[tt], sc[q0 + tt], agg);
                    hit = hit || agg >= tfv[q0];
                }
                return ballot(hit) & valid;
            }
            const int t0 = __mul24(acc[0], w.si_fix) + k.neg.x, t1 = __mul24(acc[1], w.si_fix) + k.neg.y;
            const int t2 = __mul24(acc[2], w.si_fix) + k.neg.z, t3 = __mul24(acc[3], w.si_fix) + k.neg.w;
            return (ballot(max(max(t0, t1), max(t2, t3)) >= 0) & valid) | force;
        };
        // Start of a unit's contraction: lanes that hold an item, the fixed-point factor of the
        // lane's scale, and the lanes the bound cannot be trusted for (a scale at or above 2^E, not
        // finite or not positive; every lane of the wavefront's first unit): `force`.  No branch
        // here, so that the operand reads that follow are issued before the wait for the rows.
        auto unit_begin = [&](UnitRegs<KS>& w, uint64_t& valid, uint64_t& force) {
            valid = ballot(w.item >= 0);
            force = 0;
            if (WEIGHTED) return;
            force = ballot((w.item >= 0) & !((w.si > 0.0f) & (w.si < two_E)));
            // (at least 1: the product of a tiny scale may round to zero, its ceiling does not)
            w.si_fix = max(__float2int_ru(fminf(w.si * fix_scale, (float)(1 << P))), 1);
        };
        // After a unit with forced lanes: raise the exponent over the largest usable scale met, so
        // that the units to come are covered.
        auto unit_end = [&](const UnitRegs<KS>& w, uint64_t force) {
            if (WEIGHTED || !force) return;
            float smax = (w.item >= 0 && w.si > 0.0f && w.si < __builtin_inff()) ? w.si : 0.0f;
            for (int o = 32; o > 0; o >>= 1) smax = fmaxf(smax, __shfl_xor(smax, o));
            if (smax > 0.0f) {
                const int E = ilogbf(smax) + 1;
                if (E > cur_E && E > -90 && E < 90) {
                    set_exponent(E);
                    cur_lrow = -1;  // the per-row constants in registers belong to the old exponent
                }
            }
        };
        auto unit_compute = [&](UnitRegs<KS>& w) {
            const int lrow0 = __builtin_amdgcn_readlane(glrow, w.gi);
            const int nblk = __builtin_amdgcn_readlane(gnblk, w.gi);
            uint64_t valid, force;
            unit_begin(w, valid, force);
            if (nblk == 1) {
                if (cur_lrow != lrow0) {
                    block_a(lrow0, areg);
                    if (WEIGHTED) {
                        cur_sq = row_sq(lrow0);
                        cur_tf = row_tf(lrow0);
                    } else {
                        cur_neg = row_neg(lrow0);
                    }
                    cur_lrow = lrow0;
                }
                const v4i acc = block_mfma(areg, w);
                RowK k;
                k.sq = cur_sq;
                k.tf = cur_tf;
                k.neg = cur_neg;
                { const uint64_t y = block_test(k, acc, w, valid, force); if (y) block_push(lrow0, acc, w, y); }
                unit_end(w, force);
                return;
            }
            int j = 0;
            if (KS <= 2) {  // four blocks per round: independent chains, where the registers allow it
                for (; j + 4 <= nblk; j += 4) {
                    const int l0 = lrow0 + 16 * j;
                    v4i a0[KS], a1[KS], a2[KS], a3[KS];
                    block_a(l0, a0);
                    block_a(l0 + 16, a1);
                    block_a(l0 + 32, a2);
                    block_a(l0 + 48, a3);
                    const RowK k0 = row_k(l0), k1 = row_k(l0 + 16), k2 = row_k(l0 + 32), k3 = row_k(l0 + 48);
                    const v4i c0 = block_mfma(a0, w), c1 = block_mfma(a1, w), c2 = block_mfma(a2, w), c3 = block_mfma(a3, w);
                    const uint64_t y0 = block_test(k0, c0, w, valid, force), y1 = block_test(k1, c1, w, valid, force);
                    const uint64_t y2 = block_test(k2, c2, w, valid, force), y3 = block_test(k3, c3, w, valid, force);
                    if (y0) block_push(l0, c0, w, y0);
                    if (y1) block_push(l0 + 16, c1, w, y1);
                    if (y2) block_push(l0 + 32, c2, w, y2);
                    if (y3) block_push(l0 + 48, c3, w, y3);
                }
            }
            for (; j + 2 <= nblk; j += 2) {
                const int l0 = lrow0 + 16 * j;
                v4i a0[KS], a1[KS];
                block_a(l0, a0);
                block_a(l0 + 16, a1);
                const RowK k0 = row_k(l0), k1 = row_k(l0 + 16);
                const v4i c0 = block_mfma(a0, w), c1 = block_mfma(a1, w);
                const uint64_t y0 = block_test(k0, c0, w, valid, force), y1 = block_test(k1, c1, w, valid, force);
                if (y0) block_push(l0, c0, w, y0);
                if (y1) block_push(l0 + 16, c1, w, y1);
            }
            for (; j < nblk; ++j) {
                v4i a[KS];
                block_a(lrow0 + 16 * j, a);
                const RowK k = row_k(lrow0 + 16 * j);
                const v4i acc = block_mfma(a, w);
                { const uint64_t y = block_test(k, acc, w, valid, force); if (y) block_push(lrow0 + 16 * j, acc, w, y); }
            }
            unit_end(w, force);
        };
        // Two units of one filter group at once: every block's operands serve both.
        auto unit_compute2 = [&](UnitRegs<KS>& w0, UnitRegs<KS>& w1) {
            const int lrow0 = __builtin_amdgcn_readlane(glrow, w0.gi);
            const int nblk = __builtin_amdgcn_readlane(gnblk, w0.gi);
            uint64_t valid0, force0, valid1, force1;
            unit_begin(w0, valid0, force0);
            unit_begin(w1, valid1, force1);
            int j = 0;
            for (; j + 2 <= nblk; j += 2) {
                const int l0 = lrow0 + 16 * j;
                v4i a0[KS], a1[KS];
                block_a(l0, a0);
                block_a(l0 + 16, a1);
                const RowK k0 = row_k(l0), k1 = row_k(l0 + 16);
                const v4i c00 = block_mfma(a0, w0), c01 = block_mfma(a0, w1), c10 = block_mfma(a1, w0), c11 = block_mfma(a1, w1);
                const uint64_t y00 = block_test(k0, c00, w0, valid0, force0), y01 = block_test(k0, c01, w1, valid1, force1);
                const uint64_t y10 = block_test(k1, c10, w0, valid0, force0), y11 = block_test(k1, c11, w1, valid1, force1);
                if (y00) block_push(l0, c00, w0, y00);
                if (y01) block_push(l0, c01, w1, y01);
                if (y10) block_push(l0 + 16, c10, w0, y10);
                if (y11) block_push(l0 + 16, c11, w1, y11);
            }
            for (; j < nblk; ++j) {
                const int l0 = lrow0 + 16 * j;
                v4i a[KS];
                block_a(l0, a);
                const RowK k = row_k(l0);
                const v4i c0 = block_mfma(a, w0), c1 = block_mfma(a, w1);
                const uint64_t y0 = block_test(k, c0, w0, valid0, force0), y1 = block_test(k, c1, w1, valid1, force1);
                if (y0) block_push(l0, c0, w0, y0);
                if (y1) block_push(l0, c1, w1, y1);
            }
            unit_end(w0, force0);
            unit_end(w1, force1);
        };
        if (n_units > 0) {
            UnitRegs<KS> r0, r1, r2, r3;
            auto step = [&](UnitRegs<KS>& r, int u) {
                if (u < n_units) unit_compute(r);
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
            gen_seek0();
            unit_load(r0);
            unit_load(r1);
            if (NB > 2) unit_load(r2);
            if (NB > 3) unit_load(r3);
            for (int base = 0; base < n_units; base += NB) {
                if (PAIRS) {
                    step2(r0, r1, base);
                    step2(r2, r3, base + 2);
                } else {
                    step(r0, base);
                    step(r1, base + 1);
                    if (NB > 2) step(r2, base + 2);
                    if (NB > 3) step(r3, base + 3);
                }
            }
            if (qn > 0) drain();
        }
        // (4) what the full units left over goes to the carry area: entry j of filter f, for the
        // (f, j) pairs of two passes over the wavefront.  All sources are read before anything is
        // written (a filter that contracted nothing keeps its carried entries in place).
        if (!flush) {
            uint32_t moved[2];
            bool live[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int f = (lane >> 4) + 4 * h, j = lane & 15;
                const int tot_f = __shfl(gtot, f), nc_f = __shfl(gnc, f), low_f = __shfl(glow, f), un_f = __shfl(gunits, f);
                const int idx = un_f * 16 + j;
                live[h] = f < nf && idx < tot_f;
                // (a dead lane reads entry 0 of a filter that may hold nothing: any word of the
                // filter's areas will do, the value is not used)
                const int at = live[h] ? idx : nc_f;
                moved[h] = entry_item(f < FB ? f : 0, at, nc_f, low_f);
            }
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int f = (lane >> 4) + 4 * h, j = lane & 15;
                if (live[h]) s_carry[f * kCarry + j] = moved[h];
            }
            n_carry = gtot - gunits * 16;  // lane f: < 16
        } else {
            n_carry = 0;
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

// Few passing items per filter and segment: units would be mostly padding, the carrying form
// wins; many: the first form's cheaper unit set-up wins (the cross-over lies near a dozen items
// per filter and 512-item segment).  The count comes from the first level of the same search.
template <int KS, int TT, bool WEIGHTED>
__global__ __launch_bounds__(512, 2) void scan_mfma2_kernel(ScanParams p, MfmaParams mp)
{
    const bool sparse = mp.density_acc != nullptr && *mp.density_acc < mp.density_limit;
    if (sparse)
        scan_mfma2_body<KS, TT, WEIGHTED>(p, mp);
    else
        scan_mfma_body<KS, TT, WEIGHTED, true, 8, false>(p, mp);
}

template <int KS, int TT, bool WEIGHTED>
inline hipError_t launch_scan_mfma2_t(const ScanParams& sp, const MfmaParams& mp, int gx, hipStream_t stream)
{
    static std::atomic<int> max_set{0};
    if (mp.lds_total > max_set.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&scan_mfma2_kernel<KS, TT, WEIGHTED>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, mp.lds_total);
        if (e != hipSuccess) return e;
        max_set.store(mp.lds_total, std::memory_order_release);
    }
    const dim3 grid((unsigned)gx, (unsigned)mp.q_split);
    hipLaunchKernelGGL((scan_mfma2_kernel<KS, TT, WEIGHTED>), grid, dim3(512), (size_t)mp.lds_total, stream, sp, mp);
    return hipGetLastError();
}

// Whether a launch with these parameters is served by the second form.
inline bool scan_mfma2_applies(const ScanParams& sp, const MfmaParams& mp)
{
    const bool admit = !sp.use_tau && sp.seg_per_visit == 1 && sp.seg_items <= sp.cap;
    return mp.waves == 8 && !admit && !mp.first_level && sp.use_tau && sp.d <= 256;
}

template <int KS>
inline hipError_t launch_scan_mfma2_ks(const ScanParams& sp, const MfmaParams& mp, int gx, hipStream_t stream)
{
    if (sp.weighted) {
        switch (sp.n_tasks) {
            case 1: return launch_scan_mfma2_t<KS, 1, true>(sp, mp, gx, stream);
            case 2: return launch_scan_mfma2_t<KS, 2, true>(sp, mp, gx, stream);
            case 4: return launch_scan_mfma2_t<KS, 4, true>(sp, mp, gx, stream);
            default: return hipErrorInvalidValue;
        }
    }
    return sp.n_tasks == 1 ? launch_scan_mfma2_t<KS, 1, false>(sp, mp, gx, stream) : hipErrorInvalidValue;
}

}  // namespace st
