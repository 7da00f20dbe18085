// Scan with the int8 MFMA scorer (v_mfma_i32_16x16x64_i8), for filter groups that carry enough
// query rows to make scoring a dense contraction (Sec. 4.2: item rows are streamed from the
// embedding table and multiplied with the batched queries on the fly, nothing is gathered into
// a temporary).  Queries stay resident in LDS for the whole launch; the passing items of a
// segment, compacted per filter group, are loaded straight from HBM into the B operand.
//
// Contraction layout per MFMA (M = 16 query rows, N = 16 items, K = 64 bytes of the embedding):
//   A (queries): lane l supplies row (l % 16), bytes [16*(l/16), +16) of the 64-byte k-step
//   B (items)  : lane l supplies item (l % 16), the same byte range
//   D          : lane l receives D[4*(l/16) + r][l % 16], r = 0..3  -> one item, four query rows
// so with T in {1, 2, 4} tasks the rows one lane holds are whole queries and the Value-Model
// sum needs no cross-lane traffic.
#pragma once
#include "st_search_kernels.h"

namespace st {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kMfmaFilterBatch = 8;        // distinct filters handled per pass over a segment
constexpr int kMfmaQueryLds = 64 * 1024;   // LDS bytes for resident query rows per workgroup
constexpr int kMfmaMinRows = 4;            // a group needs this many query rows to go to MFMA

struct MfmaParams {
    const int32_t* grp_blk_off;  // [F+1] first 16-row block of each group
    const int32_t* blk_row;      // [n_blocks*16] global query row (q*T + t) or -1 for padding
    int32_t n_blocks;            // all groups
    int32_t q_split;             // S: gridDim.y; block b belongs to y = b % S, local index b / S
    int32_t rows_local;          // 16 * blocks per y (max over y)
    // dynamic LDS layout (byte offsets)
    int32_t lds_sq, lds_tauf, lds_qrow, lds_cnt, lds_mask, lds_list, lds_listcnt, lds_total;
};

// chunk swizzle for the resident query rows: keeps the 16 rows of a block on distinct banks
// when the 16 lanes of a quarter-wave read the same 16-byte chunk of 16 consecutive rows
template <int KS>
__device__ inline int swz(int row)
{
    constexpr int nch = KS * 4;                       // 16-byte chunks per row
    constexpr int sh = nch >= 16 ? 0 : (nch == 8 ? 1 : 2);
    return (row >> sh) & ((nch < 16 ? nch : 16) - 1);
}

template <int KS, int TT>
__global__ __launch_bounds__(kScanThreads) void scan_mfma_kernel(ScanParams p, MfmaParams mp)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int D = KS * 64;
    int8_t* s_q = reinterpret_cast<int8_t*>(lds);
    float* s_sq = reinterpret_cast<float*>(lds + mp.lds_sq);
    float* s_tauf = reinterpret_cast<float*>(lds + mp.lds_tauf);
    int* s_qrow = reinterpret_cast<int*>(lds + mp.lds_qrow);
    uint32_t* s_cnt = reinterpret_cast<uint32_t*>(lds + mp.lds_cnt);
    uint64_t* s_mask = reinterpret_cast<uint64_t*>(lds + mp.lds_mask);      // [FB][16]
    uint16_t* s_list = reinterpret_cast<uint16_t*>(lds + mp.lds_list);      // [FB][seg_items]
    int* s_listcnt = reinterpret_cast<int*>(lds + mp.lds_listcnt);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int S = mp.q_split, y = blockIdx.y;
    const int wg_lin = blockIdx.x + y * gridDim.x;  // region index in [0, groups)
    const int l16 = lane & 15, kg = lane >> 4;

    // ---- resident state: this y's query rows (swizzled), their scales, thresholds, owners
    for (int lr = tid; lr < mp.rows_local; lr += kScanThreads) {
        const int b = (lr >> 4) * S + y;
        const int grow = b < mp.n_blocks ? mp.blk_row[b * 16 + (lr & 15)] : -1;
        s_qrow[lr] = grow;
        float sq = 0.0f, tf = __builtin_inff();
        if (grow >= 0) {
            sq = p.qscale[grow];
            const uint64_t t64 = p.use_tau ? p.tau[grow / TT] : 0ULL;
            tf = t64 ? key_score(t64) : -__builtin_inff();
        }
        s_sq[lr] = sq;
        s_tauf[lr] = tf;
        if ((lr % TT) == 0) s_cnt[lr / TT] = 0;
    }
    for (int i = tid; i < mp.rows_local * (D / 16); i += kScanThreads) {
        const int lr = i / (D / 16), c = i - lr * (D / 16);
        const int b = (lr >> 4) * S + y;
        const int grow = b < mp.n_blocks ? mp.blk_row[b * 16 + (lr & 15)] : -1;
        int4 v = make_int4(0, 0, 0, 0);
        if (grow >= 0) v = reinterpret_cast<const int4*>(p.queries + (int64_t)grow * D)[c];
        *reinterpret_cast<int4*>(s_q + lr * D + ((c ^ swz<KS>(lr)) << 4)) = v;
    }
    __syncthreads();

    const int seg_words = p.seg_items >> 6;
    const int64_t n_seg = (p.item_end - p.item_begin + p.seg_items - 1) / p.seg_items;
    const int64_t item_lim = p.item_end < p.n_items ? p.item_end : p.n_items;
    for (int64_t seg = blockIdx.x; seg < n_seg; seg += gridDim.x) {
        const int64_t item0 = p.item_begin + seg * p.seg_items;
        const int64_t word0 = item0 >> 6;
        for (int g0 = 0; g0 < p.n_groups; g0 += kMfmaFilterBatch) {
            const int nf = min(kMfmaFilterBatch, p.n_groups - g0);
            // (1) Bloom test
            for (int idx = tid; idx < nf * seg_words; idx += kScanThreads) {
                const int gi = idx / seg_words, w = idx - gi * seg_words;
                const int g = g0 + gi;
                const int r0 = p.grp_row_off[g], r1 = p.grp_row_off[g + 1];
                s_mask[gi * kTileWords + w] =
                    bloom_mask_word(p.bloom, p.m_bits, word0 + w, item_lim, p.grp_rows + r0, r1 - r0);
            }
            __syncthreads();
            // (2) compaction
            for (int gi = wave; gi < nf; gi += kScanThreads / 64) {
                uint64_t mask = lane < seg_words ? s_mask[gi * kTileWords + lane] : 0ULL;
                const int c = __popcll(mask);
                int incl = c;
                for (int o = 1; o < kTileWords; o <<= 1) {
                    const int v = __shfl_up(incl, o);
                    if (lane >= o) incl += v;
                }
                int pos = incl - c;
                uint16_t* list = s_list + gi * p.seg_items;
                while (mask) {
                    const int b = __ffsll((long long)mask) - 1;
                    mask &= mask - 1;
                    list[pos++] = (uint16_t)(lane * 64 + b);
                }
                const int total = __shfl(incl, kTileWords - 1);
                if (lane == 0) s_listcnt[gi] = total;
            }
            __syncthreads();
            // (3) contraction + epilogue: a wavefront takes 64 passing items (4 x 16) at a time
            for (int gi = 0; gi < nf; ++gi) {
                const int n = s_listcnt[gi];
                const int g = g0 + gi;
                const int blk_end = mp.grp_blk_off[g + 1];
                int blk_first = mp.grp_blk_off[g];
                blk_first += ((y - blk_first) % S + S) % S;  // first block of the group owned by this y
                if (blk_first >= blk_end) continue;
                const uint16_t* list = s_list + gi * p.seg_items;
                for (int b0 = ((wave + gi) & 3) * 64; b0 < n; b0 += kScanThreads) {
                    const int left = n - b0;
                    const int nsb = left >= 64 ? 4 : (left + 15) >> 4;
                    v4i breg[4][KS];
                    float si[4];
                    int64_t item[4];
                    bool valid[4];
#pragma unroll
                    for (int sb = 0; sb < 4; ++sb) {
                        if (sb < nsb) {
                            const int li = b0 + sb * 16 + l16;
                            valid[sb] = li < n;
                            item[sb] = item0 + (int)list[valid[sb] ? li : b0];
                            const int4* rp = reinterpret_cast<const int4*>(p.items + item[sb] * D) + kg;
#pragma unroll
                            for (int s = 0; s < KS; ++s) {
                                const int4 v = rp[4 * s];
                                breg[sb][s] = v4i{v.x, v.y, v.z, v.w};
                            }
                            si[sb] = p.iscale[item[sb]];
                        }
                    }
                    for (int blk = blk_first; blk < blk_end; blk += S) {
                        const int lrow = (blk / S) * 16;
                        v4i areg[KS];
                        {
                            const int r = lrow + l16;
                            const int8_t* qp = s_q + r * D;
                            const int sw = swz<KS>(r);
#pragma unroll
                            for (int s = 0; s < KS; ++s) {
                                const int4 v = *reinterpret_cast<const int4*>(qp + (((kg + 4 * s) ^ sw) << 4));
                                areg[s] = v4i{v.x, v.y, v.z, v.w};
                            }
                        }
                        const int row4 = lrow + 4 * kg;
                        const float4 sq4 = *reinterpret_cast<const float4*>(s_sq + row4);
                        const float4 tf4 = *reinterpret_cast<const float4*>(s_tauf + row4);
                        const float sqv[4] = {sq4.x, sq4.y, sq4.z, sq4.w};
                        const float tfv[4] = {tf4.x, tf4.y, tf4.z, tf4.w};
#pragma unroll
                        for (int sb = 0; sb < 4; ++sb) {
                            if (sb < nsb) {
                                v4i acc = {0, 0, 0, 0};
#pragma unroll
                                for (int s = 0; s < KS; ++s)
                                    acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(areg[s], breg[sb][s], acc, 0, 0, 0);
                                float sc[4];
#pragma unroll
                                for (int r = 0; r < 4; ++r) sc[r] = rescale(acc[r], sqv[r], si[sb]);
                                if (p.weighted) {
                                    // Value-Model sum over the TT tasks of each query this lane holds
#pragma unroll
                                    for (int q0 = 0; q0 < 4; q0 += TT) {
                                        float agg = 0.0f;
#pragma unroll
                                        for (int t = 0; t < TT; ++t) agg = __fmaf_rn(p.w[t], sc[q0 + t], agg);
                                        sc[q0] = agg;
                                    }
                                }
#pragma unroll
                                for (int r = 0; r < 4; r += TT) {
                                    if (sc[r] >= tfv[r]) {
                                        const int grow = s_qrow[row4 + r];
                                        if (valid[sb] && grow >= 0) {
                                            const int q = grow / TT;
                                            const uint64_t key = make_key(sc[r], (uint32_t)item[sb]);
                                            if (!p.use_tau || key >= p.tau[q]) {
                                                const uint32_t slot = atomicAdd(&s_cnt[(row4 + r) / TT], 1u);
                                                if (slot < (uint32_t)p.cap)
                                                    p.cand[((int64_t)q * p.groups + wg_lin) * p.cap + slot] = key;
                                            }
                                        }
                                    }
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
    // region fill counts: real ones for the queries this workgroup row owns, zero for the others
    for (int i = tid * TT; i < mp.n_blocks * 16; i += kScanThreads * TT) {
        const int grow = mp.blk_row[i];
        if (grow < 0) continue;
        const int q = grow / TT;
        const int b = i >> 4;
        uint32_t c = 0;
        if (b % S == y) c = s_cnt[((b / S) * 16 + (i & 15)) / TT];
        p.cnt[(int64_t)q * p.groups + wg_lin] = c < (uint32_t)p.cap ? c : (uint32_t)p.cap;
        if (c > (uint32_t)p.cap) p.ovf[q] = 1u;
    }
}

inline bool mfma_shape_ok(int d, int n_tasks)
{
    return (d == 64 || d == 128 || d == 256 || d == 512) && (n_tasks == 1 || n_tasks == 2 || n_tasks == 4);
}

// Smallest power of two S such that ceil(n_blocks / S) blocks of 16 rows of d bytes fit the LDS budget.
inline int mfma_q_split(int n_blocks, int d)
{
    int S = 1;
    while (((n_blocks + S - 1) / S) * 16 * d > kMfmaQueryLds) S <<= 1;
    return S;
}

inline void mfma_lds_layout(MfmaParams* mp, int d, int n_tasks, int seg_items)
{
    const int blocks_local = (mp->n_blocks + mp->q_split - 1) / mp->q_split;
    mp->rows_local = blocks_local * 16;
    int off = mp->rows_local * d;
    auto take = [&](int bytes) { int o = off; off = (off + bytes + 15) / 16 * 16; return o; };
    take(0);
    mp->lds_sq = take(mp->rows_local * 4);
    mp->lds_tauf = take(mp->rows_local * 4);
    mp->lds_qrow = take(mp->rows_local * 4);
    mp->lds_cnt = take((mp->rows_local / n_tasks + 1) * 4);
    mp->lds_mask = take(kMfmaFilterBatch * kTileWords * 8);
    mp->lds_list = take(kMfmaFilterBatch * seg_items * 2);
    mp->lds_listcnt = take(kMfmaFilterBatch * 4);
    mp->lds_total = off;
}

template <int KS, int TT>
inline hipError_t launch_scan_mfma_t(const ScanParams& sp, const MfmaParams& mp, hipStream_t stream)
{
    static int max_set = 0;  // largest dynamic LDS size this instantiation has been allowed
    if (mp.lds_total > max_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&scan_mfma_kernel<KS, TT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, mp.lds_total);
        if (e != hipSuccess) return e;
        max_set = mp.lds_total;
    }
    const dim3 grid((unsigned)(sp.groups / mp.q_split), (unsigned)mp.q_split);
    hipLaunchKernelGGL((scan_mfma_kernel<KS, TT>), grid, dim3(kScanThreads), (size_t)mp.lds_total, stream, sp, mp);
    return hipGetLastError();
}

inline hipError_t launch_scan_mfma(const ScanParams& sp, const MfmaParams& mp, hipStream_t stream)
{
    const int ks = sp.d / 64, tt = sp.n_tasks;
#define ST_CASE(K_, T_) \
    if (ks == K_ && tt == T_) return launch_scan_mfma_t<K_, T_>(sp, mp, stream);
    ST_CASE(1, 1) ST_CASE(1, 2) ST_CASE(1, 4)
    ST_CASE(2, 1) ST_CASE(2, 2) ST_CASE(2, 4)
    ST_CASE(4, 1) ST_CASE(4, 2) ST_CASE(4, 4)
    ST_CASE(8, 1) ST_CASE(8, 2) ST_CASE(8, 4)
#undef ST_CASE
    return hipErrorInvalidValue;
}

}  // namespace st
