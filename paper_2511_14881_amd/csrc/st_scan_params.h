// Parameters shared by the scan kernels (wavefront dot product, int8 MFMA), the seed pass and
// the selection kernel.
#pragma once
#include <stdint.h>

namespace st {

constexpr int kTauParts = 8;  // thresholds per query (the seed pass leaves one per slice; readers take the minimum)

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
    const uint64_t* tau;         // [B][kTauParts]
    int32_t tau_parts;           // entries of tau in use per query
    // Sample mode (samp_role != 0): the first level does not scan a prefix of the corpus but
    // samp_segs segments of samp_seg_items items spread evenly over it, segment s starting at item
    // s * samp_stride_items -- what its selection learns about a query's scores then does not
    // depend on trends along the item order.  Role 1: this launch scans the sample; role 2: it
    // scans [item_begin, item_end) and leaves the sample's words out.
    int64_t samp_stride_items;
    int32_t samp_segs, samp_seg_items, samp_role;
    // output regions
    uint64_t* cand;              // [B][G][cap]
    uint32_t* cnt;               // [B][G]
    uint32_t* ovf;               // [B]
    int32_t cap;
    int32_t groups;              // G (== gridDim.x)
};

}  // namespace st
