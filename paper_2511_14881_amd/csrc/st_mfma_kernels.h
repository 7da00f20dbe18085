// int8 MFMA scorer for filter groups with enough query rows to make scoring a dense contraction.
#pragma once
#include "st_search_kernels.h"

namespace st {

struct MfmaChoice {
    bool use;
};

inline MfmaChoice choose_mfma(int path, int d, int n_tasks, bool weighted, int batch, int n_groups)
{
    (void)path; (void)d; (void)n_tasks; (void)weighted; (void)batch; (void)n_groups;
    return MfmaChoice{false};
}

inline void launch_scan_mfma(const ScanParams&, const MfmaChoice&, hipStream_t) {}

}  // namespace st
