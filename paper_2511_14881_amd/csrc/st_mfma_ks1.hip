// Instantiations of the int8 MFMA scan for d = 64 (1 contraction steps of 64 bytes per row).
#include "st_mfma2_kernels.h"

namespace st {

hipError_t launch_scan_mfma_ks1(const ScanParams& sp, const MfmaParams& mp, int gx, hipStream_t stream)
{
    if (scan_mfma2_applies(sp, mp)) return launch_scan_mfma2_ks<1>(sp, mp, gx, stream);
    return launch_scan_mfma_ks<1>(sp, mp, gx, stream);
}

}  // namespace st
