// Staged-scan kernel instances for one product (see spd_scan_impl.h).
#include "spd_scan_impl.h"

namespace spd {
hipError_t launch_scan_mink_any(hipStream_t st, int R, int block, uint32_t lds_bytes, const ScanArgs &args) {
    return launch_scan_op<OP_MINK_ANY>(st, R, block, lds_bytes, args);
}
}  // namespace spd
