// Routes a scan launch to the translation unit that holds the product's kernels.
#include "spd_kernels.h"

namespace spd {
hipError_t launch_scan_dot(hipStream_t, int, int, uint32_t, const ScanArgs &);
hipError_t launch_scan_dot_knn(hipStream_t, int, int, uint32_t, const ScanArgs &);
hipError_t launch_scan_cnt(hipStream_t, int, int, uint32_t, const ScanArgs &);
hipError_t launch_scan_cnt_knn(hipStream_t, int, int, uint32_t, const ScanArgs &);
hipError_t launch_scan_l1(hipStream_t, int, int, uint32_t, const ScanArgs &);
hipError_t launch_scan_mink(hipStream_t, int, int, uint32_t, const ScanArgs &);
hipError_t launch_scan_mink_any(hipStream_t, int, int, uint32_t, const ScanArgs &);
hipError_t launch_scan_canb(hipStream_t, int, int, uint32_t, const ScanArgs &);
hipError_t launch_scan_hamm(hipStream_t, int, int, uint32_t, const ScanArgs &);
hipError_t launch_scan_kl(hipStream_t, int, int, uint32_t, const ScanArgs &);
hipError_t launch_scan_js(hipStream_t, int, int, uint32_t, const ScanArgs &);
hipError_t launch_scan_cheb(hipStream_t, int, int, uint32_t, const ScanArgs &);
hipError_t launch_scan_semi_sum(hipStream_t, int, int, uint32_t, const ScanArgs &);
hipError_t launch_scan_semi_sum_knn(hipStream_t, int, int, uint32_t, const ScanArgs &);
hipError_t launch_scan_semi_ext(hipStream_t, int, int, uint32_t, const ScanArgs &);
hipError_t launch_scan_semi_ext_knn(hipStream_t, int, int, uint32_t, const ScanArgs &);

hipError_t launch_scan(hipStream_t st, int op, int R, int block, uint32_t lds_bytes, const ScanArgs &args) {
    switch (op) {
    case OP_DOT:
        return args.knn_k > 0 ? launch_scan_dot_knn(st, R, block, lds_bytes, args)
                              : launch_scan_dot(st, R, block, lds_bytes, args);
    case OP_CNT:
        return args.knn_k > 0 ? launch_scan_cnt_knn(st, R, block, lds_bytes, args)
                              : launch_scan_cnt(st, R, block, lds_bytes, args);
    case OP_L1: return launch_scan_l1(st, R, block, lds_bytes, args);
    case OP_MINK:       // (its kernels hold the degrees 1 to 4 only)
        return degree_class(args.q.p) == 0 ? hipErrorInvalidValue : launch_scan_mink(st, R, block, lds_bytes, args);
    case OP_MINK_ANY: return launch_scan_mink_any(st, R, block, lds_bytes, args);
    case OP_CANB: return launch_scan_canb(st, R, block, lds_bytes, args);
    case OP_HAMM: return launch_scan_hamm(st, R, block, lds_bytes, args);
    case OP_KL: return launch_scan_kl(st, R, block, lds_bytes, args);
    case OP_JS: return launch_scan_js(st, R, block, lds_bytes, args);
    case OP_CHEB: return launch_scan_cheb(st, R, block, lds_bytes, args);
    case OP_SEMI_SUM:
        return args.knn_k > 0 ? launch_scan_semi_sum_knn(st, R, block, lds_bytes, args)
                              : launch_scan_semi_sum(st, R, block, lds_bytes, args);
    case OP_SEMI_EXT:
        return args.knn_k > 0 ? launch_scan_semi_ext_knn(st, R, block, lds_bytes, args)
                              : launch_scan_semi_ext(st, R, block, lds_bytes, args);
    default: return hipErrorInvalidValue;
    }
}
}  // namespace spd
