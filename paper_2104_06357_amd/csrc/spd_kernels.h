// Launch interface between the host API and the HIP kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "spd_plan.h"

namespace spd {

struct KnnEntry { float d; int32_t j; };

// Device-resident copy of a BPlan plus the repacked entries and the row norms of B.
struct BDevice {
    const uint2 *packed;          // entries {column, value bits}: slab_base[s] + t*64 + lane
    const int64_t *slab_base;     // n_slabs + 1
    const int32_t *slab_steps;    // n_slabs
    const uint8_t *slab_split;    // n_slabs, largest seg_glog of the slab
    const int64_t *seg_start;     // lanes
    const int32_t *seg_len;       // lanes
    const int32_t *seg_row;       // lanes
    const uint8_t *seg_glog;      // lanes
    const double *norms;          // n_rows * 2, derived norms
    int32_t n_slabs;
    int64_t n_rows;
};

struct ScanArgs {
    // A
    const int32_t *a_indices;
    const float *a_values;
    const ARow *arows;            // n_groups * R
    const int32_t *sumlen;        // n_groups
    int32_t n_groups;
    const int32_t *chunk_begin;   // n_chunks + 1 slab indices: how this launch cuts B
    int32_t n_chunks;
    // B (original CSR, for the Chebyshev completion of fully covered rows)
    const int64_t *b_indptr;
    const int32_t *b_indices;
    BDevice b;
    // what to compute
    OpParams q;
    int32_t kind, transform, norm;
    int32_t hscale;               // hash staging: log2 of table entries per staged entry
    int32_t cuckoo_attempts;      // hash staging, half-full tables: pairs of hash functions tried (0: linear probing at once)
    int32_t knn_seed;             // fused top-k: 1 = the wavefronts' first slabs set a bar before any candidate is queued
    uint32_t k;                   // columns
    uint32_t padcol;              // column an idle lane looks up (maps to the zero row)
    // results
    float *out;                   // pairwise: the result of (staged row i, streamed row j) goes to
    int64_t out_stride_staged;    //   out[i * out_stride_staged + j * out_stride_streamed]: (n, 1) when A is
    int64_t out_stride_streamed;  //   staged and B streamed, (1, n) when the library has exchanged their roles
    double *partial;              // slices of spilled rows: [slot][plane][n]
    double *partial_norms;        // [slot][2] raw sums
    int32_t planes;               // 1, or 2 for Jensen-Shannon
    int32_t knn_k;                // 0: pairwise
    KnnEntry *knn_part;           // k-NN: candidate lists, knn_row_off[row] + chunk * k + t
    const int64_t *knn_row_off;   // per output row
};

struct FinalizeArgs {
    const SpilledRow *spilled;
    int32_t n_spilled;
    const double *partial;
    const double *partial_norms;
    const double *norms_b;
    int32_t planes;
    int64_t n_b;
    OpParams q;
    float *out;                   // pairwise: as in ScanArgs
    int64_t out_stride_staged, out_stride_streamed;
    int32_t knn_k;
    KnnEntry *knn_part;           // k-NN: a spilled row's candidate lists, one per tile of kFinalizeTile columns,
    const int64_t *knn_row_off;   //       at knn_row_off[row] + tile * k (merged with the others afterwards)
};

constexpr int kFinalizeTile = 8192;     // columns of B one workgroup of the k-NN finalize kernel walks

hipError_t launch_pack_b(hipStream_t st, const int64_t *b_indptr, const int32_t *b_indices, const float *b_values,
                         const BDevice &b, uint2 *packed_out, double *norms_out, int metric, int transform,
                         int norm, float p, double k, uint32_t padcol);
hipError_t launch_scan(hipStream_t st, int op, int R, int block, uint32_t lds_bytes, const ScanArgs &args);
hipError_t launch_finalize(hipStream_t st, const FinalizeArgs &args);
hipError_t launch_knn_merge(hipStream_t st, const KnnEntry *part, const int64_t *row_off, const int32_t *row_lists,
                            int64_t n_rows, int k, int negate, int64_t *out_idx, float *out_dist);
hipError_t launch_validate(hipStream_t st, const int64_t *indptr, const int32_t *indices, const float *values,
                           int64_t n_rows, int64_t n_cols, int64_t nnz, int require_nonnegative, int32_t *flag);
hipError_t set_scan_lds_limit(uint32_t bytes);

}  // namespace spd
