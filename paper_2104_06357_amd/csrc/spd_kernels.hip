// Kernels around the staged scan: repacking of B into 64-lane slabs with its row norms
// (Section 3.4: norms by a row-wise reduction), summation of the slices of spilled rows
// (Section 3.3.3), merging of k-NN candidate lists, and CSR validation.
#include <hip/hip_runtime.h>

#include "spd_kernels.h"
#include "spd_scan_impl.h"

namespace spd {

// ------------------------------------------------------------------------------------
// B: CSR -> slabs.  One wavefront per slab, one segment per lane; the t-th entries of
// the 64 lanes are written side by side (a lane whose segment has ended writes the pad
// column), so the scan reads them back with one coalesced load per step.  The lane also
// sums its part of the row norm.
// ------------------------------------------------------------------------------------
constexpr int kPackTile = 16;       // steps of a slab that pass through LDS together

// kPackWaves: wavefronts of a workgroup, which take the slab's tiles in turn (8 for a B of few
// slabs, where the longest slab sets the time; 4 otherwise, so that more slabs run at once).
template <int kPackWaves>
__global__ void __launch_bounds__(kPackWaves * kWave) spd_pack_b_kernel(const int64_t *__restrict__ b_indptr,
                                                         const int32_t *__restrict__ b_indices,
                                                         const float *__restrict__ b_values, BDevice b,
                                                         uint2 *__restrict__ packed, double *__restrict__ norms,
                                                         int metric, int transform, int norm, float p, double k,
                                                         uint32_t padcol) {
    // One workgroup per slab, its wavefronts taking the slab's tiles of 16 steps in turn.
    // The CSR rows are read along the rows (16 consecutive entries of a row per quarter
    // wavefront: a cache line) into an LDS tile and written out along the steps (the 64 lanes'
    // entries of one step are 512 contiguous bytes): both sides coalesced.
    __shared__ uint2 s_tile[kPackWaves][kPackTile][kWave];
    __shared__ double s_sums[kPackWaves][kWave][2];
    const int lane = (int)threadIdx.x & 63, wave = (int)threadIdx.x >> 6;
    const int s = (int)blockIdx.x;
    const size_t at = (size_t)s * kWave + lane;
    const int64_t start = b.seg_start[at];
    const int len = b.seg_len[at];
    const int row = b.seg_row[at];
    const int glog = b.seg_glog[at];
    const int steps = b.slab_steps[s];
    uint2 *dst = packed + b.slab_base[s] + lane;
    uint2 (*tile)[kWave] = s_tile[wave];
    const int quarter = lane / kPackTile, within = lane % kPackTile;
    double s0 = 0.0, s1 = 0.0;
    for (int t0 = wave * kPackTile; t0 < steps; t0 += kPackWaves * kPackTile) {
        // fixed trip counts, so that all of a tile's loads are in flight together
        uint2 got[kPackTile];
#pragma unroll
        for (int i = 0; i < kPackTile; ++i) {
            const int r = i * (kWave / kPackTile) + quarter;
            const int rl = __shfl(len, r);
            const int64_t rs = __shfl(start, r);
            const int t = t0 + within;
            got[i] = make_uint2(padcol, 0u);
            if (t < rl) {
                const float v = transform_value(transform, b_values[rs + t]);
                // a stored zero of a set metric is absent: it takes the column that stages nothing
                const uint32_t col = (transform == TR_NONZERO && v == 0.0f) ? padcol : (uint32_t)b_indices[rs + t];
                got[i] = make_uint2(col, __float_as_uint(v));
            }
        }
#pragma unroll
        for (int i = 0; i < kPackTile; ++i) tile[within][i * (kWave / kPackTile) + quarter] = got[i];
        __builtin_amdgcn_wave_barrier();
        const int nt = min(kPackTile, steps - t0);
#pragma unroll
        for (int tt = 0; tt < kPackTile; ++tt) {
            if (tt < nt) {
                uint2 e = make_uint2(padcol, 0u);
                if (t0 + tt < len) {
                    e = tile[tt][lane];
                    norm_accumulate(norm, __uint_as_float(e.y), p, s0, s1);
                }
                dst[(size_t)(t0 + tt) * kWave] = e;
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
    // the wavefronts' shares of each row's sums, added in a fixed order
    s_sums[wave][lane][0] = s0;
    s_sums[wave][lane][1] = s1;
    __syncthreads();
    if (wave != 0) return;
    s0 = 0.0; s1 = 0.0;
#pragma unroll
    for (int w = 0; w < kPackWaves; ++w) { s0 += s_sums[w][lane][0]; s1 += s_sums[w][lane][1]; }
    if (b.slab_split[s]) {
#pragma unroll
        for (int step = 0; step < 6; ++step) {
            double o0 = __shfl_xor(s0, 1 << step), o1 = __shfl_xor(s1, 1 << step);
            if (step < glog) { s0 += o0; s1 += o1; }
        }
    }
    if (row >= 0 && (lane & ((1 << glog) - 1)) == 0) {
        double d0, d1;
        norm_derive(metric, k, s0, s1, d0, d1);
        norms[(size_t)row * 2] = d0;
        norms[(size_t)row * 2 + 1] = d1;
    }
}

hipError_t launch_pack_b(hipStream_t st, const int64_t *b_indptr, const int32_t *b_indices, const float *b_values,
                         const BDevice &b, uint2 *packed_out, double *norms_out, int metric, int transform,
                         int norm, float p, double k, uint32_t padcol) {
    if (b.n_slabs <= 0) return hipSuccess;
    dim3 grid((unsigned)b.n_slabs);
    if (b.n_slabs <= 1024)
        hipLaunchKernelGGL(spd_pack_b_kernel<8>, grid, dim3(8 * kWave), 0, st, b_indptr, b_indices, b_values, b, packed_out,
                           norms_out, metric, transform, norm, p, k, padcol);
    else
        hipLaunchKernelGGL(spd_pack_b_kernel<4>, grid, dim3(4 * kWave), 0, st, b_indptr, b_indices, b_values, b, packed_out,
                           norms_out, metric, transform, norm, p, k, padcol);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// Spilled rows of A: add up the partial results of their slices, then finish.
// Pairwise: grid (column tiles, spilled rows).  k-NN: one workgroup per spilled row keeps
// the k best while it walks the row.
// ------------------------------------------------------------------------------------
__device__ __forceinline__ float finalize_one(const FinalizeArgs &a, const SpilledRow &sr, int64_t j,
                                              double na0, double na1) {
    const bool by_max = sum_is_max(a.q.metric);
    double v0 = by_max ? -__builtin_huge_val() : 0.0, v1 = 0.0, v2 = 0.0;
    for (int q = 0; q < sr.n_slots; ++q) {
        size_t slot = (size_t)(sr.first_slot + q);
        double t = a.partial[(slot * a.planes) * (size_t)a.n_b + (size_t)j];
        if (by_max) v0 = fmax(v0, t); else v0 += t;
        if (a.planes >= 2) v1 += a.partial[(slot * a.planes + 1) * (size_t)a.n_b + (size_t)j];
        if (a.planes == 3) v2 += a.partial[(slot * 3 + 2) * (size_t)a.n_b + (size_t)j];
    }
    return finish(a.q, v0, v1, v2, na0, na1, a.norms_b[(size_t)j * 2], a.norms_b[(size_t)j * 2 + 1]);
}

__device__ __forceinline__ void spilled_row_norms(const FinalizeArgs &a, const SpilledRow &sr, double &na0,
                                                  double &na1) {
    double r0 = 0.0, r1 = 0.0;
    for (int q = 0; q < sr.n_slots; ++q) {
        r0 += a.partial_norms[(size_t)(sr.first_slot + q) * 2];
        r1 += a.partial_norms[(size_t)(sr.first_slot + q) * 2 + 1];
    }
    norm_derive(a.q.metric, a.q.k, r0, r1, na0, na1);
}

__global__ void __launch_bounds__(256) spd_finalize_pairwise_kernel(const FinalizeArgs a) {
    const SpilledRow sr = a.spilled[blockIdx.y];      // (the launcher passes `spilled` advanced to its tile of rows)
    double na0, na1;
    spilled_row_norms(a, sr, na0, na1);
    int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j < a.n_b)
        a.out[(size_t)sr.row * (size_t)a.out_stride_staged + (size_t)j * (size_t)a.out_stride_streamed] = finalize_one(a, sr, j, na0, na1);
}

__global__ void __launch_bounds__(256) spd_finalize_knn_kernel(const FinalizeArgs a) {
    // grid (tiles of kFinalizeTile columns, spilled rows): the k best of the tile go to the
    // row's candidate lists, which the merge kernel joins like those of the scan's chunks
    __shared__ KnnEntry s_area[4 * kKnnMaxK];
    const SpilledRow sr = a.spilled[blockIdx.y];
    const int lane = (int)threadIdx.x & 63, wave = (int)threadIdx.x >> 6;
    const int kk = a.knn_k;
    double na0, na1;
    spilled_row_norms(a, sr, na0, na1);
    KnnList list;
    list.reset();
    const int64_t j_begin = (int64_t)blockIdx.x * kFinalizeTile;
    const int64_t j_end = min(j_begin + (int64_t)kFinalizeTile, a.n_b);
    for (int64_t j0 = j_begin; j0 < j_end; j0 += 256) {
        int64_t j = j0 + threadIdx.x;
        bool valid = j < j_end;
        float d = 0.f;
        if (valid) {
            d = finalize_one(a, sr, j, na0, na1);
            if (a.q.metric == MT_INNER) d = 0.0f - d;
        }
        list.offer(d, (int)j, valid, kk, __builtin_huge_valf());
    }
    if (lane < kk) s_area[wave * kk + lane] = KnnEntry{list.d, list.j};
    __syncthreads();
    if (wave == 0) {
        KnnList merged;
        merged.reset();
        const int total = 4 * kk;
        for (int e0 = 0; e0 < total; e0 += 64) {
            int e = e0 + lane;
            bool valid = e < total;
            KnnEntry c = KnnEntry{0.f, 0};
            if (valid) c = s_area[e];
            valid = valid && c.j != 0x7fffffff;
            merged.offer(c.d, c.j, valid, kk, __builtin_huge_valf());
        }
        if (lane < kk) a.knn_part[a.knn_row_off[sr.row] + (int64_t)blockIdx.x * kk + lane] = KnnEntry{merged.d, merged.j};
    }
}

hipError_t launch_finalize(hipStream_t st, const FinalizeArgs &args) {
    if (args.n_spilled <= 0) return hipSuccess;
    // the second grid dimension holds at most 65,535 workgroups: the spilled rows go in tiles of that many
    constexpr int32_t kMaxGridY = 65535;
    for (int32_t first = 0; first < args.n_spilled; first += kMaxGridY) {
        FinalizeArgs part = args;
        part.spilled = args.spilled + first;
        part.n_spilled = std::min(kMaxGridY, args.n_spilled - first);
        if (args.knn_k > 0) {
            dim3 grid((unsigned)((args.n_b + kFinalizeTile - 1) / kFinalizeTile), (unsigned)part.n_spilled);
            hipLaunchKernelGGL(spd_finalize_knn_kernel, grid, dim3(256), 0, st, part);
        } else {
            dim3 grid((unsigned)((args.n_b + 255) / 256), (unsigned)part.n_spilled);
            hipLaunchKernelGGL(spd_finalize_pairwise_kernel, grid, dim3(256), 0, st, part);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ------------------------------------------------------------------------------------
// k-NN: one wavefront per query row merges the lists its chunks produced.
// ------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) spd_knn_merge_kernel(const KnnEntry *__restrict__ part,
                                                            const int64_t *__restrict__ row_off,
                                                            const int32_t *__restrict__ row_lists, int64_t n_rows,
                                                            int k, int negate, int64_t *__restrict__ out_idx,
                                                            float *__restrict__ out_dist) {
    const int lane = (int)threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + ((int)threadIdx.x >> 6);
    if (row >= n_rows) return;
    const int lists = row_lists[row];
    if (lists <= 0) return;
    KnnList merged;
    merged.reset();
    const int total = lists * k;
    const KnnEntry *src = part + row_off[row];
    for (int e0 = 0; e0 < total; e0 += 64) {
        int e = e0 + lane;
        bool valid = e < total;
        KnnEntry c = KnnEntry{0.f, 0};
        if (valid) c = src[e];
        valid = valid && c.j != 0x7fffffff;
        merged.offer(c.d, c.j, valid, k, __builtin_huge_valf());
    }
    if (lane < k) {
        out_idx[(size_t)row * k + lane] = (int64_t)merged.j;
        out_dist[(size_t)row * k + lane] = negate ? -merged.d : merged.d;
    }
}

hipError_t launch_knn_merge(hipStream_t st, const KnnEntry *part, const int64_t *row_off, const int32_t *row_lists,
                            int64_t n_rows, int k, int negate, int64_t *out_idx, float *out_dist) {
    if (n_rows <= 0) return hipSuccess;
    dim3 grid((unsigned)((n_rows + 3) / 4));
    hipLaunchKernelGGL(spd_knn_merge_kernel, grid, dim3(256), 0, st, part, row_off, row_lists, n_rows, k, negate,
                       out_idx, out_dist);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------
// CSR validation: bit 0 row pointers, bit 1 column order / range, bit 2 values.
// ------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) spd_validate_kernel(const int64_t *__restrict__ indptr,
                                                           const int32_t *__restrict__ indices,
                                                           const float *__restrict__ values, int64_t n_rows,
                                                           int64_t n_cols, int64_t nnz, int require_nonnegative,
                                                           int32_t *flag) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n_rows) return;
    int bad = 0;
    const int64_t a = indptr[i], b = indptr[i + 1];
    if ((i == 0 && a != 0) || (i == n_rows - 1 && b != nnz) || a > b || a < 0 || b > nnz) {
        bad |= 1;
    } else {
        for (int64_t q = a; q < b; ++q) {
            int32_t c = indices[q];
            if (c < 0 || c >= n_cols || (q > a && indices[q - 1] >= c)) bad |= 2;
            float v = values[q];
            if (!(v - v == 0.0f) || (require_nonnegative && v < 0.0f)) bad |= 4;
        }
    }
    if (bad) atomicOr(flag, bad);
}

hipError_t launch_validate(hipStream_t st, const int64_t *indptr, const int32_t *indices, const float *values,
                           int64_t n_rows, int64_t n_cols, int64_t nnz, int require_nonnegative, int32_t *flag) {
    if (n_rows <= 0) return hipSuccess;
    dim3 grid((unsigned)((n_rows + 255) / 256));
    hipLaunchKernelGGL(spd_validate_kernel, grid, dim3(256), 0, st, indptr, indices, values, n_rows, n_cols, nnz,
                       require_nonnegative, flag);
    return hipGetLastError();
}

}  // namespace spd
