// Host-side plan: how the rows of A are grouped and staged in LDS, and how the rows of B
// are cut into 64-lane slabs that the wavefronts scan.
//
// The paper stages one row of A per block in shared memory - dense when the dimensionality
// allows it, a hash table when only the degree does, several partitions when neither does
// (Sections 3.3.2, 3.3.3) - and balances the load over B through a COO row index
// (Section 3.3).  On an MI355X the 160 KB of LDS per compute unit are spent differently:
//   * R rows of A (up to 16) are staged together, so that every entry of B that a lane
//     loads is applied to R rows;
//   * the staged rows share ONE column map (direct strip, 16-bit column-slot strip, a bitmap of
//     the columns with running counts, or a hash table of the union of their columns) in front
//     of a table of R values per column, so a column of B is looked up once for the R rows;
//   * rows that do not fit alone are cut into contiguous slices whose partial results are
//     summed afterwards (the partitions of Section 3.3.3, by column range); or (option) they
//     stay in global memory behind a Bloom filter of their columns in LDS, and a column
//     that passes the filter is looked up by binary search (the alternative Section 3.3.2
//     closes with);
//   * B is repacked once per call into "slabs" of 64 rows of similar degree, one row per
//     lane, stored so that the t-th entries of the 64 rows are contiguous (shorter rows
//     padded with a column that stages nothing).  Each lane
//     keeps its pairs' sums in registers: no segmented reduction, no atomics.  Rows
//     longer than `split_len` are cut into 2..64 equal segments that sit in adjacent
//     lanes and are summed across lanes once, at the end of the slab.
#pragma once
#include <stdint.h>

#include <string>
#include <vector>

#include "spd_ops.h"

namespace spd {

enum StageKind { KIND_AUTO = 0, KIND_STRIP = 1, KIND_SLOT = 2, KIND_HASH = 3, KIND_BLOOM = 4, KIND_BITMAP = 5 };

constexpr int kWave = 64;
constexpr int kScanUnroll = 4;              // a slab is scanned in blocks of this many steps
constexpr int kMaxR = 32;                   // 32 only for the set metrics (one byte per staged row)
constexpr uint32_t kEmptyKey = 0xFFFFFFFFu;
constexpr int kKnnMaxK = 64;                // fused k-NN: one list entry per lane
constexpr int kTopRanks = 32;               // sum() = max: largest one-sided contributions tracked per staged row
constexpr uint32_t kStaticLds = 4096;       // upper bound of the kernels' static __shared__ use

struct PlanOptions {
    int64_t lds_budget = 160 * 1024;        // bytes of LDS per workgroup (static + dynamic)
    int force_kind = KIND_AUTO;
    int max_rows = 8;                       // 16 halves the wavefronts a compute unit can hold
    int split_len = 0;                      // 0: by the size of B (see split_len_for)
    int window = 0;                         // rows of the streamed operand per degree-sorting window (0: see window_for)
    int chunks = 0;
    int chunk_scale = 0;                    // the cost model's number of chunks is multiplied by this (0: see chunk_scale_for)
    int n_cus = 256;
    int waves_per_cu = 0;                   // wavefronts the launches aim to keep on a compute unit (0: 32)
    int bloom_long_rows = 0;                // 1: a row too long for the LDS gets a Bloom filter instead of slices
    int sort_slack = 1;                     // 1: B's rows are sorted by length in whole blocks of steps, 0: by exact length
    int partial_groups = 1;                 // 1: a group of R rows may leave a quarter of its places empty rather than fall to R/2
    int consecutive_groups = 0;             // 1: a group holds consecutive rows, in row order (see plan_a)
};

// Rows per degree-sorting window of the streamed operand.  A wide window leaves fewer idle lanes
// (a slab runs as long as its longest row: 18 % of the steps are padding on 10,000 rows of 5-250
// entries sorted 2,048 at a time, 7 % when they are sorted as one), a narrow one keeps the 64 rows
// of a slab near each other, which only matters where a lane's store is a lone 4-byte word of the
// streamed row's column: a pairwise call that stages A.  The fused top-k writes no distances, and
// with the operands' roles exchanged a lane writes whole sectors of its own row.
// (Measured: 10,000 x 10,000 rows, dominant launch of L1 0.62 -> 0.56 ms with the roles exchanged;
// a pairwise call that stages 1,024 rows against 300,000 goes from 11.2 to 13.6 ms at 8,192.)
// The cost model below counts rounds of workgroups and knows nothing of what the fused top-k does
// with a chunk: its lists meet the rows of B sorted by length, and in a shorter chunk the rows'
// lengths, hence their distances, vary less, so fewer candidates pass (and the last round of
// workgroups is a smaller share of the launch).  Measured with twice the model's chunks, k-NN calls:
// 65,536 x 26,000 L1 93.8 -> 83.4 ms, 500,000 x 2^20 Jaccard 41.8 -> 36.8, 10,000 x 10,000 cosine
// 0.61 -> 0.58 (dominant launch), 663,000 rows of two entries +3.5 % (plan_chunks leaves such short
// chunks alone); three or four times: the same or worse.  Pairwise calls: within 2 % either way, so
// they keep the model's number.
inline int chunk_scale_for(const PlanOptions &opt, bool knn) { return opt.chunk_scale > 0 ? opt.chunk_scale : (knn ? 2 : 1); }

enum WindowUse { WINDOW_SCATTERED_STORES = 0, WINDOW_NO_SCATTERED_STORES = 1 };
inline int window_for(const PlanOptions &opt, WindowUse use) {
    if (opt.window > 0) return opt.window;
    return use == WINDOW_SCATTERED_STORES ? 2048 : 65536;
}

// Bloom staging: filter bits per stored entry (two hash functions: ~1.4 % false positives), and
// the bounds of a filter's size.
constexpr uint32_t kBloomBitsPerEntry = 16;
constexpr uint32_t kBloomMinBits = 1024, kBloomMaxBits = 1u << 19;
// The products a Bloom-staged row serves: one row per workgroup, values fetched from global
// memory (not the byte-counted set metrics, not the ranked completion of sum() = max).
SPD_HD constexpr bool bloom_serves(int op) { return op != OP_CNT && op != OP_CHEB && op != OP_SEMI_EXT; }

// 4-byte words a slot of the staged value table holds for R rows: one fp32 per row, or one
// byte per row for the set metrics.
SPD_HD constexpr int table_words(int op, int R) { return op == OP_CNT ? (R + 3) / 4 : R; }
constexpr int kCntMaxSteps = 252;           // byte counters are folded into 32-bit counts at least this often

// Rows of B at least this long are cut over several lanes.  Long segments amortise what a slab
// costs beside its steps; a small B needs many short slabs to keep every wavefront busy.
inline int split_len_for(const PlanOptions &opt, int64_t nnz_b) {
    if (opt.split_len > 0) return opt.split_len;
    return nnz_b >= ((int64_t)4 << 20) ? 512 : 256;
}

// Sums a pair carries through the slices of a spilled row.
SPD_HD constexpr int metric_planes(int metric) {
    return (metric == MT_MINKOWSKI || metric == MT_L2_UNEXPANDED || metric == MT_SEMI_SUM)
               ? 3 : ((metric == MT_JS || metric == MT_KL_STRICT) ? 2 : 1);
}

// Metrics whose sum() is a maximum: a staged row's largest one-sided contributions are ranked
// beside the value table, and the slices of a spilled row are joined by max.
SPD_HD constexpr bool sum_is_max(int metric) { return metric == MT_CHEBYSHEV || metric == MT_SEMI_EXT; }
// Products that carry two fp64 sums (or more) per pair: at most 8 rows are staged together.
SPD_HD constexpr bool wide_sums(int metric) {
    return metric == MT_JS || metric == MT_MINKOWSKI || metric == MT_L2_UNEXPANDED || metric == MT_SEMI_SUM || metric == MT_SEMI_EXT;
}

// Largest workgroup a scan kernel instance may be launched with: the instances that carry
// the most per-lane state get 256 registers per lane instead of 128.
SPD_HD constexpr int scan_max_block(int op, int R, bool knn) {
    if (op == OP_CNT) return (knn && R >= 16) ? 512 : 1024;
    if (op == OP_MINK || op == OP_MINK_ANY) return 512;
    return (R == 16 || ((op == OP_JS || op == OP_CHEB) && R == 8)) ? 512 : 1024;
}

// Wavefronts per SIMD the compiler is asked to make room for (it bounds the registers per
// lane: 8 means at most 64).  The light pairwise instances of eight rows run two workgroups of
// 16 wavefronts per compute unit that way, and hide the LDS reads of a step behind each other;
// every other instance runs fewer wavefronts and looks its columns up a block of steps ahead.
SPD_HD constexpr int scan_min_waves(int op, int R, int kind, bool knn) {
    if (!knn && R == 8 && kind != 3 /* KIND_HASH */ && kind != 5 /* KIND_BITMAP */ && (op == OP_DOT || op == OP_L1 || op == OP_CNT || op == OP_HAMM || op == OP_CANB)) return 8;
    // (the fused top-k keeps its lists in LDS: these instances fit the 64 registers as well, spilling a
    // dozen words in the slab epilogue; 10,000 x 10,000 rows, cosine, k = 32: 0.67 -> 0.55 ms.  Not the set
    // metrics' sixteen rows: 0.54 -> 0.63 ms)
    if (knn && R == 8 && kind != 3 /* KIND_HASH */ && kind != 5 /* KIND_BITMAP */ && (op == OP_DOT || op == OP_L1 || op == OP_HAMM || op == OP_CANB)) return 8;
    // (the k-NN instances of these sit a register or two above 128 otherwise)
    if (knn && R == 8 && ((op == OP_JS && kind != 3 /* KIND_HASH */) || op == OP_CHEB)) return 4;
    return 1;
}

// Dynamic-LDS layout of one staged group.  The same function sizes the launch on the host
// and carves the buffer in the kernel.  `R` here is table_words(op, rows).
struct LdsLayout {
    uint32_t nslots;     // rows of the value table (R floats each)
    uint32_t cap;        // hash capacity in entries (power of two, two entries per bucket), 0 otherwise
    uint32_t off_vals, off_map, off_rank, off_knn, total;
};

// Fused k-NN: per staged row the workgroup keeps one sorted list of the best candidates so far
// (64 keys of 8 bytes) and a queue of 64 candidates waiting to be merged into it.
constexpr uint32_t kKnnAreaBytes = 2u * 64u * 8u;

// Bitmap staging: one 8-byte word per 32 columns {the columns' bits, the number of staged columns
// below the word plus one}; the word of the column one past the last (the idle column) exists too.
SPD_HD constexpr uint32_t bitmap_words(uint32_t k) { return (k >> 5) + 1u; }

SPD_HD uint32_t pow2_at_least(uint32_t v) {
    uint32_t c = 16;
    while (c < v) c <<= 1;
    return c;
}

// `hscale`: the hash table holds at least sumlen << hscale entries (1..3: load <= 1/2, 1/4, 1/8).
// `knn_rows`: staged rows that keep a k-NN list (0 for a pairwise launch).
SPD_HD LdsLayout lds_layout(int kind, int R, uint32_t sumlen, uint32_t k, bool cheb, int hscale, uint32_t knn_rows = 0) {
    LdsLayout L;
    L.cap = 0;
    if (kind == KIND_BLOOM) {
        // only the filter: `cap` bits at off_map; the values stay in global memory
        uint32_t want = sumlen > kBloomMaxBits / kBloomBitsPerEntry ? kBloomMaxBits : sumlen * kBloomBitsPerEntry;
        uint32_t bits = kBloomMinBits;
        while (bits < want && bits < kBloomMaxBits) bits <<= 1;
        L.cap = bits;
        L.nslots = 0;
        L.off_vals = 0; L.off_map = 0;
        L.off_rank = bits / 8u;
        L.off_knn = bits / 8u;
        L.total = bits / 8u + knn_rows * kKnnAreaBytes;
        return L;
    }
    L.nslots = (kind == KIND_STRIP) ? k + 1u : sumlen + 1u;
    uint32_t off = 0;
    L.off_vals = off;
    off += ((L.nslots * (uint32_t)R * 4u) + 15u) & ~15u;
    L.off_map = off;
    if (kind == KIND_SLOT) {
        off += ((k + 1u) * 2u + 15u) & ~15u;
    } else if (kind == KIND_BITMAP) {
        off += (bitmap_words(k) * 8u + 15u) & ~15u;
    } else if (kind == KIND_HASH) {
        L.cap = pow2_at_least(sumlen << hscale);
        off += L.cap * 8u;
    }
    L.off_rank = off;
    if (cheb) off += ((L.nslots * (uint32_t)R) + 15u) & ~15u;
    L.off_knn = off;
    off += knn_rows * kKnnAreaBytes;
    L.total = off;
    return L;
}

// One row (or slice of a row) of A staged by a workgroup.
struct ARow {
    int64_t start;   // first element in A's CSR arrays
    int32_t len;     // number of stored entries of the slice
    int32_t out;     // >= 0: output row i;  -1: unused;  <= -2: partial-result slot (-2 - out)
    uint32_t flags;  // bit 0: holds the first entry of its row, bit 1: holds the last one
    uint32_t reserved;
};
constexpr uint32_t kRowFirst = 1u, kRowLast = 2u;

// One kernel launch: groups of R rows that share the staging kind.
struct AClass {
    int R = 0;
    int kind = 0;
    int hscale = 1;             // KIND_HASH: log2 of table entries per staged entry
    int block = 0;              // threads per workgroup
    uint32_t lds_bytes = 0;     // dynamic LDS of the launch (max over its groups)
    int n_groups = 0;
    std::vector<ARow> rows;         // n_groups * R
    std::vector<int32_t> sumlen;    // n_groups
    int n_chunks = 0;               // how this launch cuts B's slabs (plan_chunks)
    std::vector<int32_t> chunk_begin;   // n_chunks + 1 slab indices
    double cost = 0.0;              // plan_chunks' estimate of the launch's time, in slab steps of one wavefront
    int pool_slot = 0;              // where the planner keeps this class's buffers between calls
};

struct SpilledRow { int32_t row, first_slot, n_slots; };

struct APlan {
    int64_t n_rows = 0;
    std::vector<AClass> classes;
    std::vector<SpilledRow> spilled;
    int n_partial_slots = 0;
    // buffers the planner reuses from call to call (a plan object that is planned into
    // again allocates nothing once it has seen the largest input)
    std::vector<AClass> pool;
    std::vector<ARow> items, sorted;
    std::vector<uint32_t> sort_start;
};

struct BPlan {
    int64_t n_rows = 0, nnz = 0;
    int32_t n_slabs = 0;
    std::vector<int64_t> slab_base;    // n_slabs + 1, offsets into the packed entries (64 * steps each)
    std::vector<int32_t> slab_steps;   // n_slabs, longest segment of the slab rounded up to whole blocks
    std::vector<uint8_t> slab_split;   // n_slabs, largest log2(lanes per row) in the slab: 0 = no split rows
    std::vector<int64_t> seg_start;    // n_slabs*64, first CSR element of the lane's segment
    std::vector<int32_t> seg_len;      // n_slabs*64
    std::vector<int32_t> seg_row;      // n_slabs*64, row j of B, -1 for an unused lane
    std::vector<uint8_t> seg_glog;     // n_slabs*64, log2(lanes the row is split over)
    // planner scratch, kept between calls
    struct LongRow { int32_t row; int64_t len; int glog; };
    std::vector<LongRow> longs, longs_sorted;
    std::vector<int32_t> order, window_end, bucket_count, pos;
};

// Staging kind for a column count, the largest number of rows staged together, and the
// longest slice of a row that fits alone (0 = no limit).  Empty string on success.
// `op` is the product whose kernels will run (the metric's own, or OP_DOT standing in for OP_CNT).
std::string plan_staging(int64_t n_cols, int metric, int op, bool knn, const PlanOptions &opt, int &kind, int &max_r,
                         int &min_r, uint64_t &dmax);

// Both return an empty string on success, else the reason.
std::string plan_b(const int64_t *indptr, int64_t n_rows, const PlanOptions &opt, BPlan &out);
// With opt.consecutive_groups the staged rows are not sorted by length: rows 8q .. 8q+7 (32q .. 32q+31
// for the set metrics) form a group, halved where the eight do not fit together, so that the R
// results a lane holds for one streamed row are neighbours in a matrix whose fast dimension is
// the staged operand's row number (the library stages B and streams A that way when the output's
// stores would otherwise be scattered: a lane then writes whole 32-byte sectors).
std::string plan_a(const int64_t *indptr, int64_t n_rows, int64_t n_cols, int metric, int op, int knn_k,
                   const PlanOptions &opt, APlan &out);
// Cuts B's slabs into chunks for one launch: enough workgroups to fill the chip, yet chunks
// long enough that a workgroup's wavefronts stay evenly loaded and staging is amortised.
void plan_chunks(const BPlan &b, AClass &c, const PlanOptions &opt);

// Checks every index a kernel will form from the plan (bounds of segments, slabs, groups,
// LDS sizes).  Empty string if consistent.
std::string plan_check(const APlan &a, const BPlan &b, const int64_t *a_indptr, const int64_t *b_indptr,
                       int64_t n_cols, int metric, int op, int knn_k, const PlanOptions &opt);

}  // namespace spd
