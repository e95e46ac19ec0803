// Host planner: degree binning of the rows of A and B (see spd_plan.h).
#include "spd_plan.h"

#include <algorithm>
#include <functional>
#include <numeric>

namespace spd {

namespace {

std::string fmt(const char *what, long long a, long long b = 0) {
    return std::string(what) + " (" + std::to_string(a) + ", " + std::to_string(b) + ")";
}

int block_for(uint32_t stage_bytes, int64_t lds_total, int waves_per_cu) {
    // As many workgroups per compute unit as the LDS holds (at most eight), sized so that
    // together they bring `waves_per_cu` wavefronts.
    int64_t per_cu = std::max<int64_t>(1, std::min<int64_t>(8, lds_total / (int64_t)(stage_bytes + kStaticLds)));
    int block = 64;
    while (block < 1024 && (int64_t)block * per_cu < (int64_t)waves_per_cu * 64) block *= 2;
    return std::max(block, 256);
}

// Launches are kept apart by how many workgroups of their LDS size a compute unit holds (four
// or more, two or three, one), so that groups needing little are not held to the occupancy of
// the heaviest.
int occupancy_bucket(uint32_t stage_bytes, int64_t lds_total) {
    int64_t per_cu = lds_total / (int64_t)(stage_bytes + kStaticLds);
    return per_cu >= 4 ? 0 : (per_cu >= 2 ? 1 : 2);
}

}  // namespace

// ------------------------------------------------------------------------------------
// B: slabs of 64 lanes
// ------------------------------------------------------------------------------------
std::string plan_b(const int64_t *indptr, int64_t n_rows, const PlanOptions &opt, BPlan &out) {
    out.n_rows = 0; out.nnz = 0; out.n_slabs = 0;
    if (n_rows < 0) return "negative row count";
    if (n_rows >= (int64_t)1 << 31) return "more than 2^31-1 rows";
    const int64_t T = std::max<int64_t>(2, split_len_for(opt, n_rows > 0 ? indptr[n_rows] : 0));
    const int64_t seg_target = std::max<int64_t>(1, T / 2);
    const int64_t Wn = std::max<int64_t>(kWave, (window_for(opt, WINDOW_SCATTERED_STORES) / kWave) * kWave);
    out.n_rows = n_rows;
    out.nnz = n_rows ? indptr[n_rows] : 0;
    if (n_rows && indptr[0] != 0) return "indptr[0] != 0";
    for (int64_t j = 0; j < n_rows; ++j)
        if (indptr[j + 1] < indptr[j]) return fmt("row pointers decrease at row", j);

    // Rows of a window are sorted by their length in whole blocks of kScanUnroll steps (a
    // slab's steps are a multiple of that anyway, so the coarser key costs nothing), longest first,
    // and by row number among equals: the rows of a slab then lie closer together in B, and
    // the 64 results of a slab's store touch fewer cache lines (a matrix whose rows hold one to
    // four entries is written in row order).  Option sort_slack 0 sorts by the exact length.
    const int64_t quantum = opt.sort_slack > 0 ? kScanUnroll : 1;
    auto class_of = [quantum](int64_t len) -> int64_t { return quantum == 1 ? len : (len + 3) >> 2; };
    static_assert(kScanUnroll == 4, "the shift above divides by kScanUnroll");
    using Long = BPlan::LongRow;
    std::vector<Long> &longs = out.longs;
    std::vector<int32_t> &order = out.order;            // short rows, window by window, longest first
    std::vector<int32_t> &window_end = out.window_end;  // prefix positions in `order`
    std::vector<int32_t> &bucket_count = out.bucket_count, &pos = out.pos;
    longs.clear(); order.clear(); window_end.clear();
    order.reserve((size_t)n_rows);
    bucket_count.assign((size_t)T + 1, 0); pos.assign((size_t)T + 1, 0);
    for (int64_t w0 = 0; w0 < n_rows; w0 += Wn) {
        int64_t w1 = std::min(n_rows, w0 + Wn);
        std::fill(bucket_count.begin(), bucket_count.end(), 0);
        for (int64_t j = w0; j < w1; ++j) {
            int64_t len = indptr[j + 1] - indptr[j];
            if (len >= T) {
                // the fewest lanes (a power of two, at most 64) whose segments are at most seg_target long
                int glog = 1;
                while (glog < 6 && (seg_target << glog) < len) ++glog;
                longs.push_back({(int32_t)j, len, glog});
            } else {
                ++bucket_count[(size_t)class_of(len)];
            }
        }
        // counting sort, longest first, stable in j
        int32_t acc = 0;
        for (int64_t l = T - 1; l >= 0; --l) { pos[(size_t)l] = acc; acc += bucket_count[(size_t)l]; }
        size_t base = order.size();
        order.resize(base + (size_t)acc);
        for (int64_t j = w0; j < w1; ++j) {
            int64_t len = indptr[j + 1] - indptr[j];
            if (len < T) order[base + (size_t)pos[(size_t)class_of(len)]++] = (int32_t)j;
        }
        window_end.push_back((int32_t)order.size());
    }
    // groups of equal size side by side, and within them segments of similar length: a stable
    // counting sort by (lanes per row, segment length), both descending.  Segments longer than
    // the last bucket belong to rows that fill a slab alone, so their order costs no padding.
    if (longs.size() > 1) {
        constexpr int kSegBuckets = 1024;
        auto key_of = [&](const Long &l) {
            int64_t seg = (l.len + ((int64_t)1 << l.glog) - 1) >> l.glog;
            int sb = (int)std::min<int64_t>(seg, kSegBuckets - 1);
            return (6 - l.glog) * kSegBuckets + (kSegBuckets - 1 - sb);      // ascending key = descending order
        };
        std::vector<int32_t> &count = out.bucket_count;       // reused below only per window: free here
        count.assign((size_t)7 * kSegBuckets + 1, 0);
        for (const Long &l : longs) ++count[(size_t)key_of(l) + 1];
        for (size_t q = 1; q < count.size(); ++q) count[q] += count[q - 1];
        out.longs_sorted.resize(longs.size());
        for (const Long &l : longs) out.longs_sorted[(size_t)count[(size_t)key_of(l)]++] = l;
        longs.swap(out.longs_sorted);
    }

    // count slabs
    int64_t long_lanes = 0;
    for (const Long &l : longs) long_lanes += (int64_t)1 << l.glog;
    int64_t n_long_slabs = (long_lanes + kWave - 1) / kWave;
    int64_t n_short_slabs = 0;
    {
        int32_t prev = 0;
        for (int32_t e : window_end) { n_short_slabs += (e - prev + kWave - 1) / kWave; prev = e; }
    }
    int64_t n_slabs = n_long_slabs + n_short_slabs;
    if (n_slabs >= ((int64_t)1 << 31) / kWave) return "too many slabs";
    out.n_slabs = (int32_t)n_slabs;
    size_t lanes = (size_t)n_slabs * kWave;
    // every lane is written exactly once below (the arrays keep their size from call to call)
    out.seg_start.resize(lanes);
    out.seg_len.resize(lanes);
    out.seg_row.resize(lanes);
    out.seg_glog.resize(lanes);
    out.slab_split.assign((size_t)n_slabs, 0);
    int64_t *const seg_start = out.seg_start.data();
    int32_t *const seg_len = out.seg_len.data();
    int32_t *const seg_row = out.seg_row.data();
    uint8_t *const seg_glog = out.seg_glog.data();
    auto idle = [&](size_t from, size_t to) {
        for (size_t q = from; q < to; ++q) { seg_start[q] = 0; seg_len[q] = 0; seg_row[q] = -1; seg_glog[q] = 0; }
    };

    size_t lane = 0;
    for (const Long &l : longs) {
        const int G = 1 << l.glog;
        const int64_t s0 = indptr[l.row];
        int64_t lo = 0;
        for (int q = 0; q < G; ++q, ++lane) {
            const int64_t hi = (l.len * (q + 1)) >> l.glog;        // equal shares, the remainder spread
            seg_start[lane] = s0 + lo;
            seg_len[lane] = (int32_t)(hi - lo);
            seg_row[lane] = l.row;
            seg_glog[lane] = (uint8_t)l.glog;
            lo = hi;
        }
        uint8_t &deepest = out.slab_split[(lane - 1) / kWave];
        deepest = std::max<uint8_t>(deepest, (uint8_t)l.glog);
    }
    idle(lane, (size_t)n_long_slabs * kWave);
    lane = (size_t)n_long_slabs * kWave;
    {
        int32_t prev = 0;
        for (int32_t e : window_end) {
            for (int32_t t = prev; t < e; ++t, ++lane) {
                int32_t j = order[(size_t)t];
                seg_start[lane] = indptr[j];
                seg_len[lane] = (int32_t)(indptr[j + 1] - indptr[j]);
                seg_row[lane] = j;
                seg_glog[lane] = 0;
            }
            const size_t end = (lane + kWave - 1) / kWave * kWave;
            idle(lane, end);
            lane = end;
            prev = e;
        }
    }
    out.slab_base.assign((size_t)n_slabs + 1, 0);
    out.slab_steps.assign((size_t)n_slabs, 0);
    // a slab stores steps x 64 entries: entry t of lane l at slab_base + t*64 + l, lanes whose
    // segment is shorter are padded with a column that no row stages; steps is a whole
    // number of scan blocks
    for (int64_t s = 0; s < n_slabs; ++s) {
        int32_t mx = 0;
        for (int l = 0; l < kWave; ++l) mx = std::max(mx, out.seg_len[(size_t)s * kWave + l]);
        mx = (mx + kScanUnroll - 1) / kScanUnroll * kScanUnroll;
        out.slab_base[(size_t)s + 1] = out.slab_base[(size_t)s] + (int64_t)mx * kWave;
        out.slab_steps[(size_t)s] = mx;
    }
    return std::string();
}

void plan_chunks(const BPlan &b, AClass &c, const PlanOptions &opt) {
    int64_t total = 0;
    int64_t longest = 1;
    for (int32_t s : b.slab_steps) { total += std::max(1, s); longest = std::max<int64_t>(longest, s); }
    const int waves = std::max(1, c.block / kWave);
    int nc = opt.chunks;
    // Model of the launch time in slab steps: workgroups pass over the chip's slots in
    // rounds; each stages its rows, then its wavefronts share the chunk's slabs, the
    // last one finishing up to a quarter of a slab after the others.
    const int64_t per_cu = std::max<int64_t>(1, std::min<int64_t>(opt.lds_budget / ((int64_t)c.lds_bytes + kStaticLds),
                                                                  (int64_t)32 / waves));
    const int64_t slots = (int64_t)opt.n_cus * per_cu;
    const double stage = 24.0;
    const bool light = per_cu >= 4;
    auto model = [&](int cand) {
        const int64_t wgs = (int64_t)c.n_groups * cand;
        // (workgroups do not run in lockstep: beyond one round the chip's slots are refilled as
        // they come free, and what is left of whole rounds is half a round on average.  Light
        // workgroups, four or more to a compute unit, differ enough in length that the half
        // round shows in a single round too: measured, their launches want more and smaller
        // chunks than one round's worth, the heavy ones do not.)
        const double rounds = (light || wgs > slots) ? (double)wgs / (double)slots + 0.5 : 1.0;
        // (a wavefront works its slab alone: no chunk is done before its longest slab is)
        const double per_wg = stage + std::max((double)total / cand / waves, (double)longest) + 0.25 * (double)longest;
        return rounds * per_wg;
    };
    if (nc <= 0) {
        // more workgroups than four per slot buy nothing
        const int64_t useful = 4 * slots / std::max(1, c.n_groups) + 1;
        const int max_nc = (int)std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(4096, useful), b.n_slabs / waves));
        double best = -1.0;
        nc = 1;
        for (int cand = 1; cand <= max_nc; cand = cand < 8 ? cand + 1 : (light ? (cand < 16 ? cand + 2 : (cand < 32 ? cand + 4 : cand + 8)) : cand + 8)) {
            const double t = model(cand);
            if (best < 0.0 || t < best * 0.98) { best = t; nc = cand; }
        }
        // (the caller has resolved the automatic value; a wavefront keeps a thousand steps or more to
        // itself: below that the staging and the lists of the extra workgroups cost what the shorter
        // chunks save, 663,000 rows of two entries: +3.5 %)
        int scale = opt.chunk_scale;
        while (scale > 1 && total / ((int64_t)nc * scale) / waves < 1024) --scale;
        if (scale > 1) {
            const int64_t cap = std::min<int64_t>(std::min<int64_t>(4096, (int64_t)scale * useful), std::max<int64_t>(1, b.n_slabs / waves));
            nc = (int)std::max<int64_t>(1, std::min<int64_t>((int64_t)nc * scale, cap));
        }
    }
    c.n_chunks = nc;
    c.cost = model(nc);
    c.chunk_begin.assign((size_t)nc + 1, b.n_slabs);
    c.chunk_begin[0] = 0;
    int64_t run = 0;
    int at = 1;
    for (int32_t s = 0; s < b.n_slabs && at < nc; ++s) {
        run += std::max(1, b.slab_steps[(size_t)s]);
        while (at < nc && run * nc >= total * at) c.chunk_begin[(size_t)at++] = s + 1;
    }
    for (; at < nc; ++at) c.chunk_begin[(size_t)at] = b.n_slabs;
    c.chunk_begin[(size_t)nc] = b.n_slabs;
}

namespace {

// `R`: words per slot of the value table; `knn_rows`: staged rows that keep a k-NN list.
bool staging_fits(int kind, int R, uint64_t sumlen, uint32_t k, bool cheb, int64_t budget, uint32_t knn_rows) {
    if (kind == KIND_BLOOM)
        return (int64_t)lds_layout(kind, R, (uint32_t)std::min<uint64_t>(sumlen, 1u << 30), k, cheb, 1, knn_rows).total <= budget;
    if (kind != KIND_STRIP && sumlen > 65534u) return false;      // 16-bit slot ids
    uint64_t nslots = (kind == KIND_STRIP) ? (uint64_t)k + 1u : sumlen + 1u;
    if (nslots * (uint64_t)R * 5u > (uint64_t)budget) return false;   // also keeps the 32-bit layout math safe
    LdsLayout L = lds_layout(kind, R, (uint32_t)sumlen, k, cheb, 1, knn_rows);
    return (int64_t)L.total <= budget;
}

}  // namespace

std::string plan_staging(int64_t n_cols, int metric, int op, bool knn, const PlanOptions &opt, int &kind, int &max_r,
                         int &min_r, uint64_t &dmax) {
    const bool cheb = sum_is_max(metric);
    const uint32_t k = (uint32_t)n_cols;
    max_r = std::min(opt.max_rows, 16);
    if (wide_sums(metric)) max_r = std::min(max_r, 8);   // two fp64 sums per pair
    // Minkowski: three sums per pair and the powers beside them: 4 rows keep the kernel within 128
    // registers, so that a compute unit holds two workgroups of 8 wavefronts
    if (op == OP_MINK || op == OP_MINK_ANY) max_r = std::min(max_r, 4);
    // The semiring kernels pick the product at run time, inside the step: with eleven products to
    // choose from and eight rows the compiler keeps a block's entries in scratch memory, and four rows
    // sweep B faster than eight (10,000 x 10,000 rows, {plus, min}: 1.23 against 1.62 ms)
    if (op == OP_SEMI_SUM || op == OP_SEMI_EXT) max_r = std::min(max_r, 4);
    if (max_r < 1) max_r = 1;
    while (max_r & (max_r - 1)) max_r &= max_r - 1;         // power of two
    min_r = 1;
    if (op == OP_CNT) {
        // a byte per row: four rows to the word; with the k-NN lists in registers as well, 8 rows
        // run faster than 16 (which max_rows = 16 still selects)
        min_r = 4;
        max_r = std::min(4 * max_r, knn ? (opt.max_rows > 8 ? 32 : 16) : 32);
    }
    auto words = [&](int R) { return table_words(op, R); };
    auto lists = [&](int R) { return knn ? (uint32_t)R : 0u; };
    if (opt.lds_budget <= (int64_t)kStaticLds + 256) return "lds_budget too small";
    const int64_t budget = opt.lds_budget - kStaticLds;
    kind = opt.force_kind;
    if (kind == KIND_AUTO) {
        if (staging_fits(KIND_STRIP, words(std::min(4 * min_r, max_r)), 0, k, cheb, budget, lists(std::min(4 * min_r, max_r)))) kind = KIND_STRIP;
        else if ((int64_t)(k + 1) * 2 <= budget / 3) kind = KIND_SLOT;
        else if ((int64_t)bitmap_words(k) * 8 <= budget / 3) kind = KIND_BITMAP;
        else kind = KIND_HASH;
    }
    if (kind < KIND_STRIP || kind > KIND_BITMAP) return "bad staging kind";
    dmax = 0;
    if (kind == KIND_BLOOM) {
        if (!bloom_serves(op)) return "Bloom staging does not serve this product";
        if ((int64_t)kBloomMaxBits / 8 > budget) return "lds_budget too small for a Bloom filter";
        max_r = min_r = 1;
        return std::string();
    }
    if (kind == KIND_STRIP) {
        if (!staging_fits(KIND_STRIP, words(min_r), 0, k, cheb, budget, lists(min_r))) return "dense strip does not fit the LDS budget";
        while (max_r > min_r && !staging_fits(KIND_STRIP, words(max_r), 0, k, cheb, budget, lists(max_r))) max_r /= 2;
        return std::string();
    }
    if (!staging_fits(kind, words(min_r), 1, k, cheb, budget, lists(min_r))) return "LDS budget too small to stage a single entry";
    uint64_t lo = 1, hi = 65534;
    while (lo < hi) {
        uint64_t mid = (lo + hi + 1) / 2;
        if (staging_fits(kind, words(min_r), mid, k, cheb, budget, lists(min_r))) lo = mid; else hi = mid - 1;
    }
    dmax = lo;
    return std::string();
}

// ------------------------------------------------------------------------------------
// A: groups of R staged rows
// ------------------------------------------------------------------------------------
std::string plan_a(const int64_t *indptr, int64_t n_rows, int64_t n_cols, int metric, int op, int knn_k,
                   const PlanOptions &opt, APlan &out) {
    // take the buffers of the previous plan back before anything else
    constexpr size_t kPool = 6 * 3 + 2;       // 6 group sizes x 3 occupancies, the dense strip's one class, the Bloom class
    if (out.pool.size() != kPool) out.pool.assign(kPool, AClass());
    for (AClass &c : out.classes) { const int slot = c.pool_slot; out.pool[(size_t)slot] = std::move(c); }
    out.classes.clear();
    out.spilled.clear();
    out.n_partial_slots = 0;
    for (AClass &c : out.pool) { c.rows.clear(); c.sumlen.clear(); c.chunk_begin.clear(); c.n_groups = 0; c.n_chunks = 0; c.hscale = 1; }
    out.n_rows = n_rows;
    if (n_rows < 0 || n_cols < 0) return "negative size";
    if (n_rows >= (int64_t)1 << 31 || n_cols >= ((int64_t)1 << 31) - 1) return "more than 2^31-2 rows or columns";
    if (n_rows && indptr[0] != 0) return "indptr[0] != 0";
    int64_t longest = 0;
    for (int64_t i = 0; i < n_rows; ++i) {
        if (indptr[i + 1] < indptr[i]) return fmt("row pointers decrease at row", i);
        longest = std::max(longest, indptr[i + 1] - indptr[i]);
    }
    const bool cheb = sum_is_max(metric);
    const uint32_t k = (uint32_t)n_cols;
    int kind = 0, max_r = 1, min_r = 1;
    uint64_t dmax = 0;
    {
        std::string why = plan_staging(n_cols, metric, op, knn_k > 0, opt, kind, max_r, min_r, dmax);
        if (!why.empty()) return why;
    }
    const int64_t budget = opt.lds_budget - kStaticLds;
    auto lists = [&](int R) { return knn_k > 0 ? (uint32_t)R : 0u; };
    auto fits = [&](int kd, int R, uint64_t sumlen) { return staging_fits(kd, table_words(op, R), sumlen, k, cheb, budget, lists(R)); };
    const int want_waves = opt.waves_per_cu > 0 ? opt.waves_per_cu : 32;

    auto finish_class = [&](AClass &c) {
        auto need_at = [&](int hs) {
            uint32_t need = 0;
            for (int g = 0; g < c.n_groups; ++g)
                need = std::max(need, lds_layout(c.kind, table_words(op, c.R), (uint32_t)c.sumlen[(size_t)g], k, cheb, hs, lists(c.R)).total);
            return need;
        };
        uint32_t need = need_at(1);
        c.hscale = 1;
        if (c.kind == KIND_HASH) {
            // a sparser table shortens the probe sequences: take the sparsest one that
            // leaves the launch as many workgroups per compute unit as it has now
            const int now = occupancy_bucket(need, opt.lds_budget);
            for (int hs = 3; hs >= 2; --hs) {
                uint32_t wider = need_at(hs);
                if ((int64_t)wider <= budget && occupancy_bucket(wider, opt.lds_budget) == now) { c.hscale = hs; need = wider; break; }
            }
        }
        c.block = std::min(block_for(need, opt.lds_budget, want_waves), scan_max_block(op, c.R, knn_k > 0));
        c.lds_bytes = (need + 15u) & ~15u;
    };

    if (kind == KIND_STRIP) {
        int R = max_r;
        AClass &c = out.pool[kPool - 2];
        c.pool_slot = (int)kPool - 2;
        c.R = R; c.kind = KIND_STRIP;
        c.n_groups = (int)((n_rows + R - 1) / R);
        c.rows.assign((size_t)c.n_groups * R, ARow{0, 0, -1, kRowFirst | kRowLast, 0});
        c.sumlen.assign((size_t)c.n_groups, 0);
        for (int64_t i = 0; i < n_rows; ++i) {
            int64_t len = indptr[i + 1] - indptr[i];
            if (len > (int64_t)k) return fmt("row longer than the column count", i);
            c.rows[(size_t)i] = ARow{indptr[i], (int32_t)len, (int32_t)i, kRowFirst | kRowLast, 0};
            c.sumlen[(size_t)(i / R)] += (int32_t)len;
        }
        if (c.n_groups) { finish_class(c); out.classes.push_back(std::move(c)); }
        return std::string();
    }

    // rows behind a Bloom filter: one per workgroup, whole, whatever their length
    AClass &bloom = out.pool[kPool - 1];
    bloom.pool_slot = (int)kPool - 1;
    bloom.R = 1; bloom.kind = KIND_BLOOM;
    const bool bloom_all = kind == KIND_BLOOM;
    const bool bloom_long = !bloom_all && opt.bloom_long_rows && bloom_serves(op) &&
                            (int64_t)kBloomMaxBits / 8 <= budget;
    // Rows (and slices of rows) sorted by length, longest first, stable: a counting sort whose
    // histogram is filled while the items are made.
    std::vector<ARow> &items = out.items;
    std::vector<uint32_t> &start = out.sort_start;
    const size_t len_cap = (size_t)std::min<uint64_t>(std::min<uint64_t>(dmax, (uint64_t)longest), 65534u) + 2;   // lengths 0..dmax
    start.assign(len_cap + 1, 0);
    items.resize((size_t)n_rows);
    size_t n_items = 0;
    for (int64_t i = 0; i < n_rows; ++i) {
        const int64_t len = indptr[i + 1] - indptr[i];
        if (len > (int64_t)k) return fmt("row longer than the column count", i);
        if ((uint64_t)len <= dmax && !bloom_all) {
            items[n_items++] = ARow{indptr[i], (int32_t)len, (int32_t)i, kRowFirst | kRowLast, 0};
            ++start[(size_t)len];
        } else if (bloom_all || bloom_long) {
            bloom.rows.push_back(ARow{indptr[i], (int32_t)len, (int32_t)i, kRowFirst | kRowLast, 0});
            bloom.sumlen.push_back((int32_t)len);
            ++bloom.n_groups;
        } else {
            int64_t parts = (len + (int64_t)dmax - 1) / (int64_t)dmax;
            if (out.n_partial_slots + parts > (1 << 24)) return "too many row slices";
            out.spilled.push_back(SpilledRow{(int32_t)i, out.n_partial_slots, (int32_t)parts});
            if (items.size() < n_items + (size_t)parts + (size_t)(n_rows - i)) items.resize(n_items + (size_t)parts + (size_t)(n_rows - i));
            for (int64_t q = 0; q < parts; ++q) {
                int64_t lo = len * q / parts, hi = len * (q + 1) / parts;
                uint32_t fl = (q == 0 ? kRowFirst : 0u) | (q == parts - 1 ? kRowLast : 0u);
                items[n_items++] = ARow{indptr[i] + lo, (int32_t)(hi - lo), -2 - (out.n_partial_slots++), fl, 0};
                ++start[(size_t)(hi - lo)];
            }
        }
    }
    items.resize(n_items);
    {
        // start[l] = number of items longer than l
        uint32_t longer = 0;
        for (size_t l = len_cap; l-- > 0;) { const uint32_t here = start[l]; start[l] = longer; longer += here; }
        std::vector<ARow> &sorted = out.sorted;
        sorted.resize(n_items);
        for (const ARow &r : items) sorted[start[(size_t)r.len]++] = r;
        items.swap(sorted);
    }

    // one launch per (R, workgroups per compute unit): groups that need little LDS are not
    // held to the occupancy of the heaviest ones
    AClass *by_key[6][3];                     // R = 32, 16, 8, 4, 2, 1  x  workgroups of that LDS size per compute unit
    for (int q = 0; q < 6; ++q)
        for (int b = 0; b < 3; ++b) {
            by_key[q][b] = &out.pool[(size_t)(q * 3 + b)];
            by_key[q][b]->pool_slot = q * 3 + b;
            by_key[q][b]->R = 32 >> q;
            by_key[q][b]->kind = kind;
        }
    // the largest sum of lengths a group of R rows may stage (staging_fits is monotone in it)
    uint64_t room[6];
    for (int q = 0; q < 6; ++q) {
        const int R = 32 >> q;
        room[q] = 0;
        if (R > max_r || R < min_r || !fits(kind, R, 0)) continue;
        uint64_t lo = 0, hi = 65534;
        while (lo < hi) {
            const uint64_t mid = (lo + hi + 1) / 2;
            if (fits(kind, R, mid)) lo = mid; else hi = mid - 1;
        }
        room[q] = lo;
    }
    auto room_of = [&](int R) { int q = 0; while ((32 >> q) != R) ++q; return room[q]; };
    auto fits_group = [&](int R, uint64_t sum) { return sum <= room_of(R) && (sum == 0 ? fits(kind, R, 0) : true); };
    auto emit_group = [&](int R, const ARow *rows, size_t n, uint64_t sum) {
        int ci = 0;
        while ((32 >> ci) != R) ++ci;
        uint32_t need = lds_layout(kind, table_words(op, R), (uint32_t)sum, k, cheb, 1, lists(R)).total;
        AClass &c = *by_key[ci][occupancy_bucket(need, opt.lds_budget)];
        for (int q = 0; q < R; ++q)
            c.rows.push_back((size_t)q < n ? rows[q] : ARow{0, 0, -1, kRowFirst | kRowLast, 0});
        c.sumlen.push_back((int32_t)sum);
        ++c.n_groups;
    };
    size_t t = 0;
    if (opt.consecutive_groups) {
        // Whole rows in row order, in aligned blocks of R0; the slices of the rows that do not fit
        // alone (sorted to the front of `items`, their outputs are partial slots) are grouped among
        // themselves below.  A block that is too much for the table is cut in halves, each half
        // keeping its place in the row order; a row that was taken out as slices leaves an empty
        // place behind.
        int R0 = op == OP_CNT ? max_r : std::min(max_r, 8);
        while (R0 > min_r && room_of(R0) == 0 && !fits(kind, R0, 0)) R0 /= 2;
        std::vector<ARow> whole((size_t)n_rows, ARow{0, 0, -1, kRowFirst | kRowLast, 0});
        std::vector<ARow> &sl = out.sorted;          // the slices, still sorted by length
        sl.clear();
        for (const ARow &r : items) {
            if (r.out >= 0) whole[(size_t)r.out] = r;
            else sl.push_back(r);
        }
        std::function<void(int64_t, int)> place = [&](int64_t first, int R) {
            const int64_t last = std::min<int64_t>(first + R, n_rows);
            if (first >= last) return;
            uint64_t sum = 0;
            int live = 0;
            for (int64_t i = first; i < last; ++i)
                if (whole[(size_t)i].out >= 0) { sum += (uint64_t)whole[(size_t)i].len; ++live; }
            if (live == 0) return;
            if (fits_group(R, sum) || R == min_r) {
                if (!fits_group(R, sum)) {
                    // the smallest group size and still too much (rows that fit alone, R = min_r > 1):
                    // one row per group, the other places empty
                    for (int64_t i = first; i < last; ++i)
                        if (whole[(size_t)i].out >= 0) emit_group(R, &whole[(size_t)i], 1, (uint64_t)whole[(size_t)i].len);
                    return;
                }
                emit_group(R, &whole[(size_t)first], (size_t)(last - first), sum);
                return;
            }
            place(first, R / 2);
            place(first + R / 2, R / 2);
        };
        for (int64_t first = 0; first < n_rows; first += R0) place(first, R0);
        items.swap(sl);                              // what is left for the sorted grouping: the slices
    }
    while (t < items.size()) {
        size_t remaining = items.size() - t;
        int R = max_r;
        // (the last few items take a smaller group only where that opens no launch of its own)
        auto in_use = [&](int r) {
            int q = 0;
            while ((32 >> q) != r) ++q;
            return by_key[q][0]->n_groups + by_key[q][1]->n_groups + by_key[q][2]->n_groups > 0;
        };
        while (R > min_r && remaining < (size_t)R) {
            const bool half_holds_them = (size_t)(R / 2) >= remaining;
            if (half_holds_them ? (in_use(R / 2) || !in_use(R)) : (!in_use(R) && in_use(R / 2))) R /= 2;
            else break;
        }
        for (;; R /= 2) {
            size_t n = std::min<size_t>((size_t)R, remaining);
            uint64_t sum = 0;
            for (size_t q = 0; q < n; ++q) sum += (uint64_t)items[t + q].len;
            bool take = fits_group(R, sum) || R == min_r;
            const bool cheap_visit = op == OP_DOT || op == OP_L1 || op == OP_HAMM;   // two or three instructions
            if (!take && opt.partial_groups && n == (size_t)R &&
                (op == OP_CNT || (R == 4 && !cheb) || (R == 8 && cheap_visit && opt.partial_groups == 2))) {
                // Three rows out of four per sweep of B still beat two: where R rows are too much
                // for the LDS but three quarters of them are not, the group keeps its size and
                // leaves places empty.  It pays while the idle places' arithmetic is small against
                // what a step costs anyway (the lookup, the loads): in groups of four (measured for
                // every product; not where sum() = max, whose idle place still ranks its column),
                // and at any size for the set metrics, whose visits are a byte add.
                const size_t n3 = (size_t)(R - R / 4);
                uint64_t s3 = 0;
                for (size_t q = 0; q < n3; ++q) s3 += (uint64_t)items[t + q].len;
                if (fits_group(R, s3)) { n = n3; sum = s3; take = true; }
            }
            if (take) {
                // the smallest group may have to leave places empty (longest items come first)
                while (n > 1 && !fits_group(R, sum)) sum -= (uint64_t)items[t + --n].len;
                if (!fits_group(R, sum)) return "internal: slice does not fit";
                emit_group(R, &items[t], n, sum);
                t += n;
                break;
            }
        }
    }
    // A launch of a few groups costs as much time as one of a few hundred: a small class joins
    // the class of the same R that needs more LDS, if there is one
    constexpr int kFewGroups = 32;
    for (int q = 0; q < 6; ++q)
        for (int b = 0; b < 2; ++b) {
            AClass &from = *by_key[q][b];
            if (from.n_groups == 0 || from.n_groups >= kFewGroups) continue;
            AClass *to = nullptr;
            for (int b2 = b + 1; b2 < 3 && !to; ++b2) if (by_key[q][b2]->n_groups) to = by_key[q][b2];
            if (!to) continue;
            to->rows.insert(to->rows.end(), from.rows.begin(), from.rows.end());
            to->sumlen.insert(to->sumlen.end(), from.sumlen.begin(), from.sumlen.end());
            to->n_groups += from.n_groups;
            from.rows.clear(); from.sumlen.clear(); from.n_groups = 0;
        }
    for (int q = 0; q < 6; ++q)
        for (int b = 0; b < 3; ++b)
            if (by_key[q][b]->n_groups) { finish_class(*by_key[q][b]); out.classes.push_back(std::move(*by_key[q][b])); }
    if (bloom.n_groups) { finish_class(bloom); out.classes.push_back(std::move(bloom)); }
    return std::string();
}

// ------------------------------------------------------------------------------------
// consistency check of everything the kernels index with
// ------------------------------------------------------------------------------------
std::string plan_check(const APlan &a, const BPlan &b, const int64_t *a_indptr, const int64_t *b_indptr,
                       int64_t n_cols, int metric, int op, int knn_k, const PlanOptions &opt) {
    const bool cheb = sum_is_max(metric);
    const int64_t a_nnz = a.n_rows ? a_indptr[a.n_rows] : 0;
    std::vector<int64_t> covered((size_t)a.n_rows, 0);
    std::vector<int64_t> slot_lo((size_t)a.n_partial_slots, -1), slot_hi((size_t)a.n_partial_slots, -1);
    std::vector<uint32_t> slot_flags((size_t)a.n_partial_slots, 0);
    for (const AClass &c : a.classes) {
        if (c.R != 1 && c.R != 2 && c.R != 4 && c.R != 8 && c.R != 16 && c.R != 32) return "class R";
        if (op == OP_CNT ? c.R < 4 : c.R > 16) return "class R outside the product's range";
        if (wide_sums(metric) && c.R > 8) return "two-sum product with R > 8";
        if ((op == OP_MINK || op == OP_MINK_ANY) && c.R > 4) return "Minkowski with R > 4";
        if (c.kind < KIND_STRIP || c.kind > KIND_BITMAP) return "class kind";
        if (c.kind == KIND_BLOOM && (c.R != 1 || !bloom_serves(op))) return "Bloom class outside its range";
        if (c.block != 256 && c.block != 512 && c.block != 1024 && c.block != 128 && c.block != 64) return "class block";
        if ((int64_t)c.lds_bytes + kStaticLds > opt.lds_budget) return "class LDS over budget";
        if ((size_t)c.n_groups * c.R != c.rows.size() || (size_t)c.n_groups != c.sumlen.size()) return "class sizes";
        if (c.block > scan_max_block(op, c.R, knn_k > 0)) return "class block over the kernel's bound";
        for (int g = 0; g < c.n_groups; ++g) {
            int64_t sum = 0;
            for (int r = 0; r < c.R; ++r) {
                const ARow &row = c.rows[(size_t)g * c.R + r];
                if (row.len < 0 || row.start < 0 || row.start + row.len > a_nnz) return "A slice out of range";
                if (row.out == -1) { if (row.len != 0) return "unused lane with entries"; continue; }
                sum += row.len;
                if (row.out >= 0) {
                    if (row.out >= a.n_rows) return "A output row out of range";
                    if (row.start != a_indptr[row.out] || row.start + row.len != a_indptr[row.out + 1]) return "A row range";
                    if (row.flags != (kRowFirst | kRowLast)) return "whole row without both end flags";
                    ++covered[(size_t)row.out];
                } else {
                    int slot = -2 - row.out;
                    if (slot < 0 || slot >= a.n_partial_slots) return "partial slot out of range";
                    if (slot_lo[(size_t)slot] != -1) return "partial slot used twice";
                    if (row.len < 1) return "empty slice";
                    slot_flags[(size_t)slot] = row.flags;
                    slot_lo[(size_t)slot] = row.start;
                    slot_hi[(size_t)slot] = row.start + row.len;
                }
            }
            if (sum != c.sumlen[(size_t)g]) return "group sumlen";
            if (c.hscale < 1 || c.hscale > 3) return "class hash scale";
            LdsLayout L = lds_layout(c.kind, table_words(op, c.R), (uint32_t)sum, (uint32_t)n_cols, cheb, c.hscale,
                                     knn_k > 0 ? (uint32_t)c.R : 0u);
            if (knn_k > 0 && (L.off_knn & 7u)) return "k-NN lists not 8-byte aligned";
            if (c.kind == KIND_HASH && (L.cap < 2u * (uint32_t)sum || L.cap < 16u)) return "hash table too full";
            if (L.total > c.lds_bytes) return "group LDS over the launch size";
            if (c.kind != KIND_STRIP && L.nslots > 65535u) return "slot ids over 16 bits";
            if (c.kind == KIND_BLOOM && (L.cap < kBloomMinBits || L.cap > kBloomMaxBits || (L.cap & (L.cap - 1)))) return "Bloom filter size";
        }
    }
    for (const SpilledRow &s : a.spilled) {
        if (s.row < 0 || s.row >= a.n_rows || s.n_slots < 2 || s.first_slot < 0 ||
            s.first_slot + s.n_slots > a.n_partial_slots) return "spilled row record";
        int64_t at = a_indptr[s.row];
        for (int q = 0; q < s.n_slots; ++q) {
            if (slot_lo[(size_t)(s.first_slot + q)] != at) return "spilled slices not contiguous";
            uint32_t want = (q == 0 ? kRowFirst : 0u) | (q == s.n_slots - 1 ? kRowLast : 0u);
            if (slot_flags[(size_t)(s.first_slot + q)] != want) return "spilled slice end flags";
            at = slot_hi[(size_t)(s.first_slot + q)];
        }
        if (at != a_indptr[s.row + 1]) return "spilled slices do not cover the row";
        ++covered[(size_t)s.row];
    }
    for (int64_t i = 0; i < a.n_rows; ++i)
        if (covered[(size_t)i] != 1) return fmt("A row not covered exactly once", i, covered[(size_t)i]);

    if ((size_t)b.n_slabs + 1 != b.slab_base.size() || (size_t)b.n_slabs != b.slab_steps.size()) return "B slab arrays";

    size_t lanes = (size_t)b.n_slabs * kWave;
    if (b.seg_len.size() != lanes || b.seg_row.size() != lanes || b.seg_start.size() != lanes || b.seg_glog.size() != lanes)
        return "B lane arrays";
    std::vector<int64_t> next((size_t)b.n_rows);
    std::vector<uint8_t> seen((size_t)b.n_rows, 0);
    int64_t total_entries = 0;
    for (int64_t j = 0; j < b.n_rows; ++j) next[(size_t)j] = b_indptr[j];
    for (int32_t s = 0; s < b.n_slabs; ++s) {
        int64_t sum = 0;
        int32_t mx = 0;
        for (int l = 0; l < kWave; ++l) {
            size_t at = (size_t)s * kWave + l;
            int32_t j = b.seg_row[at], len = b.seg_len[at];
            int G = 1 << b.seg_glog[at];
            if (len < 0) return "B negative segment";
            sum += len; mx = std::max(mx, len);
            if (j < 0) { if (len != 0 || j != -1) return "B unused lane"; continue; }
            if (j >= b.n_rows || G > kWave) return "B segment row";
            if (G > 1 && !b.slab_split[(size_t)s]) return "split row in an unsplit slab";
            int first = l & ~(G - 1);
            if (l == first) { if (seen[(size_t)j]) return "B row in two groups"; seen[(size_t)j] = 1; }
            else if (b.seg_row[(size_t)s * kWave + first] != j) return "B group not aligned";
            if (b.seg_start[at] != next[(size_t)j]) return "B segments not contiguous";
            next[(size_t)j] += len;
            if ((l & (G - 1)) == G - 1 && next[(size_t)j] != b_indptr[j + 1]) return "B segments do not cover the row";
        }
        mx = (mx + kScanUnroll - 1) / kScanUnroll * kScanUnroll;
        if (b.slab_base[(size_t)s + 1] - b.slab_base[(size_t)s] != (int64_t)mx * kWave || b.slab_steps[(size_t)s] != mx)
            return "B slab sizes";
        total_entries += sum;
    }
    for (int64_t j = 0; j < b.n_rows; ++j)
        if (!seen[(size_t)j] || next[(size_t)j] != b_indptr[j + 1]) return fmt("B row not covered", j);
    if (total_entries != b.nnz) return "B entries != nnz";
    for (const AClass &c : a.classes) {
        if (c.n_chunks < 1 || (size_t)c.n_chunks + 1 != c.chunk_begin.size()) return "chunk arrays";
        if (c.chunk_begin[0] != 0 || c.chunk_begin[(size_t)c.n_chunks] != b.n_slabs) return "chunk ends";
        for (int q = 0; q < c.n_chunks; ++q)
            if (c.chunk_begin[(size_t)q] > c.chunk_begin[(size_t)q + 1]) return "chunks not monotone";
        if ((int64_t)c.n_groups * c.n_chunks >= ((int64_t)1 << 31)) return "launch grid beyond 2^31 workgroups";
    }
    return std::string();
}

}  // namespace spd
