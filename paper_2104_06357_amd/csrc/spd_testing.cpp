// Host-only test hooks (include/spd_testing.h).  No GPU call is made here, and nothing
// here is reachable from spd_pairwise / spd_knn.
#include "../../include/spd_testing.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "spd_ops.h"
#include "spd_plan.h"

using namespace spd;

namespace {

template <int OP>
void pair_sums(const OpParams &q, int transform, const int32_t *a_cols, const float *a_vals, int64_t a_len,
               const int32_t *b_cols, const float *b_vals, int64_t b_len, double &v0, double &v1, double &v2) {
    typename Op<OP>::Acc acc;
    Op<OP>::init(acc);
    for (int64_t t = 0; t < b_len; ++t) {
        const int32_t *hit = std::lower_bound(a_cols, a_cols + a_len, b_cols[t]);
        float a = 0.0f;
        if (hit != a_cols + a_len && *hit == b_cols[t]) a = transform_value(transform, a_vals[hit - a_cols]);
        typename Op<OP>::Bv bv = Op<OP>::prep(transform_value(transform, b_vals[t]), q);
        Op<OP>::visit(acc, a, bv, q);
    }
    v0 = Op<OP>::v0(acc);
    v1 = Op<OP>::v1(acc);
    v2 = Op<OP>::v2(acc);
}

}  // namespace

extern "C" {

spd_status spd_host_pair_value(spd_metric metric, float p, int64_t n_cols, const int32_t *a_cols,
                               const float *a_vals, int64_t a_len, const int32_t *b_cols, const float *b_vals,
                               int64_t b_len, float *out) {
    if (!out || (a_len > 0 && (!a_cols || !a_vals)) || (b_len > 0 && (!b_cols || !b_vals))) return SPD_ERR_NULL;
    if ((int)metric < 0 || (int)metric >= SPD_METRIC_COUNT) return SPD_ERR_BAD_METRIC;
    if (metric == SPD_MINKOWSKI && !(p > 0.0f && std::isfinite(p))) return SPD_ERR_BAD_P;
    if (a_len < 0 || b_len < 0 || n_cols < 0) return SPD_ERR_DIM_MISMATCH;
    const MetricInfo mi = metric_info((int)metric);
    OpParams q;
    q.p = metric == SPD_MINKOWSKI ? p : (metric == SPD_L2_UNEXPANDED ? 2.0f : 1.0f);
    q.inv_p = 1.0f / q.p;
    q.k = (double)n_cols;
    q.metric = (int)metric;
    double ra0 = 0, ra1 = 0, rb0 = 0, rb1 = 0;
    for (int64_t t = 0; t < a_len; ++t) norm_accumulate(mi.norm, transform_value(mi.transform, a_vals[t]), q.p, ra0, ra1);
    for (int64_t t = 0; t < b_len; ++t) norm_accumulate(mi.norm, transform_value(mi.transform, b_vals[t]), q.p, rb0, rb1);
    double a0, a1, b0, b1;
    norm_derive(q.metric, q.k, ra0, ra1, a0, a1);
    norm_derive(q.metric, q.k, rb0, rb1, b0, b1);
    double v0 = 0, v1 = 0, v2 = 0;
    switch (mi.op) {
    case OP_DOT:  pair_sums<OP_DOT>(q, mi.transform, a_cols, a_vals, a_len, b_cols, b_vals, b_len, v0, v1, v2); break;
    case OP_CNT:  pair_sums<OP_CNT>(q, mi.transform, a_cols, a_vals, a_len, b_cols, b_vals, b_len, v0, v1, v2); break;
    case OP_L1:   pair_sums<OP_L1>(q, mi.transform, a_cols, a_vals, a_len, b_cols, b_vals, b_len, v0, v1, v2); break;
    case OP_MINK: pair_sums<OP_MINK>(q, mi.transform, a_cols, a_vals, a_len, b_cols, b_vals, b_len, v0, v1, v2); break;
    case OP_CANB: pair_sums<OP_CANB>(q, mi.transform, a_cols, a_vals, a_len, b_cols, b_vals, b_len, v0, v1, v2); break;
    case OP_HAMM: pair_sums<OP_HAMM>(q, mi.transform, a_cols, a_vals, a_len, b_cols, b_vals, b_len, v0, v1, v2); break;
    case OP_KL:   pair_sums<OP_KL>(q, mi.transform, a_cols, a_vals, a_len, b_cols, b_vals, b_len, v0, v1, v2); break;
    case OP_JS:   pair_sums<OP_JS>(q, mi.transform, a_cols, a_vals, a_len, b_cols, b_vals, b_len, v0, v1, v2); break;
    case OP_CHEB: {
        pair_sums<OP_CHEB>(q, mi.transform, a_cols, a_vals, a_len, b_cols, b_vals, b_len, v0, v1, v2);
        // the entries of `a` that `b` does not store: the kernel takes the largest of them
        for (int64_t t = 0; t < a_len; ++t)
            if (!std::binary_search(b_cols, b_cols + b_len, a_cols[t])) v0 = std::max(v0, (double)std::fabs(a_vals[t]));
        break;
    }
    default: return SPD_ERR_BAD_METRIC;
    }
    *out = finish(q, v0, v1, v2, a0, a1, b0, b1);
    return SPD_OK;
}

spd_status spd_host_plan_summary(const int64_t *a_indptr, int64_t a_rows, const int64_t *b_indptr, int64_t b_rows,
                                 int64_t n_cols, spd_metric metric, int k_neighbors, const char *const *option_names,
                                 const int64_t *option_values, int n_options, char *json, size_t cap) {
    if (!a_indptr || !b_indptr || !json || cap == 0) return SPD_ERR_NULL;
    json[0] = 0;
    if ((int)metric < 0 || (int)metric >= SPD_METRIC_COUNT) return SPD_ERR_BAD_METRIC;
    PlanOptions opt;
    for (int i = 0; i < n_options; ++i) {
        std::string s(option_names[i]);
        int64_t v = option_values[i];
        if (s == "lds_budget") opt.lds_budget = v;
        else if (s == "force_kind") opt.force_kind = (int)v;
        else if (s == "max_rows") opt.max_rows = (int)v;
        else if (s == "split_len") opt.split_len = (int)v;
        else if (s == "window") opt.window = (int)v;
        else if (s == "chunks") opt.chunks = (int)v;
        else if (s == "n_cus") opt.n_cus = (int)v;
        else if (s == "bloom_long_rows") opt.bloom_long_rows = (int)v;
        else if (s == "sort_slack") opt.sort_slack = (int)v;
        else if (s == "partial_groups") opt.partial_groups = (int)v;
        else if (s == "consecutive_groups") opt.consecutive_groups = (int)v;
        else if (s == "chunk_scale") opt.chunk_scale = (int)v;
        else return SPD_ERR_UNSUPPORTED;
    }
    APlan ap;
    BPlan bp;
    std::string why = plan_b(b_indptr, b_rows, opt, bp);
    int op = metric_info((int)metric).op;
    if (op == OP_CNT && opt.force_kind == KIND_BLOOM) op = OP_DOT;      // as the library does
    // (the planner hook has no degree: it plans Minkowski for the small integer degrees)
    if (why.empty()) why = plan_a(a_indptr, a_rows, n_cols, (int)metric, op, k_neighbors, opt, ap);
    if (why.empty()) {
        PlanOptions opt_c = opt;
        opt_c.chunk_scale = chunk_scale_for(opt, k_neighbors > 0);
        for (AClass &c : ap.classes) plan_chunks(bp, c, opt_c);
        why = plan_check(ap, bp, a_indptr, b_indptr, n_cols, (int)metric, op, k_neighbors, opt);
    }
    std::string js = "{";
    if (!why.empty()) {
        js += "\"error\": \"" + why + "\"}";
        std::snprintf(json, cap, "%s", js.c_str());
        return SPD_ERR_UNSUPPORTED;
    }
    js += "\"classes\": [";
    for (size_t i = 0; i < ap.classes.size(); ++i) {
        const AClass &c = ap.classes[i];
        int64_t max_sum = 0;
        for (int32_t s : c.sumlen) max_sum = std::max<int64_t>(max_sum, s);
        char buf[320];
        std::snprintf(buf, sizeof buf,
                      "%s{\"R\": %d, \"kind\": %d, \"block\": %d, \"lds_bytes\": %u, \"groups\": %d, \"max_sumlen\": %lld, "
                      "\"chunks\": %d, \"cost\": %.1f, \"hscale\": %d}",
                      i ? ", " : "", c.R, c.kind, c.block, c.lds_bytes, c.n_groups, (long long)max_sum, c.n_chunks, c.cost,
                      c.hscale);
        js += buf;
    }
    int64_t split_rows = 0, max_steps = 0, total_steps = 0;
    for (size_t l = 0; l < bp.seg_glog.size(); ++l)
        if (bp.seg_glog[l] && (l & ((1u << bp.seg_glog[l]) - 1)) == 0) ++split_rows;
    for (int32_t s : bp.slab_steps) { max_steps = std::max<int64_t>(max_steps, s); total_steps += s; }
    char buf[512];
    std::snprintf(buf, sizeof buf,
                  "], \"spilled_rows\": %zu, \"partial_slots\": %d, \"slabs\": %d, \"split_rows\": %lld, "
                  "\"max_slab_steps\": %lld, \"total_slab_steps\": %lld, \"packed_entries\": %lld}",
                  ap.spilled.size(), ap.n_partial_slots, bp.n_slabs, (long long)split_rows, (long long)max_steps,
                  (long long)total_steps, (long long)bp.nnz);
    js += buf;
    std::snprintf(json, cap, "%s", js.c_str());
    return js.size() < cap ? SPD_OK : SPD_ERR_WORKSPACE;
}

}  // extern "C"
