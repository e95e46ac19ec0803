// Host-only driver for tests/test_planner_sanitized.py: random row-pointer arrays and sparse
// rows through the planner and the per-pair host arithmetic of the library, built with the
// address and undefined-behaviour sanitizers.  Any report of theirs ends the process with a
// non-zero status; a plan that fails its own consistency check is printed and counted.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <random>
#include <string>
#include <vector>

#include "spd_testing.h"

namespace {

std::vector<int64_t> row_pointers(std::mt19937_64 &rng, int64_t n_rows, int64_t n_cols, int law) {
    std::vector<int64_t> ip((size_t)n_rows + 1, 0);
    std::uniform_real_distribution<double> u(0.0, 1.0);
    for (int64_t i = 0; i < n_rows; ++i) {
        int64_t len = 0;
        switch (law) {
        case 0: len = (int64_t)(u(rng) * 8.0); break;                                        // short, some empty
        case 1: len = (int64_t)std::min<double>((double)n_cols, 1.0 / std::pow(1.0 - u(rng) + 1e-9, 1.2)); break;  // heavy tail
        case 2: len = (u(rng) < 0.01) ? n_cols : 1; break;                                   // a few full rows
        case 3: len = (int64_t)(u(rng) * (double)std::min<int64_t>(n_cols, 700)); break;     // medium, around the split length
        default: len = 0; break;                                                             // all empty
        }
        ip[(size_t)i + 1] = ip[(size_t)i] + std::min(len, n_cols);
    }
    return ip;
}

}  // namespace

int main(int argc, char **argv) {
    const int rounds = argc > 1 ? std::atoi(argv[1]) : 200;
    std::mt19937_64 rng(20210406357ull);
    std::vector<char> json(1 << 16);
    int refused = 0, planned = 0, bad = 0;
    const int64_t col_choices[] = {1, 7, 64, 513, 4096, 20000, 70000, 1 << 20};
    const int64_t row_choices[] = {0, 1, 2, 63, 64, 65, 1000, 5000};
    for (int it = 0; it < rounds; ++it) {
        const int64_t n_cols = col_choices[rng() % 8];
        const int64_t a_rows = row_choices[rng() % 8], b_rows = row_choices[rng() % 8];
        std::vector<int64_t> a = row_pointers(rng, a_rows, n_cols, (int)(rng() % 5));
        std::vector<int64_t> b = row_pointers(rng, b_rows, n_cols, (int)(rng() % 5));
        const spd_metric metric = (spd_metric)(rng() % SPD_METRIC_COUNT);
        int k = (rng() % 3 == 0 && b_rows > 0) ? (int)std::min<int64_t>(b_rows, 1 + (int64_t)(rng() % 64)) : 0;
        std::vector<const char *> names;
        std::vector<int64_t> values;
        if (rng() % 2) { names.push_back("force_kind"); values.push_back((int64_t)(rng() % 5)); }
        if (rng() % 3 == 0) { names.push_back("lds_budget"); values.push_back(8192 + (int64_t)(rng() % 150000)); }
        if (rng() % 3 == 0) { names.push_back("max_rows"); values.push_back(1 << (rng() % 6)); }
        if (rng() % 3 == 0) { names.push_back("split_len"); values.push_back(2 + (int64_t)(rng() % 600)); }
        if (rng() % 3 == 0) { names.push_back("window"); values.push_back(64 << (rng() % 8)); }
        if (rng() % 3 == 0) { names.push_back("chunks"); values.push_back((int64_t)(rng() % 9)); }
        if (rng() % 4 == 0) { names.push_back("n_cus"); values.push_back(1 + (int64_t)(rng() % 300)); }
        if (rng() % 4 == 0) { names.push_back("bloom_long_rows"); values.push_back((int64_t)(rng() % 2)); }
        if (rng() % 4 == 0) { names.push_back("sort_slack"); values.push_back((int64_t)(rng() % 2)); }
        if (rng() % 3 == 0) { names.push_back("partial_groups"); values.push_back((int64_t)(rng() % 3)); }
        if (rng() % 3 == 0) { names.push_back("consecutive_groups"); values.push_back((int64_t)(rng() % 2)); }
        spd_status st = spd_host_plan_summary(a.data(), a_rows, b.data(), b_rows, n_cols, metric, k, names.data(),
                                              values.data(), (int)names.size(), json.data(), json.size());
        if (st == SPD_OK) {
            ++planned;
        } else if (std::strstr(json.data(), "\"error\"")) {
            // a refusal with a reason (a forced kind that cannot hold the rows, a budget too small):
            // fine; a plan that was made and then failed its own check is not
            const char *inconsistent[] = {"chunk", "slab", "group", "class R", "class block", "rows of A", "merge area"};
            bool broken = false;
            for (const char *w : inconsistent) broken = broken || std::strstr(json.data(), w) != nullptr;
            if (broken) { ++bad; std::printf("case %d: %s\n", it, json.data()); }
            ++refused;
        } else {
            ++refused;
        }
    }
    // the per-pair arithmetic on rows with repeated, extreme and zero values
    int pairs = 0;
    std::uniform_real_distribution<double> u(0.0, 1.0);
    for (int it = 0; it < rounds; ++it) {
        const int64_t n_cols = 1 + (int64_t)(rng() % 300);
        auto row = [&](std::vector<int32_t> &c, std::vector<float> &v) {
            for (int64_t j = 0; j < n_cols; ++j)
                if (u(rng) < 0.3) {
                    c.push_back((int32_t)j);
                    const int kind = (int)(rng() % 6);
                    v.push_back(kind == 0 ? 0.0f : kind == 1 ? 1e-30f : kind == 2 ? 3e18f : (float)(u(rng) * 10.0));
                }
        };
        std::vector<int32_t> ac, bc;
        std::vector<float> av, bv;
        row(ac, av);
        row(bc, bv);
        for (int m = 0; m < SPD_METRIC_COUNT; ++m) {
            float out = 0.0f;
            const float p = (m == SPD_MINKOWSKI) ? (float)(0.25 + u(rng) * 6.0) : 2.0f;
            spd_status st = spd_host_pair_value((spd_metric)m, p, n_cols, ac.data(), av.data(), (int64_t)ac.size(),
                                                bc.data(), bv.data(), (int64_t)bc.size(), &out);
            if (st != SPD_OK) { ++bad; std::printf("pair case %d metric %d: status %d\n", it, m, (int)st); }
            ++pairs;
        }
    }
    std::printf("planned %d refused %d inconsistent %d pairs %d\n", planned, refused, bad, pairs);
    return bad ? 1 : 0;
}
