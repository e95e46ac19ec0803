/*
 * CPU oracle for all-pairs distances between the rows of two CSR matrices.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64.  It is not part of the product and
 * shares no code, header, table or helper with the HIP library: only tests, the smoke
 * check and the benchmark's CPU-baseline leg may build or call it.
 *
 * What it computes (problem statement of Section 2 of the paper: A is m x k, B is n x k,
 * the result is the dense m x n matrix of d(A_i, B_j)): for one pair of rows, both rows
 * are scattered into two zero-filled dense fp64 vectors x and y of length k, and the
 * textbook formula of the distance (Table 1, "Formula" column, read as described per
 * metric below) is evaluated by a plain loop.
 *
 *   mode 0 ("full dense")        : the loop runs over every column 0..k-1.
 *   mode 1 ("support restricted"): the loop runs over the columns where x or y holds a
 *       stored entry; the columns left out hold (0,0), where every per-column term of
 *       every formula below vanishes.  The two places where k itself enters (the means
 *       of the correlation, the 1/k of Hamming) use k explicitly.  Tests prove mode 1
 *       equal to mode 0.
 *
 * No blocking, no fusion, no expanded forms: the expanded forms of Table 1 and the
 * two-pass union of Section 3.3 are what the GPU path uses, and they are checked against
 * these definitions, not used here.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum {
    M_INNER = 0, M_COSINE, M_EUCLIDEAN, M_CORRELATION, M_JACCARD, M_DICE, M_HELLINGER,
    M_MANHATTAN, M_CHEBYSHEV, M_MINKOWSKI, M_CANBERRA, M_HAMMING, M_KL, M_JENSEN_SHANNON,
    M_RUSSELL_RAO, M_KL_STRICT, M_JACCARD_LITERAL, M_COUNT
};

static const char *const k_names[M_COUNT] = {
    "inner_product", "cosine", "euclidean", "correlation", "jaccard", "dice", "hellinger",
    "manhattan", "chebyshev", "minkowski", "canberra", "hamming", "kl_divergence",
    "jensen_shannon", "russell_rao", "kl_divergence_strict", "jaccard_literal"
};

int oracle_metric_id(const char *name) {
    for (int i = 0; i < M_COUNT; ++i)
        if (strcmp(name, k_names[i]) == 0) return i;
    return -1;
}

/* Column visited at step t: every column (cols == NULL) or the listed ones. */
#define COL(t) (cols ? (int64_t)cols[t] : (int64_t)(t))

/*
 * d(x, y) for dense fp64 vectors.  `nc` columns are visited (k of them in mode 0); the
 * columns not visited hold x = y = 0.  k is the full dimensionality.
 */
static double eval_pair(int metric, double p, const double *x, const double *y,
                        const int32_t *cols, int64_t nc, int64_t k) {
    switch (metric) {
    case M_INNER: {                      /* Table 1, "Dot Product": sum x_i y_i */
        double s = 0.0;
        for (int64_t t = 0; t < nc; ++t) { int64_t c = COL(t); s += x[c] * y[c]; }
        return s;
    }
    case M_COSINE: {
        /* Table 1, "Cosine".  The formula column prints the similarity; the distance is
         * one minus it (the expansion column starts with "1 -", and only norms to the
         * first power make it scale invariant).  A zero row has similarity 0 with
         * anything, and distance 0 to another zero row. */
        double s = 0.0, xx = 0.0, yy = 0.0;
        for (int64_t t = 0; t < nc; ++t) {
            int64_t c = COL(t);
            s += x[c] * y[c]; xx += x[c] * x[c]; yy += y[c] * y[c];
        }
        if (xx == 0.0 && yy == 0.0) return 0.0;
        if (xx == 0.0 || yy == 0.0) return 1.0;
        return 1.0 - s / (sqrt(xx) * sqrt(yy));
    }
    case M_EUCLIDEAN: {                  /* Table 1, "Euclidean", formula column */
        double s = 0.0;
        for (int64_t t = 0; t < nc; ++t) { int64_t c = COL(t); double d = x[c] - y[c]; s += d * d; }
        return sqrt(s);
    }
    case M_CORRELATION: {
        /* Table 1, "Correlation": one minus the Pearson correlation, means taken over
         * all k columns.  A row without variance has no correlation: distance 1. */
        double sx = 0.0, sy = 0.0;
        for (int64_t t = 0; t < nc; ++t) { int64_t c = COL(t); sx += x[c]; sy += y[c]; }
        double mx = sx / (double)k, my = sy / (double)k;
        double num = 0.0, vx = 0.0, vy = 0.0;
        for (int64_t t = 0; t < nc; ++t) {
            int64_t c = COL(t);
            double dx = x[c] - mx, dy = y[c] - my;
            num += dx * dy; vx += dx * dx; vy += dy * dy;
        }
        /* the k - nc columns not visited hold (0, 0): their centred values are -mx, -my */
        double rest = (double)(k - nc);
        num += rest * mx * my; vx += rest * mx * mx; vy += rest * my * my;
        if (vx <= 0.0 || vy <= 0.0) return 1.0;
        return 1.0 - num / (sqrt(vx) * sqrt(vy));
    }
    case M_JACCARD: {
        /* Table 1, "Jaccard", read on the supports (norm column L0):
         * 1 - |sx & sy| / |sx | sy|; two empty rows are at distance 0. */
        double both = 0.0, any = 0.0;
        for (int64_t t = 0; t < nc; ++t) {
            int64_t c = COL(t);
            int a = x[c] != 0.0, b = y[c] != 0.0;
            both += (double)(a && b); any += (double)(a || b);
        }
        if (any == 0.0) return 0.0;
        return 1.0 - both / any;
    }
    case M_DICE: {
        /* Table 1, "Dice-Sorensen" (norm column L0), as a distance:
         * 1 - 2|sx & sy| / (|sx| + |sy|); two empty rows are at distance 0. */
        double both = 0.0, nx = 0.0, ny = 0.0;
        for (int64_t t = 0; t < nc; ++t) {
            int64_t c = COL(t);
            int a = x[c] != 0.0, b = y[c] != 0.0;
            both += (double)(a && b); nx += (double)a; ny += (double)b;
        }
        if (nx + ny == 0.0) return 0.0;
        return 1.0 - 2.0 * both / (nx + ny);
    }
    case M_HELLINGER: {                  /* Table 1, "Hellinger", formula column; x, y >= 0 */
        double s = 0.0;
        for (int64_t t = 0; t < nc; ++t) {
            int64_t c = COL(t);
            double d = sqrt(x[c]) - sqrt(y[c]);
            s += d * d;
        }
        return sqrt(s) / sqrt(2.0);
    }
    case M_MANHATTAN: {                  /* Table 1, "Manhattan"; appendix worked example */
        double s = 0.0;
        for (int64_t t = 0; t < nc; ++t) { int64_t c = COL(t); s += fabs(x[c] - y[c]); }
        return s;
    }
    case M_CHEBYSHEV: {                  /* Section 2.1: Minkowski "with degree max" */
        double s = 0.0;
        for (int64_t t = 0; t < nc; ++t) { int64_t c = COL(t); double d = fabs(x[c] - y[c]); if (d > s) s = d; }
        return s;
    }
    case M_MINKOWSKI: {                  /* Table 1, "Minkowski" */
        double s = 0.0;
        for (int64_t t = 0; t < nc; ++t) { int64_t c = COL(t); s += pow(fabs(x[c] - y[c]), p); }
        return pow(s, 1.0 / p);
    }
    case M_CANBERRA: {                   /* Table 1, "Canberra"; a (0,0) column adds 0 */
        double s = 0.0;
        for (int64_t t = 0; t < nc; ++t) {
            int64_t c = COL(t);
            double den = fabs(x[c]) + fabs(y[c]);
            if (den != 0.0) s += fabs(x[c] - y[c]) / den;
        }
        return s;
    }
    case M_HAMMING: {                    /* Table 1, "Hamming": mismatching columns over k */
        double s = 0.0;
        for (int64_t t = 0; t < nc; ++t) { int64_t c = COL(t); s += (double)(x[c] != y[c]); }
        return s / (double)k;
    }
    case M_KL: {
        /* Table 1, "KL-Divergence", with the product a log(a/b) applied where both
         * entries are present (Section 2.2: the product replaces the multiplication of
         * the dot-product semiring, so a column missing on either side adds nothing). */
        double s = 0.0;
        for (int64_t t = 0; t < nc; ++t) {
            int64_t c = COL(t);
            if (x[c] > 0.0 && y[c] > 0.0) s += x[c] * log(x[c] / y[c]);
        }
        return s;
    }
    case M_JENSEN_SHANNON: {             /* Table 1, "Jensen-Shannon"; 0 log 0 = 0 */
        double s = 0.0;
        for (int64_t t = 0; t < nc; ++t) {
            int64_t c = COL(t);
            double mu = 0.5 * (x[c] + y[c]);
            if (x[c] > 0.0) s += x[c] * log(x[c] / mu);
            if (y[c] > 0.0) s += y[c] * log(y[c] / mu);
        }
        if (s < 0.0) s = 0.0;
        return sqrt(0.5 * s);
    }
    case M_RUSSELL_RAO: {                /* Table 1, "Russel-Rao", on the supports */
        double both = 0.0;
        for (int64_t t = 0; t < nc; ++t) {
            int64_t c = COL(t);
            both += (double)(x[c] != 0.0 && y[c] != 0.0);
        }
        return ((double)k - both) / (double)k;
    }
    case M_KL_STRICT: {
        /* The textbook KL divergence, sum x log(x/y) with 0 log 0 = 0: infinite as soon as
         * x holds mass in a column where y holds none (the variant Section 2.2's product,
         * which only sees columns present on both sides, leaves out). */
        double s = 0.0;
        for (int64_t t = 0; t < nc; ++t) {
            int64_t c = COL(t);
            if (x[c] > 0.0) {
                if (!(y[c] > 0.0)) return INFINITY;
                s += x[c] * log(x[c] / y[c]);
            }
        }
        return s;
    }
    case M_JACCARD_LITERAL: {
        /* Table 1, "Jaccard", expansion column taken literally: the dot product of the
         * stored values over (|x|_0 + |y|_0 - dot), as a distance; 0 where that denominator
         * vanishes (two empty rows).  Equal to the set reading on 0/1 data. */
        double dot = 0.0, nx = 0.0, ny = 0.0;
        for (int64_t t = 0; t < nc; ++t) {
            int64_t c = COL(t);
            dot += x[c] * y[c]; nx += (double)(x[c] != 0.0); ny += (double)(y[c] != 0.0);
        }
        double den = nx + ny - dot;
        if (den == 0.0) return 0.0;
        return 1.0 - dot / den;
    }
    default:
        return NAN;
    }
}

/*
 * A semiring product between two rows (Section 2.2; the tropical semiring of Eq. 1 is one
 * instance): result = sum()-fold of product(x_c, y_c) over the columns c of the domain,
 *   domain = columns stored (non-zero) in BOTH rows when the product annihilates on 0,
 *   domain = columns stored in EITHER row, the missing side read as 0, for a
 *            non-annihilating product (the NAMM of Section 2.2, Eq. 2);
 * an empty domain gives the identity of sum(): 0 for +, +infinity for min, -infinity for max.
 * Every distance of Table 1 is such a fold with a transform of the stored values in front of it
 * and an epilogue after it (Section 2.2 for the products, Table 1's "Expansion" column and
 * Section 3.4 for the epilogues of the dot-product family; the C++ interface shown in Section 4.2
 * passes the product and the sum as functors to one primitive): the transforms and epilogues are
 * spelled out here, each from its definition, so that the composition can be checked against the
 * plain formulas of eval_pair above.
 */
enum {
    P_TIMES = 0, P_PLUS, P_MIN, P_MAX, P_ABS_DIFF, P_SQ_DIFF,
    P_ABS_DIFF_POW,      /* |a - b|^p                                  (Table 1, Minkowski)      */
    P_CANBERRA,          /* |a - b| / (|a| + |b|), 0 at (0, 0)         (Table 1, Canberra)       */
    P_NOT_EQUAL,         /* 1 where a != b, else 0                     (Table 1, Hamming)        */
    P_X_LOG_X_OVER_Y,    /* a log(a / b) where both are positive       (Table 1, KL; Section 2.2)*/
    P_JS_TERM,           /* a log(a/mu) + b log(b/mu), mu = (a + b)/2, 0 log 0 = 0 (Jensen-Shannon) */
    P_COUNT
};
enum { S_PLUS = 0, S_MIN, S_MAX, S_COUNT };
/* applied to every stored value before anything else (Table 1: Hellinger works on square roots,
 * the set distances on the supports) */
enum { T_NONE = 0, T_SQRT, T_NONZERO, T_COUNT };
/* what turns the folded value v into the distance: Table 1's "Expansion" column for the
 * dot-product family (norms of the transformed rows x, y over k columns), the closing steps
 * of the others */
enum {
    E_NONE = 0,
    E_ROOT_P,            /* v^(1/p)                                                  */
    E_DIV_K,             /* v / k                                                    */
    E_SQRT_HALF,         /* sqrt(v / 2)                                              */
    E_COSINE,            /* 1 - v / (|x|_2 |y|_2); 1 if one row is zero, 0 if both   */
    E_L2,                /* sqrt(|x|_2^2 - 2 v + |y|_2^2)                            */
    E_CORRELATION,       /* 1 - (k v - sum x sum y) / sqrt((k sum x^2 - (sum x)^2)(k sum y^2 - (sum y)^2)); 1 without variance */
    E_JACCARD,           /* 1 - v / (|x|_0 + |y|_0 - v); 0 where the denominator is 0 */
    E_DICE,              /* 1 - 2 v / (|x|_0 + |y|_0); 0 if both rows are empty       */
    E_HELLINGER,         /* sqrt((|x|_2^2 + |y|_2^2) / 2 - v)                         */
    E_RUSSELL_RAO,       /* (k - v) / k                                               */
    E_STRICT,            /* v if y is positive wherever x is, else +infinity          */
    E_COUNT
};

typedef struct { int product, sum, over_union; double p; int transform, epilogue; } semiring_t;

static double semiring_transform(int transform, double v) {
    if (transform == T_SQRT) return sqrt(v);
    if (transform == T_NONZERO) return v != 0.0 ? 1.0 : 0.0;
    return v;
}

static double semiring_product(int product, double p, double a, double b) {
    switch (product) {
    case P_TIMES: return a * b;
    case P_PLUS: return a + b;
    case P_MIN: return a < b ? a : b;
    case P_MAX: return a > b ? a : b;
    case P_ABS_DIFF: return fabs(a - b);
    case P_SQ_DIFF: return (a - b) * (a - b);
    case P_ABS_DIFF_POW: return pow(fabs(a - b), p);
    case P_CANBERRA: { double den = fabs(a) + fabs(b); return den != 0.0 ? fabs(a - b) / den : 0.0; }
    case P_NOT_EQUAL: return a != b ? 1.0 : 0.0;
    case P_X_LOG_X_OVER_Y: return (a > 0.0 && b > 0.0) ? a * log(a / b) : 0.0;
    case P_JS_TERM: {
        double mu = 0.5 * (a + b), s = 0.0;
        if (a > 0.0) s += a * log(a / mu);
        if (b > 0.0) s += b * log(b / mu);
        return s;
    }
    default: return NAN;
    }
}

/* The columns not visited hold (0, 0): no product and no norm below gets anything from them,
 * and the places where k itself enters use k. */
static double eval_semiring(const semiring_t *sr, const double *x, const double *y,
                            const int32_t *cols, int64_t nc, int64_t k) {
    double acc = sr->sum == S_PLUS ? 0.0 : (sr->sum == S_MIN ? INFINITY : -INFINITY);
    double sx = 0.0, sy = 0.0, sxx = 0.0, syy = 0.0, n0x = 0.0, n0y = 0.0;
    int covered = 1;
    for (int64_t t = 0; t < nc; ++t) {
        int64_t c = COL(t);
        double u = semiring_transform(sr->transform, x[c]), v = semiring_transform(sr->transform, y[c]);
        sx += u; sy += v; sxx += u * u; syy += v * v;
        n0x += (double)(u != 0.0); n0y += (double)(v != 0.0);
        if (u > 0.0 && !(v > 0.0)) covered = 0;
        int in_x = u != 0.0, in_y = v != 0.0;
        int in_domain = sr->over_union ? (in_x || in_y) : (in_x && in_y);
        if (!in_domain) continue;
        double w = semiring_product(sr->product, sr->p, u, v);
        if (sr->sum == S_PLUS) acc += w;
        else if (sr->sum == S_MIN) { if (w < acc) acc = w; }
        else { if (w > acc) acc = w; }
    }
    double kk = (double)k;
    switch (sr->epilogue) {
    case E_NONE: return acc;
    case E_ROOT_P: return pow(acc, 1.0 / sr->p);
    case E_DIV_K: return acc / kk;
    case E_SQRT_HALF: return sqrt(0.5 * (acc > 0.0 ? acc : 0.0));
    case E_COSINE:
        if (sxx == 0.0 && syy == 0.0) return 0.0;
        if (sxx == 0.0 || syy == 0.0) return 1.0;
        return 1.0 - acc / (sqrt(sxx) * sqrt(syy));
    case E_L2: { double r = sxx - 2.0 * acc + syy; return sqrt(r > 0.0 ? r : 0.0); }
    case E_CORRELATION: {
        double vx = kk * sxx - sx * sx, vy = kk * syy - sy * sy;
        if (vx <= 0.0 || vy <= 0.0) return 1.0;
        return 1.0 - (kk * acc - sx * sy) / (sqrt(vx) * sqrt(vy));
    }
    case E_JACCARD: { double den = n0x + n0y - acc; return den == 0.0 ? 0.0 : 1.0 - acc / den; }
    case E_DICE: return (n0x + n0y == 0.0) ? 0.0 : 1.0 - 2.0 * acc / (n0x + n0y);
    case E_HELLINGER: { double r = 0.5 * (sxx + syy) - acc; return sqrt(r > 0.0 ? r : 0.0); }
    case E_RUSSELL_RAO: return (kk - acc) / kk;
    case E_STRICT: return covered ? acc : INFINITY;
    default: return NAN;
    }
}

typedef struct {
    int64_t n_rows, n_cols;
    const int64_t *indptr;
    const int32_t *indices;
    const float *values;
} csr_t;

/*
 * out[a * n_sel_b + b] = d(A[sel_a[a]], B[sel_b[b]]), fp64.
 * sel_a / sel_b may be NULL (all rows in order).  mode: 0 full dense, 1 support restricted.
 * n_threads <= 0: all hardware threads.  Returns the number of threads used, <0 on error.
 */
static int run_pairs(int64_t a_rows, int64_t n_cols, const int64_t *a_indptr, const int32_t *a_indices,
                     const float *a_values, int64_t b_rows, const int64_t *b_indptr,
                     const int32_t *b_indices, const float *b_values, int metric, double p,
                     const semiring_t *sr, const int64_t *sel_a, int64_t n_sel_a, const int64_t *sel_b,
                     int64_t n_sel_b, int mode, int n_threads, double *out) {
    if (!sel_a) n_sel_a = a_rows;
    if (!sel_b) n_sel_b = b_rows;
    int used = 1;
#ifdef _OPENMP
    if (n_threads <= 0) n_threads = omp_get_max_threads();
    used = n_threads;
#else
    n_threads = 1;
#endif
    int failed = 0;
#pragma omp parallel num_threads(n_threads)
    {
        double *x = (double *)calloc((size_t)n_cols + 1, sizeof(double));
        double *y = (double *)calloc((size_t)n_cols + 1, sizeof(double));
        unsigned char *seen = (unsigned char *)calloc((size_t)n_cols + 1, 1);
        int32_t *cols = NULL;
        if (!x || !y || !seen) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(dynamic, 1)
            for (int64_t ia = 0; ia < n_sel_a; ++ia) {
                int64_t i = sel_a ? sel_a[ia] : ia;
                int64_t a0 = a_indptr[i], a1 = a_indptr[i + 1];
                for (int64_t q = a0; q < a1; ++q) x[a_indices[q]] = (double)a_values[q];
                for (int64_t jb = 0; jb < n_sel_b; ++jb) {
                    int64_t j = sel_b ? sel_b[jb] : jb;
                    int64_t b0 = b_indptr[j], b1 = b_indptr[j + 1];
                    for (int64_t q = b0; q < b1; ++q) y[b_indices[q]] = (double)b_values[q];
                    double d;
                    if (mode == 0) {
                        d = sr ? eval_semiring(sr, x, y, NULL, n_cols, n_cols)
                               : eval_pair(metric, p, x, y, NULL, n_cols, n_cols);
                    } else {
                        int64_t cap = (a1 - a0) + (b1 - b0), nc = 0;
                        cols = (int32_t *)realloc(cols, (size_t)(cap > 0 ? cap : 1) * sizeof(int32_t));
                        for (int64_t q = a0; q < a1; ++q) {
                            int32_t c = a_indices[q];
                            if (!seen[c]) { seen[c] = 1; cols[nc++] = c; }
                        }
                        for (int64_t q = b0; q < b1; ++q) {
                            int32_t c = b_indices[q];
                            if (!seen[c]) { seen[c] = 1; cols[nc++] = c; }
                        }
                        d = sr ? eval_semiring(sr, x, y, cols, nc, n_cols) : eval_pair(metric, p, x, y, cols, nc, n_cols);
                        for (int64_t t = 0; t < nc; ++t) seen[cols[t]] = 0;
                    }
                    out[ia * n_sel_b + jb] = d;
                    for (int64_t q = b0; q < b1; ++q) y[b_indices[q]] = 0.0;
                }
                for (int64_t q = a0; q < a1; ++q) x[a_indices[q]] = 0.0;
            }
        }
        free(x); free(y); free(seen); free(cols);
    }
    return failed ? -2 : used;
}

int oracle_pairwise(int64_t a_rows, int64_t n_cols, const int64_t *a_indptr, const int32_t *a_indices,
                    const float *a_values, int64_t b_rows, const int64_t *b_indptr,
                    const int32_t *b_indices, const float *b_values, int metric, double p,
                    const int64_t *sel_a, int64_t n_sel_a, const int64_t *sel_b, int64_t n_sel_b,
                    int mode, int n_threads, double *out) {
    if (metric < 0 || metric >= M_COUNT) return -1;
    return run_pairs(a_rows, n_cols, a_indptr, a_indices, a_values, b_rows, b_indptr, b_indices, b_values,
                     metric, p, NULL, sel_a, n_sel_a, sel_b, n_sel_b, mode, n_threads, out);
}

/* The same for a semiring: out[a * n_sel_b + b] = epilogue of the sum()-fold of product() over
 * the domain, on the transformed values. */
int oracle_semiring_pairwise(int64_t a_rows, int64_t n_cols, const int64_t *a_indptr, const int32_t *a_indices,
                             const float *a_values, int64_t b_rows, const int64_t *b_indptr,
                             const int32_t *b_indices, const float *b_values, int product, int sum,
                             int over_union, double p, int transform, int epilogue, const int64_t *sel_a,
                             int64_t n_sel_a, const int64_t *sel_b, int64_t n_sel_b, int mode, int n_threads,
                             double *out) {
    if (product < 0 || product >= P_COUNT || sum < 0 || sum >= S_COUNT) return -1;
    if (transform < 0 || transform >= T_COUNT || epilogue < 0 || epilogue >= E_COUNT) return -1;
    semiring_t sr = {product, sum, over_union != 0, p, transform, epilogue};
    return run_pairs(a_rows, n_cols, a_indptr, a_indices, a_values, b_rows, b_indptr, b_indices, b_values,
                     0, 0.0, &sr, sel_a, n_sel_a, sel_b, n_sel_b, mode, n_threads, out);
}

int oracle_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
