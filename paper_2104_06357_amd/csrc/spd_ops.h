// Per-visit products, row norms and expansion functions of the distances of Table 1,
// in the single-pass form the kernels use.
//
// Every distance is evaluated as
//     d(x, y) = finish( sum over the stored entries b_c of y of  g(x_c, b_c),  N(x), N(y) )
// where x_c is 0 when column c is not stored in x, and g(0, b) = 0 for every product, so
// that only columns present in both rows contribute:
//   * dot-product family (Section 3.4): g = x*y on transformed values, N = row norms,
//     finish = the expansion function.
//   * union family (Section 2.2, Eq. 2): with f the non-annihilating product,
//     sum over the union of f = F(x) + F(y) + sum over the intersection of
//     [ f(x_c,y_c) - f(x_c,0) - f(0,y_c) ], F(x) = sum_c f(x_c, 0).  This covers the three
//     parts of Eq. 2 in one sweep over y instead of the two passes of Section 3.3.
//   * Chebyshev (sum() = max) keeps max |x_c - y_c| over the entries of y; the part of x
//     that y does not store is completed by the kernel from x's largest entries.
//   * semirings built from a menu of product() and sum() (Section 2.2; Eq. 1 is (min, +)):
//     sum() = + works like the union family with product(., 0) in the place of the row norm,
//     sum() = min / max like Chebyshev, with x's entries ranked by product(x_c, 0).
// Sums are carried in fp64 so the cancellations of the expanded forms (Section 2.1) stay
// far below the fp32 result's resolution.
#pragma once
#include <math.h>
#include <stdint.h>

#if defined(__HIPCC__)
#define SPD_HD __host__ __device__ __forceinline__
#else
#define SPD_HD inline
#endif

namespace spd {

enum OpId {
    OP_DOT = 0, OP_L1, OP_MINK, OP_CANB, OP_HAMM, OP_KL, OP_JS, OP_CHEB, OP_CNT, OP_SEMI_SUM, OP_SEMI_EXT,
    OP_MINK_ANY,      // Minkowski of a degree other than 1..4 (powers through exp2 / log2: kernels of their own)
    OP_COUNT
};
enum Transform { TR_ID = 0, TR_SQRT, TR_NONZERO };
enum NormKind {
    NORM_NONE = 0, NORM_SUMSQ, NORM_SUM_SUMSQ, NORM_SUM, NORM_SUM_ABS, NORM_SUM_POW, NORM_NNZ,
    NORM_SEMI            // NORM_SEMI + product id: the sum of product(t, 0), and the number of entries
};
// products and sums a semiring may be built from; the ids follow spd_product / spd_sum in include/spd.h
enum SemiProduct {
    SP_TIMES = 0, SP_PLUS, SP_MIN, SP_MAX, SP_ABS_DIFF, SP_SQ_DIFF,
    SP_ABS_DIFF_POW, SP_CANBERRA, SP_NOT_EQUAL, SP_X_LOG_X_OVER_Y, SP_JS_TERM,     // the other products of Table 1
    SP_COUNT
};
enum SemiSum { SS_PLUS = 0, SS_MIN, SS_MAX, SS_COUNT };
// what a semiring call applies to the folded value; the ids follow spd_epilogue in include/spd.h
// (the expansions over row norms that follow SE_SQRT_HALF there run as the metrics they spell)
enum SemiEpilogue { SE_NONE = 0, SE_ROOT_P, SE_DIV_K, SE_SQRT_HALF };

// metric ids follow spd_metric in include/spd.h
enum MetricId {
    MT_INNER = 0, MT_COSINE, MT_L2, MT_CORRELATION, MT_JACCARD, MT_DICE, MT_HELLINGER, MT_L1,
    MT_CHEBYSHEV, MT_MINKOWSKI, MT_CANBERRA, MT_HAMMING, MT_KL, MT_JS, MT_RUSSELL_RAO,
    MT_L2_UNEXPANDED, MT_KL_STRICT, MT_JACCARD_LITERAL, MT_COUNT,
    // not in spd_metric: what the semiring entry points run as
    MT_SEMI_SUM = MT_COUNT,   // sum() = +
    MT_SEMI_EXT               // sum() = min or max
};

struct MetricInfo { int op, transform, norm; };

SPD_HD constexpr MetricInfo metric_info(int metric) {
    switch (metric) {
    case MT_INNER:       return {OP_DOT, TR_ID, NORM_NONE};
    case MT_COSINE:      return {OP_DOT, TR_ID, NORM_SUMSQ};
    case MT_L2:          return {OP_DOT, TR_ID, NORM_SUMSQ};
    case MT_CORRELATION: return {OP_DOT, TR_ID, NORM_SUM_SUMSQ};
    case MT_JACCARD:     return {OP_CNT, TR_NONZERO, NORM_SUM};
    case MT_DICE:        return {OP_CNT, TR_NONZERO, NORM_SUM};
    case MT_HELLINGER:   return {OP_DOT, TR_SQRT, NORM_SUMSQ};
    case MT_L1:          return {OP_L1, TR_ID, NORM_SUM_ABS};
    case MT_CHEBYSHEV:   return {OP_CHEB, TR_ID, NORM_NONE};
    case MT_MINKOWSKI:   return {OP_MINK, TR_ID, NORM_SUM_POW};
    case MT_CANBERRA:    return {OP_CANB, TR_ID, NORM_NNZ};
    case MT_HAMMING:     return {OP_HAMM, TR_ID, NORM_NNZ};
    case MT_KL:          return {OP_KL, TR_ID, NORM_NONE};
    case MT_JS:          return {OP_JS, TR_ID, NORM_SUM};
    case MT_RUSSELL_RAO: return {OP_CNT, TR_NONZERO, NORM_NONE};
    case MT_L2_UNEXPANDED:   return {OP_MINK, TR_ID, NORM_SUM_POW};      // Minkowski with p fixed at 2
    case MT_KL_STRICT:       return {OP_KL, TR_ID, NORM_NNZ};            // the row's entries must all be met
    case MT_JACCARD_LITERAL: return {OP_DOT, TR_ID, NORM_NNZ};
    case MT_SEMI_SUM:        return {OP_SEMI_SUM, TR_ID, NORM_SEMI};     // the caller adds the product id
    case MT_SEMI_EXT:        return {OP_SEMI_EXT, TR_ID, NORM_NONE};
    default:             return {-1, 0, 0};
    }
}

struct OpParams {
    float p;        // Minkowski degree
    float inv_p;
    double k;       // number of columns
    int metric;
    // semirings
    int product = 0;      // SemiProduct
    int over_union = 0;   // 1: product() over the union of the stored columns, the missing side read as 0
    float sign = 1.0f;    // sum() = min is carried as the max of the negated products
    int epilogue = 0;     // SemiEpilogue
};

// log2, exp2 and 1/x as the kernels use them: the hardware's transcendental units on the device
// (v_log_f32, v_exp_f32, v_rcp_f32: about 1 ulp, far inside the 1e-4 tolerance), libm on the
// host (test hooks only).  Everything built on them below is the same code on both sides.
SPD_HD float fast_log2(float x) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_logf(x);
#else
    return log2f(x);
#endif
}
SPD_HD float fast_exp2(float x) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_exp2f(x);
#else
    return exp2f(x);
#endif
}
SPD_HD float fast_rcp(float x) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_rcpf(x);
#else
    return 1.0f / x;
#endif
}
SPD_HD float fast_div(float x, float y) { return x * fast_rcp(y); }

// x / d in fp32 through a reciprocal: quotient estimate, exact residual (one FMA), correction
// (one FMA).  With the reciprocal good to an ulp this is the correctly rounded quotient (in
// particular exactly 1 for x == d, exactly 1/2 for d == 2x), at 5 instructions per quotient
// where the IEEE sequence with its range scaling takes 11.  The divisor is prepared once and
// serves many numerators; one whose magnitude lies outside [2^-100, 2^100] is brought into
// range by a power of two that the numerator then shares (a quotient beyond the fp32 range
// is undefined, where IEEE division gives 0 or infinity).
struct Divisor { float d, y, s; };        // scaled divisor, its reciprocal, the scale
SPD_HD Divisor divisor_of(float d) {
    const float m = fabsf(d);
    const float s = m < 0x1p-100f ? 0x1p64f : (m > 0x1p100f ? 0x1p-64f : 1.0f);
    const float ds = d * s;
    return {ds, fast_rcp(ds), s};
}
SPD_HD float divide(float x, const Divisor &v) {
    const float xs = x * v.s;
    const float q = xs * v.y;
    const float r = __builtin_fmaf(-q, v.d, xs);
    return __builtin_fmaf(r, v.y, q);
}

// The same for one quotient whose divisor is known to lie in [2^-100, 2^100].
SPD_HD float divide_in_range(float x, float d) {
    const float y = fast_rcp(d);
    const float q = x * y;
    const float r = __builtin_fmaf(-q, d, x);
    return __builtin_fmaf(r, y, q);
}

// Median of three: v clamped to [lo, hi] when lo <= hi.
SPD_HD float median3(float v, float lo, float hi) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_fmed3f(v, lo, hi);
#else
    return fmaxf(fminf(v, hi), fminf(fmaxf(v, hi), lo));
#endif
}

// Median of (a, b, 0): the one of a and b nearer to zero when they have the same sign, else 0.
SPD_HD float median_with_zero(float a, float b) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_fmed3f(a, b, 0.0f);
#else
    return fmaxf(fminf(a, b), fminf(fmaxf(a, b), 0.0f));
#endif
}

// |v|^p in fp32.  The same function feeds the row norm F and the per-visit product, so
// the terms that have to cancel are bit-identical (pow_abs(0) == 0).  Small integer
// degrees are plain products.
SPD_HD float pow_abs(float v, float p) {
    float a = fabsf(v);
    if (p == 1.0f) return a;
    if (p == 2.0f) return a * a;
    if (p == 3.0f) return a * a * a;
    if (p == 4.0f) { float q = a * a; return q * q; }
    return a == 0.0f ? 0.0f : fast_exp2(p * fast_log2(a));
}

// product() of a semiring, in the type it is accumulated in.
SPD_HD float abs_of(float v) { return __builtin_fabsf(v); }
SPD_HD double abs_of(double v) { return __builtin_fabs(v); }
SPD_HD float min_of(float a, float b) { return __builtin_fminf(a, b); }
SPD_HD double min_of(double a, double b) { return __builtin_fmin(a, b); }
SPD_HD float max_of(float a, float b) { return __builtin_fmaxf(a, b); }
SPD_HD double max_of(double a, double b) { return __builtin_fmax(a, b); }
// The five products beyond the first six are formed in fp32 from the (exact) fp32 values, with
// the same quotient and logarithm routines as the distances they come from, and widened:
//   |a - b|^p;  |a - b| / (|a| + |b|) (0 at (0, 0));  [a != b];  a ln(a / b) where both are
//   positive (else 0);  a ln(a / mu) + b ln(b / mu), mu = (a + b) / 2, 0 ln 0 = 0.
// Equal entries give exactly 0 in all five.
template <int P> SPD_HD float semi_product_f32(float a, float b, float p) {
    const float LN2 = 0.693147180559945309f;
    if constexpr (P == SP_ABS_DIFF_POW) {
        return pow_abs(a - b, p);
    } else if constexpr (P == SP_CANBERRA) {
        const float den = fabsf(a) + fabsf(b);
        return den != 0.0f ? divide(fabsf(a - b), divisor_of(den)) : 0.0f;
    } else if constexpr (P == SP_NOT_EQUAL) {
        return a != b ? 1.0f : 0.0f;
    } else if constexpr (P == SP_X_LOG_X_OVER_Y) {
        const bool both = a > 0.0f && b > 0.0f;
        return both ? LN2 * (a * fast_log2(divide(a, divisor_of(b)))) : 0.0f;
    } else {
        static_assert(P == SP_JS_TERM, "the products formed in fp32");
        const bool in_a = a > 0.0f, in_b = b > 0.0f;
        if (in_a && in_b) {
            const float sum = median3(a + b, 0x1p-100f, 0x1p100f);
            const float u = median3(divide_in_range(a, sum), 0x1p-126f, 0x1.fffffep-1f);
            return LN2 * (a * fast_log2(2.0f * u) + b * fast_log2(2.0f * (1.0f - u)));
        }
        return in_a ? LN2 * a : (in_b ? LN2 * b : 0.0f);
    }
}
template <int P, typename T> SPD_HD T semi_product(T a, T b, float p) {
    (void)p;
    if constexpr (P == SP_TIMES) return a * b;
    else if constexpr (P == SP_PLUS) return a + b;
    else if constexpr (P == SP_MIN) return min_of(a, b);
    else if constexpr (P == SP_MAX) return max_of(a, b);
    else if constexpr (P == SP_ABS_DIFF) return abs_of(a - b);
    else if constexpr (P == SP_SQ_DIFF) { T d = a - b; return d * d; }
    else return (T)semi_product_f32<P>((float)a, (float)b, p);
}
// A product and where it is applied (UNION: over the columns either row stores), as a type.
template <int P, bool UNION = false> struct ProductTag {
    static constexpr int value = P;
    static constexpr bool over_union = UNION;
};
// Calls f(ProductTag<p, u>) for the product id `product` and the domain `over_union`.
template <typename F> SPD_HD void for_product(int product, bool over_union, F &&f) {
#define SPD_CASE(P) case P: if (over_union) f(ProductTag<P, true>{}); else f(ProductTag<P, false>{}); break;
    switch (product) {
        SPD_CASE(SP_TIMES) SPD_CASE(SP_PLUS) SPD_CASE(SP_MIN) SPD_CASE(SP_MAX) SPD_CASE(SP_ABS_DIFF) SPD_CASE(SP_SQ_DIFF)
        SPD_CASE(SP_ABS_DIFF_POW) SPD_CASE(SP_CANBERRA) SPD_CASE(SP_NOT_EQUAL) SPD_CASE(SP_X_LOG_X_OVER_Y) SPD_CASE(SP_JS_TERM)
    default: break;
    }
#undef SPD_CASE
}
template <typename T> SPD_HD T semi_product_of(int product, T a, T b, float p) {
    T out = (T)0;
    for_product(product, false, [&](auto tag) { out = semi_product<decltype(tag)::value, T>(a, b, p); });
    return out;
}

// |v|^p with the degree known at compile time: DEG 1..4 are plain products, 0 is any other p.
// pow_abs(v, p) == pow_abs_as<degree_class(p)>(v, p) bit for bit.
template <int DEG> SPD_HD float pow_abs_as(float v, float p) {
    float a = fabsf(v);
    if constexpr (DEG == 1) return a;
    else if constexpr (DEG == 2) return a * a;
    else if constexpr (DEG == 3) return a * a * a;
    else if constexpr (DEG == 4) { float q = a * a; return q * q; }
    else return a == 0.0f ? 0.0f : fast_exp2(p * fast_log2(a));
}
SPD_HD int degree_class(float p) { return p == 1.0f ? 1 : (p == 2.0f ? 2 : (p == 3.0f ? 3 : (p == 4.0f ? 4 : 0))); }
// Calls f(ProductTag<d>) for the class d of the Minkowski degree p.
template <typename F> SPD_HD void for_degree(float p, F &&f) {
    switch (degree_class(p)) {
    case 1: f(ProductTag<1>{}); break;
    case 2: f(ProductTag<2>{}); break;
    case 3: f(ProductTag<3>{}); break;
    case 4: f(ProductTag<4>{}); break;
    default: f(ProductTag<0>{}); break;
    }
}

SPD_HD float transform_value(int tr, float v) {
    if (tr == TR_SQRT) return sqrtf(v);
    if (tr == TR_NONZERO) return v != 0.0f ? 1.0f : 0.0f;
    return v;
}

// Contribution of one (transformed) stored value to the two raw row sums.
SPD_HD void norm_accumulate(int norm, float t, float p, double &s0, double &s1) {
    double d = (double)t;
    switch (norm) {
    case NORM_SUMSQ:     s0 += d * d; break;
    case NORM_SUM_SUMSQ: s0 += d; s1 += d * d; break;
    case NORM_SUM:       s0 += d; break;
    case NORM_SUM_ABS:   s0 += fabs(d); break;
    case NORM_SUM_POW:   s0 += (double)pow_abs(t, p); s1 += (t != 0.0f) ? 1.0 : 0.0; break;
    case NORM_NNZ:       s0 += (t != 0.0f) ? 1.0 : 0.0; break;
    default:
        if (norm >= NORM_SEMI && t != 0.0f) { s0 += semi_product_of<double>(norm - NORM_SEMI, d, 0.0, p); s1 += 1.0; }
        break;
    }
}

// Raw row sums -> the two numbers the expansion function reads.
SPD_HD void norm_derive(int metric, double k, double s0, double s1, double &d0, double &d1) {
    d0 = s0; d1 = s1;
    if (metric == MT_COSINE) {
        d1 = s0 > 0.0 ? 1.0 / sqrt(s0) : 0.0;
    } else if (metric == MT_CORRELATION) {
        double var = k * s1 - s0 * s0;                 // k^2 times the variance
        d1 = var > 0.0 ? 1.0 / sqrt(var) : 0.0;
    }
}

// ------------------------------------------------------------------------------------
// per-visit products.  Acc is what one (A row, B row) pair accumulates; Bv what is
// derived once from a stored value of B and reused for every staged A row.
// v0/v1/v2 expose the sums as doubles (for the slices of spilled rows and for finish()).
// ------------------------------------------------------------------------------------
template <int OP> struct Op;

template <> struct Op<OP_DOT> {
    struct Acc { double v; };
    struct Bv { double db; };
    SPD_HD static void init(Acc &x) { x.v = 0.0; }
    SPD_HD static Bv prep(float b, const OpParams &) { return {(double)b}; }
    SPD_HD static void visit(Acc &x, float a, const Bv &b, const OpParams &) { x.v = fma((double)a, b.db, x.v); }
    SPD_HD static void combine(Acc &x, const Acc &y) { x.v += y.v; }
    SPD_HD static double v0(const Acc &x) { return x.v; }
    SPD_HD static double v1(const Acc &) { return 0.0; }
    SPD_HD static double v2(const Acc &) { return 0.0; }
};

// |a - b| - |a| - |b| is -2 min(|a|, |b|) when a and b have the same sign and 0 otherwise
// (also when a == 0): the sum keeps c = |median(a, b, 0)|, which is exact in fp32.
template <> struct Op<OP_L1> {
    struct Acc { double v; };
    struct Bv { float b; };
    SPD_HD static void init(Acc &x) { x.v = 0.0; }
    SPD_HD static Bv prep(float b, const OpParams &) { return {b}; }
    SPD_HD static void visit(Acc &x, float a, const Bv &b, const OpParams &) {
        x.v += (double)fabsf(median_with_zero(a, b.b));
    }
    SPD_HD static void combine(Acc &x, const Acc &y) { x.v += y.v; }
    SPD_HD static double v0(const Acc &x) { return -2.0 * x.v; }
    SPD_HD static double v1(const Acc &) { return 0.0; }
    SPD_HD static double v2(const Acc &) { return 0.0; }
};

// Minkowski keeps the differences on shared columns (d) apart from what they replace in the
// two row norms (s), and counts the shared columns: the p-th root would otherwise blow the
// rounding residue of F(x) + F(y) - s up when the two rows have the same support.
template <> struct Op<OP_MINK> {
    struct Acc { double d, s; int hits; };
    struct Bv { float b; double pwb; };
    SPD_HD static void init(Acc &x) { x.d = 0.0; x.s = 0.0; x.hits = 0; }
    SPD_HD static Bv prep(float b, const OpParams &q) { return {b, (double)pow_abs(b, q.p)}; }
    template <int DEG> SPD_HD static void visit_as(Acc &x, float a, const Bv &b, const OpParams &q) {
        bool hit = (a != 0.0f) && (b.b != 0.0f);
        if constexpr (DEG != 0) {
            // a power is 0 at 0: a column one side does not store is silenced by clearing the other
            // side's value (the power of b is cheap enough to form again, bit for bit the norm's)
            const float am = (b.b != 0.0f) ? a : 0.0f, bm = (a != 0.0f) ? b.b : 0.0f;
            x.d += (double)pow_abs_as<DEG>(am - bm, q.p);
            x.s += (double)pow_abs_as<DEG>(am, q.p) + (double)pow_abs_as<DEG>(bm, q.p);
        } else {
            x.d += hit ? (double)pow_abs_as<DEG>(a - b.b, q.p) : 0.0;
            x.s += hit ? (double)pow_abs_as<DEG>(a, q.p) + b.pwb : 0.0;
        }
        x.hits += hit ? 1 : 0;
    }
    SPD_HD static void visit(Acc &x, float a, const Bv &b, const OpParams &q) {
        for_degree(q.p, [&](auto tag) { visit_as<decltype(tag)::value>(x, a, b, q); });
    }
    SPD_HD static void combine(Acc &x, const Acc &y) { x.d += y.d; x.s += y.s; x.hits += y.hits; }
    SPD_HD static double v0(const Acc &x) { return x.d; }
    SPD_HD static double v1(const Acc &x) { return x.s; }
    SPD_HD static double v2(const Acc &x) { return (double)x.hits; }
};

// The same sums for any other degree: the powers go through exp2 / log2, which takes so many
// more registers that these kernels are kept apart from the ones of the small integer degrees.
template <> struct Op<OP_MINK_ANY> : Op<OP_MINK> {
    SPD_HD static void visit(Acc &x, float a, const Bv &b, const OpParams &q) { Op<OP_MINK>::visit_as<0>(x, a, b, q); }
};

template <> struct Op<OP_CANB> {
    struct Acc { double v; };
    struct Bv { float b; };
    SPD_HD static void init(Acc &x) { x.v = 0.0; }
    SPD_HD static Bv prep(float b, const OpParams &) { return {b}; }
    SPD_HD static void visit(Acc &x, float a, const Bv &b, const OpParams &) {
        bool hit = (a != 0.0f) && (b.b != 0.0f);
        // each one-sided column counts 1: a shared one replaces two of them by its ratio; elsewhere
        // the ratio (0/0 where both are absent) is replaced by the 2 that cancels
        float ratio = hit ? fast_div(fabsf(a - b.b), fabsf(a) + fabsf(b.b)) : 2.0f;
        x.v += (double)ratio - 2.0;
    }
    SPD_HD static void combine(Acc &x, const Acc &y) { x.v += y.v; }
    SPD_HD static double v0(const Acc &x) { return x.v; }
    SPD_HD static double v1(const Acc &) { return 0.0; }
    SPD_HD static double v2(const Acc &) { return 0.0; }
};

template <> struct Op<OP_HAMM> {
    struct Acc { int c; };
    struct Bv { float b; };
    SPD_HD static void init(Acc &x) { x.c = 0; }
    SPD_HD static Bv prep(float b, const OpParams &) { return {b}; }
    SPD_HD static void visit(Acc &x, float a, const Bv &b, const OpParams &) {
        bool hit = (a != 0.0f) && (b.b != 0.0f);
        x.c += hit ? ((a != b.b) ? -1 : -2) : 0;
    }
    SPD_HD static void combine(Acc &x, const Acc &y) { x.c += y.c; }
    SPD_HD static double v0(const Acc &x) { return (double)x.c; }
    SPD_HD static double v1(const Acc &) { return 0.0; }
    SPD_HD static double v2(const Acc &) { return 0.0; }
};

// Set metrics: the number of shared columns.  The scan kernel counts it for many staged
// rows at a time in byte lanes of 32-bit words (one byte of the staged table per row); this
// form, one pair at a time, serves the host.
template <> struct Op<OP_CNT> {
    struct Acc { int c; };
    struct Bv { float b; };
    SPD_HD static void init(Acc &x) { x.c = 0; }
    SPD_HD static Bv prep(float b, const OpParams &) { return {b}; }
    SPD_HD static void visit(Acc &x, float a, const Bv &b, const OpParams &) {
        x.c += ((a != 0.0f) && (b.b != 0.0f)) ? 1 : 0;
    }
    SPD_HD static void combine(Acc &x, const Acc &y) { x.c += y.c; }
    SPD_HD static double v0(const Acc &x) { return (double)x.c; }
    SPD_HD static double v1(const Acc &) { return 0.0; }
    SPD_HD static double v2(const Acc &) { return 0.0; }
};

// KL: a log(a/b) = ln 2 * a log2(a/b) on shared columns, with a correctly rounded quotient so
// that equal entries give exactly 0; the factor ln 2 is applied once, by finish().
template <> struct Op<OP_KL> {
    struct Acc { double v; int hits; };      // hits: columns where both rows hold mass (the strict variant needs them)
    struct Bv { float b; Divisor by_b; };
    SPD_HD static void init(Acc &x) { x.v = 0.0; x.hits = 0; }
    SPD_HD static Bv prep(float b, const OpParams &) { return {b, divisor_of(b > 0.0f ? b : 1.0f)}; }
    SPD_HD static void visit(Acc &x, float a, const Bv &b, const OpParams &) {
        bool hit = (a > 0.0f) && (b.b > 0.0f);
        // elsewhere the quotient is 1, its logarithm 0 and the term a * 0: nothing to select away
        float t = a * fast_log2(hit ? divide(a, b.by_b) : 1.0f);
        x.v += (double)t;
        x.hits += hit ? 1 : 0;
    }
    SPD_HD static void combine(Acc &x, const Acc &y) { x.v += y.v; x.hits += y.hits; }
    SPD_HD static double v0(const Acc &x) { return x.v; }
    SPD_HD static double v1(const Acc &x) { return (double)x.hits; }
    SPD_HD static double v2(const Acc &) { return 0.0; }
};

// Jensen-Shannon: on a shared column, with u = a/(a+b),
//   a log(2a/(a+b)) + b log(2b/(a+b)) = ln 2 [ a log2(2u) + b log2(2(1-u)) ],
// exactly 0 for a == b (u = 1/2 exactly, 2u = 1) and accurate when a is close to b (the two
// logarithms are then small and each is formed directly).  The bracket is accumulated; the
// factor ln 2 is applied by finish().  A one-sided column adds its value times log 2, which
// finish() takes from the row sums minus `s`, the sum of the values seen on shared columns.
template <> struct Op<OP_JS> {
    struct Acc { double f, s; };
    struct Bv { float b; double db; };
    SPD_HD static void init(Acc &x) { x.f = 0.0; x.s = 0.0; }
    SPD_HD static Bv prep(float b, const OpParams &) { return {b, (double)b}; }
    SPD_HD static void visit(Acc &x, float a, const Bv &b, const OpParams &) {
        bool hit = (a > 0.0f) && (b.b > 0.0f);
        float aa = hit ? a : 1.0f, bb = hit ? b.b : 1.0f;
        // (a sum outside [2^-100, 2^100] is clamped: below it, the two entries' term is far below the
        // result's resolution whatever u is taken; above it lie sums of values beyond 6e29)
        float sum = median3(aa + bb, 0x1p-100f, 0x1p100f);
        // correctly rounded: 1/2 for aa == bb.  Kept inside [2^-126, 1 - 2^-24]: a quotient that
        // rounds to 1 (aa beyond 2^25 bb) would leave log2(0) on the other side, one that
        // underflows log2(0) on this one; what the clamp changes is below 1e-6 of the larger entry
        float u = median3(divide_in_range(aa, sum), 0x1p-126f, 0x1.fffffep-1f);
        float t = aa * fast_log2(2.0f * u) + bb * fast_log2(2.0f * (1.0f - u));
        x.f += (double)t;                                // elsewhere aa == bb == 1: u = 1/2, both logarithms 0
        x.s += hit ? (double)a + b.db : 0.0;
    }
    SPD_HD static void combine(Acc &x, const Acc &y) { x.f += y.f; x.s += y.s; }
    SPD_HD static double v0(const Acc &x) { return x.f; }
    SPD_HD static double v1(const Acc &x) { return x.s; }
    SPD_HD static double v2(const Acc &) { return 0.0; }
};

template <> struct Op<OP_CHEB> {
    struct Acc { float m; };
    struct Bv { float b; };
    SPD_HD static void init(Acc &x) { x.m = 0.0f; }
    SPD_HD static Bv prep(float b, const OpParams &) { return {b}; }
    SPD_HD static void visit(Acc &x, float a, const Bv &b, const OpParams &) { x.m = fmaxf(x.m, fabsf(a - b.b)); }
    SPD_HD static void combine(Acc &x, const Acc &y) { x.m = fmaxf(x.m, y.m); }
    SPD_HD static double v0(const Acc &x) { return (double)x.m; }
    SPD_HD static double v1(const Acc &) { return 0.0; }
    SPD_HD static double v2(const Acc &) { return 0.0; }
};

// Semiring with sum() = + (Section 2.2).  Over the intersection the sum of product(a, b) is the
// result.  Over the union (a non-annihilating product) the one-sided columns add product(a, 0)
// and product(0, b): they come from the two rows' sums of product(., 0) minus `s`, the share of
// those sums that falls on shared columns; `hits` counts the shared columns, so that two rows
// with the same support leave exactly nothing (as for Minkowski).  Terms are formed in fp64:
// products and sums of fp32 values are exact there.
template <> struct Op<OP_SEMI_SUM> {
    struct Acc { double d, s; int hits; };
    struct Bv { float b; };
    SPD_HD static void init(Acc &x) { x.d = 0.0; x.s = 0.0; x.hits = 0; }
    SPD_HD static Bv prep(float b, const OpParams &) { return {b}; }
    template <int P, bool UNION> SPD_HD static void visit_as(Acc &x, float a, const Bv &b, const OpParams &q) {
        // every product offered gives 0 at (0, 0): a column that one side does not store is
        // silenced by clearing the other side's value, not by selecting among the fp64 results
        const double da = (double)((b.b != 0.0f) ? a : 0.0f), db = (double)((a != 0.0f) ? b.b : 0.0f);
        x.d += semi_product<P, double>(da, db, q.p);
        if constexpr (UNION) {
            x.s += semi_product<P, double>(da, 0.0, q.p) + semi_product<P, double>(0.0, db, q.p);
            x.hits += ((a != 0.0f) && (b.b != 0.0f)) ? 1 : 0;
        }
    }
    SPD_HD static void visit(Acc &x, float a, const Bv &b, const OpParams &q) {
        for_product(q.product, q.over_union != 0, [&](auto tag) {
            visit_as<decltype(tag)::value, decltype(tag)::over_union>(x, a, b, q);
        });
    }
    SPD_HD static void combine(Acc &x, const Acc &y) { x.d += y.d; x.s += y.s; x.hits += y.hits; }
    SPD_HD static double v0(const Acc &x) { return x.d; }
    SPD_HD static double v1(const Acc &x) { return x.s; }
    SPD_HD static double v2(const Acc &x) { return (double)x.hits; }
};

// Semiring with sum() = max, or min as the max of the negated products (`sign`).  A column
// takes part when both rows store it, or, over the union, when either does (a then may be 0);
// what only x stores is completed by the kernel like Chebyshev's.  The product is formed in
// fp32: rounding is monotone, so the maximum of the rounded terms is the rounded maximum.
template <> struct Op<OP_SEMI_EXT> {
    struct Acc { float m; };
    struct Bv { float b; };
    SPD_HD static void init(Acc &x) { x.m = -__builtin_huge_valf(); }
    SPD_HD static Bv prep(float b, const OpParams &) { return {b}; }
    template <int P, bool UNION> SPD_HD static void visit_as(Acc &x, float a, const Bv &b, const OpParams &q) {
        const bool in_a = a != 0.0f, in_b = b.b != 0.0f;
        const bool take = UNION ? (in_a || in_b) : (in_a && in_b);
        const float v = q.sign * semi_product<P, float>(a, b.b, q.p);
        x.m = fmaxf(x.m, take ? v : -__builtin_huge_valf());
    }
    SPD_HD static void visit(Acc &x, float a, const Bv &b, const OpParams &q) {
        for_product(q.product, q.over_union != 0, [&](auto tag) {
            visit_as<decltype(tag)::value, decltype(tag)::over_union>(x, a, b, q);
        });
    }
    SPD_HD static void combine(Acc &x, const Acc &y) { x.m = fmaxf(x.m, y.m); }
    SPD_HD static double v0(const Acc &x) { return (double)x.m; }
    SPD_HD static double v1(const Acc &) { return 0.0; }
    SPD_HD static double v2(const Acc &) { return 0.0; }
};

// What a staged row's entry a would contribute in a column the other row does not store, as the
// key the rows' largest such contributions are ranked by (Chebyshev: |a|).
template <int OP> SPD_HD float one_sided_key(float a, const OpParams &q) {
    if constexpr (OP == OP_SEMI_EXT) return q.sign * semi_product_of<float>(q.product, a, 0.0f, q.p);
    else return fabsf(a);
}

// One visit, with the product and the domain of a semiring known at compile time (they are
// ignored otherwise).
template <int OP, int P, bool UNION>
SPD_HD void visit_with(typename Op<OP>::Acc &x, float a, const typename Op<OP>::Bv &b, const OpParams &q) {
    if constexpr (OP == OP_SEMI_SUM || OP == OP_SEMI_EXT) Op<OP>::template visit_as<P, UNION>(x, a, b, q);
    else if constexpr (OP == OP_MINK) Op<OP>::template visit_as<(P == 0 ? 2 : P)>(x, a, b, q);   // P: the class of the degree, 1..4
    else Op<OP>::visit(x, a, b, q);
}

// Expansion function (Table 1, "Expansion" column, and the closing steps of the union
// family).  v, s, w: the accumulated sums; a0,a1 / b0,b1: derived norms of the two rows.
// The metric is a template argument so that a kernel can pick the formula once per slab
// instead of once per pair.
// The closing step of a semiring call on its folded value: nothing, the p-th root, the division
// by the number of columns, or the square root of the half.
SPD_HD float semi_epilogue(const OpParams &q, double v) {
    switch (q.epilogue) {
    case SE_ROOT_P: {
        const float tf = (float)v;
        if (q.p == 1.0f) return tf;
        if (q.p == 2.0f) return sqrtf(tf);
        return tf == 0.0f ? 0.0f : fast_exp2(q.inv_p * fast_log2(tf));
    }
    case SE_DIV_K: return (float)(v / q.k);
    case SE_SQRT_HALF: return sqrtf((float)(v > 0.0 ? 0.5 * v : 0.0));
    default: return (float)v;
    }
}

template <int MT>
SPD_HD float finish_as(const OpParams &q, double v, double s, double w, double a0, double a1, double b0, double b1) {
    const double LN2 = 0.693147180559945309417232121458;
    (void)s; (void)w; (void)a0; (void)a1; (void)b0; (void)b1; (void)q;
    if constexpr (MT == MT_INNER || MT == MT_CHEBYSHEV) {
        return (float)v;
    } else if constexpr (MT == MT_COSINE) {
        return (float)((a0 == 0.0 && b0 == 0.0) ? 0.0 : ((a0 == 0.0 || b0 == 0.0) ? 1.0 : 1.0 - v * a1 * b1));
    } else if constexpr (MT == MT_L2) {
        double t = a0 - 2.0 * v + b0;
        return sqrtf((float)(t > 0.0 ? t : 0.0));
    } else if constexpr (MT == MT_CORRELATION) {
        return (float)((a1 == 0.0 || b1 == 0.0) ? 1.0 : 1.0 - (q.k * v - a0 * b0) * a1 * b1);
    } else if constexpr (MT == MT_JACCARD) {
        // counts below 2^24 are exact in fp32, and a correctly rounded fp32 quotient is well inside
        // the tolerance and the same for equal ratios (pairs that tie exactly stay tied): the
        // 64-bit division is kept for rows beyond that
        // (with fewer than 2^23 columns every count and the union's size are exact in fp32, and
        // the question is settled once per launch, not once per pair)
        if (q.k < 8388608.0) {
            const float vf = (float)v, uf = ((float)a0 + (float)b0) - vf;
            return uf == 0.0f ? 0.0f : 1.0f - vf / uf;
        }
        double u = a0 + b0 - v;
        if (u < 16777216.0) { float uf = (float)u; return uf == 0.0f ? 0.0f : 1.0f - (float)v / uf; }
        return (float)(1.0 - v / u);
    } else if constexpr (MT == MT_DICE) {
        if (q.k < 4194304.0) {
            const float tf = (float)a0 + (float)b0;
            return tf == 0.0f ? 0.0f : 1.0f - (2.0f * (float)v) / tf;
        }
        double t = a0 + b0;
        if (t < 8388608.0) { float tf = (float)t; return tf == 0.0f ? 0.0f : 1.0f - (2.0f * (float)v) / tf; }
        return (float)(1.0 - 2.0 * v / t);
    } else if constexpr (MT == MT_HELLINGER) {
        double t = 0.5 * (a0 + b0) - v;
        return sqrtf((float)(t > 0.0 ? t : 0.0));
    } else if constexpr (MT == MT_L1 || MT == MT_CANBERRA) {
        double t = a0 + b0 + v;
        return (float)(t > 0.0 ? t : 0.0);
    } else if constexpr (MT == MT_MINKOWSKI || MT == MT_L2_UNEXPANDED) {
        // v: differences on shared columns, s: their share of the norms, w: how many;
        // a1 / b1 count the entries of the rows: equal supports leave no one-sided part
        double one_sided = (w == a1 && w == b1) ? 0.0 : (a0 + b0) - s;
        double t = v + (one_sided > 0.0 ? one_sided : 0.0);
        float tf = (float)t;
        if (q.p == 1.0f) return tf;
        if (q.p == 2.0f) return sqrtf(tf);
        return tf == 0.0f ? 0.0f : fast_exp2(q.inv_p * fast_log2(tf));
    } else if constexpr (MT == MT_HAMMING) {
        return (float)((a0 + b0 + v) / q.k);
    } else if constexpr (MT == MT_KL) {
        return (float)(LN2 * v);
    } else if constexpr (MT == MT_KL_STRICT) {
        // s counts the columns where both rows hold mass, a0 the entries of x: an entry of x that
        // met nothing in y makes the divergence infinite
        return s == a0 ? (float)(LN2 * v) : __builtin_huge_valf();
    } else if constexpr (MT == MT_JACCARD_LITERAL) {
        double u = a0 + b0 - v;
        return (float)((u == 0.0) ? 0.0 : 1.0 - v / u);
    } else if constexpr (MT == MT_JS) {
        double t = 0.5 * LN2 * (((a0 + b0) - s) + v);
        return sqrtf((float)(t > 0.0 ? t : 0.0));
    } else if constexpr (MT == MT_RUSSELL_RAO) {
        return (float)((q.k - v) / q.k);
    } else if constexpr (MT == MT_SEMI_SUM) {
        // v: products on shared columns, s: what those columns hold of the two rows' sums of
        // product(., 0), w: how many they are; a1 / b1 count the entries of the rows
        if (!q.over_union) return semi_epilogue(q, v);
        return semi_epilogue(q, v + ((w == a1 && w == b1) ? 0.0 : (a0 + b0) - s));
    } else if constexpr (MT == MT_SEMI_EXT) {
        return semi_epilogue(q, (double)q.sign * v);
    } else {
        return 0.0f;
    }
}

template <int MT> struct MetricTag { static constexpr int value = MT; };

// The product that computes a metric, and OP_DOT for the set metrics too (a dot product of
// 0/1 values counts the shared columns: the route the option "byte_counters" 0 selects).
SPD_HD constexpr bool op_serves(int op, int metric) {
    return metric_info(metric).op == op || (op == OP_DOT && metric_info(metric).op == OP_CNT) ||
           (op == OP_MINK_ANY && metric == MT_MINKOWSKI);
}

// Calls f(MetricTag<m>) for the metric `metric`, which must be one that product OP serves
// (the others are not instantiated: a kernel of one product carries only its own formulas).
template <int OP, typename F> SPD_HD void for_metric_of(int metric, F &&f) {
#define SPD_CASE(M) case M: if constexpr (op_serves(OP, M)) f(MetricTag<M>{}); break;
    switch (metric) {
        SPD_CASE(MT_INNER) SPD_CASE(MT_COSINE) SPD_CASE(MT_L2) SPD_CASE(MT_CORRELATION) SPD_CASE(MT_JACCARD)
        SPD_CASE(MT_DICE) SPD_CASE(MT_HELLINGER) SPD_CASE(MT_L1) SPD_CASE(MT_CHEBYSHEV) SPD_CASE(MT_MINKOWSKI)
        SPD_CASE(MT_CANBERRA) SPD_CASE(MT_HAMMING) SPD_CASE(MT_KL) SPD_CASE(MT_JS) SPD_CASE(MT_RUSSELL_RAO)
        SPD_CASE(MT_L2_UNEXPANDED) SPD_CASE(MT_KL_STRICT) SPD_CASE(MT_JACCARD_LITERAL)
        SPD_CASE(MT_SEMI_SUM) SPD_CASE(MT_SEMI_EXT)
    default: break;
    }
#undef SPD_CASE
}

// The same with the metric known only at run time.
SPD_HD float finish(const OpParams &q, double v, double s, double w, double a0, double a1, double b0, double b1) {
    switch (q.metric) {
#define SPD_CASE(M) case M: return finish_as<M>(q, v, s, w, a0, a1, b0, b1);
        SPD_CASE(MT_INNER) SPD_CASE(MT_COSINE) SPD_CASE(MT_L2) SPD_CASE(MT_CORRELATION) SPD_CASE(MT_JACCARD)
        SPD_CASE(MT_DICE) SPD_CASE(MT_HELLINGER) SPD_CASE(MT_L1) SPD_CASE(MT_CHEBYSHEV) SPD_CASE(MT_MINKOWSKI)
        SPD_CASE(MT_CANBERRA) SPD_CASE(MT_HAMMING) SPD_CASE(MT_KL) SPD_CASE(MT_JS) SPD_CASE(MT_RUSSELL_RAO)
        SPD_CASE(MT_L2_UNEXPANDED) SPD_CASE(MT_KL_STRICT) SPD_CASE(MT_JACCARD_LITERAL)
        SPD_CASE(MT_SEMI_SUM) SPD_CASE(MT_SEMI_EXT)
#undef SPD_CASE
    default: return 0.0f;
    }
}

}  // namespace spd
