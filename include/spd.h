/*
 * spd - all-pairs distances between the rows of two CSR matrices on one MI355X (gfx950),
 * computed as a sparse semiring product, with an optional fused brute-force k-NN.
 *
 * The operation is the one stated in Section 2 of "GPU Semiring Primitives for Sparse
 * Neighborhood Methods": A is m x k, B is n x k, both in CSR with ascending columns
 * inside each row, and the result is the dense m x n matrix C with C[i][j] = d(A_i, B_j),
 * produced without transposing or copying the inputs in full.  Each distance of Table 1
 * is a product()/sum() pair; the distances of the dot-product family are finished by
 * an expansion function over row norms (Section 3.4), the others apply their product over
 * the union of the non-zero columns of the two rows (Section 2.2, Eq. 2).  k-NN follows
 * the benchmark protocol of Section 4.2: distances of every query row to every index row,
 * then the k nearest.
 *
 * Conventions
 *  - Every pointer inside spd_csr and every `out*` pointer is a DEVICE pointer owned by
 *    the caller.  Inputs are read only.  Outputs need no initialisation and are fully
 *    overwritten.  A and B may be the same matrix.
 *  - All functions return a status; nothing is thrown across the boundary.
 *    spd_last_error() gives a text for the last failure on the handle.
 *  - spd_pairwise / spd_knn bin the rows by degree on the host.  They take the row pointers from
 *    `host_indptr` where the caller has a host copy, and else read the device arrays back (one
 *    stream synchronisation); then they enqueue all kernels on the handle's stream and return
 *    without waiting for them.  With host copies of both operands a call does not wait for the
 *    stream at all, so the planning of one call runs while the kernels of the one before it do.
 *    A host copy that differs from the device array gives wrong results (its last entry is
 *    checked against nnz, and no access leaves the arrays).
 *  - Scratch memory comes from the handle's own grow-only allocation, or from the caller
 *    through spd_set_workspace().
 *  - A handle serves one call at a time (calls on one handle from several threads must be
 *    serialised by the caller; different handles are independent).  A handle owns one helper
 *    thread, started by its first call, on which part of the planning runs (after a call it
 *    polls for the next one for 300 microseconds before it sleeps), and up to three internal
 *    streams of default priority beside the caller's stream.
 *  - Stored zeros are legal and count as absent.  Values must be finite; Hellinger, KL and
 *    Jensen-Shannon expect non-negative values (anything else is undefined, and reported by
 *    spd_csr_validate()); for KL and Jensen-Shannon the quotient of two entries of one column
 *    must lie within the fp32 range.
 */
#ifndef SPD_H
#define SPD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct spd_handle spd_handle;
typedef struct spd_index spd_index;

typedef struct {
    int64_t n_rows, n_cols, nnz;
    const int64_t *indptr;  /* device, n_rows+1, indptr[0]==0, non-decreasing, last==nnz */
    const int32_t *indices; /* device, nnz, strictly ascending inside a row, 0<=c<n_cols  */
    const float *values;    /* device, nnz, finite                                        */
    const int64_t *host_indptr; /* HOST, optional (NULL if there is none): a copy of indptr in
                                   host memory, n_rows+1, valid and unchanged during the call  */
} spd_csr;

/* Table 1 of the paper.  The comment gives the value returned for rows x, y of length k. */
typedef enum {
    SPD_INNER_PRODUCT = 0,  /* sum x y (a similarity; spd_knn returns the LARGEST values)   */
    SPD_COSINE,             /* 1 - <x,y>/(|x|_2 |y|_2); 1 if one row is zero, 0 if both are */
    SPD_L2_EXPANDED,        /* sqrt(max(0, |x|^2 - 2<x,y> + |y|^2))                         */
    SPD_CORRELATION,        /* 1 - Pearson correlation, means over all k; 1 if no variance  */
    SPD_JACCARD,            /* 1 - |sx & sy|/|sx | sy| on the supports; 0 if both empty     */
    SPD_DICE,               /* 1 - 2|sx & sy|/(|sx|+|sy|) on the supports; 0 if both empty  */
    SPD_HELLINGER,          /* sqrt(sum (sqrt x - sqrt y)^2)/sqrt 2, x,y >= 0               */
    SPD_L1,                 /* sum |x-y|                                                     */
    SPD_CHEBYSHEV,          /* max |x-y|                                                     */
    SPD_MINKOWSKI,          /* (sum |x-y|^p)^(1/p), p > 0                                    */
    SPD_CANBERRA,           /* sum |x-y|/(|x|+|y|), 0/0 = 0                                  */
    SPD_HAMMING,            /* #{x != y} / k                                                 */
    SPD_KL_DIVERGENCE,      /* sum over columns present in both rows of x log(x/y)           */
    SPD_JENSEN_SHANNON,     /* sqrt(sum(x log(x/mu) + y log(y/mu))/2), mu=(x+y)/2           */
    SPD_RUSSELL_RAO,        /* (k - |sx & sy|)/k                                             */
    /* variants */
    SPD_L2_UNEXPANDED,      /* sqrt(sum (x-y)^2) through the union product (Section 2.1: the
                               expanded form cancels for close rows; this one is Minkowski, p = 2) */
    SPD_KL_STRICT,          /* sum x log(x/y), +infinity where x > 0 meets y = 0 (textbook KL)       */
    SPD_JACCARD_LITERAL,    /* 1 - <x,y>/(|x|_0 + |y|_0 - <x,y>): Table 1's expansion column by the
                               letter (the set reading on 0/1 data; 0 if the denominator is 0)      */
    SPD_METRIC_COUNT
} spd_metric;

typedef enum {
    SPD_OK = 0,
    SPD_ERR_NULL,          /* a required pointer is NULL                                   */
    SPD_ERR_DIM_MISMATCH,  /* A.n_cols != B.n_cols, or negative / inconsistent sizes       */
    SPD_ERR_BAD_CSR,       /* row pointers or (spd_csr_validate only) contents are invalid */
    SPD_ERR_BAD_METRIC,
    SPD_ERR_BAD_P,         /* Minkowski needs a finite p > 0                               */
    SPD_ERR_BAD_K,         /* k < 1, k > index rows, or k > SPD_KNN_MAX_K                  */
    SPD_ERR_WORKSPACE,     /* caller workspace too small, or allocation failed             */
    SPD_ERR_HIP,           /* a HIP runtime call failed (no device, launch failure, ...)   */
    SPD_ERR_UNSUPPORTED    /* sizes beyond what the kernels index (see spd_last_error)     */
} spd_status;

/* Largest k the fused selection keeps per query (one list entry per lane of a wavefront). */
#define SPD_KNN_MAX_K 64

/* Creates a handle bound to a HIP stream (`hip_stream` is a hipStream_t, NULL = the null
 * stream) on the current device.  The handle owns pinned staging memory and, unless
 * spd_set_workspace() is used, its device scratch.  Destroy it with spd_destroy(). */
spd_status spd_create(spd_handle **handle, void *hip_stream);
spd_status spd_destroy(spd_handle *handle);

/* Upper bound, from the shapes alone, of the device scratch one spd_pairwise /
 * spd_knn call with these operands needs (`k_neighbors` = 0 for spd_pairwise). */
spd_status spd_workspace_bytes(const spd_handle *handle, const spd_csr *A, const spd_csr *B,
                               spd_metric metric, int k_neighbors, size_t *bytes);

/* Makes the handle use caller memory (device, 256-byte aligned) as scratch instead of its
 * own allocation; (NULL, 0) returns to the internal one.  The memory must stay valid until
 * the work enqueued by later calls has finished. */
spd_status spd_set_workspace(spd_handle *handle, void *device_ptr, size_t bytes);

/* out[i * B.n_rows + j] = d(A_i, B_j), fp32, row-major, m x n (Section 2; Table 1).
 * `p` is read for SPD_MINKOWSKI only. */
spd_status spd_pairwise(spd_handle *handle, const spd_csr *A, const spd_csr *B, spd_metric metric,
                        float p, float *out);

/* spd_pairwise for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments and same result as spd_pairwise,
 * but the call allocates nothing (no hipMalloc, hipHostMalloc, hipFree, stream or event creation):
 * its scratch is a static array of SPD_STATIC_SCRATCH_BYTES bytes that every GPU the library runs
 * on holds from the library's first use there until the process ends, and its plans pass through
 * the SPD_STATIC_STAGING_BYTES bytes of pinned memory every handle holds from spd_create.
 *  - Both operands must bring `host_indptr` (nothing is copied back, the stream is not waited for).
 *  - Operands whose packed copy of B, plans and partial sums exceed the array, or whose plans
 *    exceed the staging memory, are rejected with SPD_ERR_WORKSPACE before anything is enqueued
 *    (B up to some 3.5 million stored entries fits; spd_last_error gives the bytes needed).
 *  - Everything runs on the handle's stream (no internal side streams), launch timing is off.
 *  - All calls on one GPU, from any handle, share that GPU's array and leave their data in it:
 *    no kernel reads scratch it has not written in the same call, so nothing needs clearing, but
 *    two calls that overlap in time on one GPU (two handles, two streams) race.  Calls on one
 *    stream, or ordered by events, are safe. */
#define SPD_STATIC_SCRATCH_BYTES (32u << 20)
#define SPD_STATIC_STAGING_BYTES (4u << 20)
spd_status spd_pairwise_static(spd_handle *handle, const spd_csr *A, const spd_csr *B, spd_metric metric,
                               float p, float *out);

/* For each query row the k index rows at the smallest distance (largest value for
 * SPD_INNER_PRODUCT), selected inside the distance kernels without materialising the
 * m x n matrix (Section 4.2).  out_idx[i*k + t] (int64) and out_dist[i*k + t] (fp32) are
 * ordered by (distance, index) ascending: equal distances go to the lower index. */
spd_status spd_knn(spd_handle *handle, const spd_csr *Q, const spd_csr *Index, spd_metric metric,
                   float p, int k, int64_t *out_idx, float *out_dist);

/* An index: the second operand of a distance, prepared once for many calls (Section 4.2's
 * protocol fits the whole dataset, then queries it batch by batch).  spd_index_create does what
 * every spd_pairwise / spd_knn call does for B - reads its row pointers back, bins its rows by
 * degree, repacks it and sums its row norms for `metric` (`p`: SPD_MINKOWSKI only) - into device
 * memory the index owns (about 8 bytes per stored entry and 40 per row); spd_index_pairwise /
 * spd_index_knn then return exactly what spd_pairwise / spd_knn return for the same operands.
 * The index keeps the pointers of `Index`, not a copy: the three arrays must stay valid and
 * unchanged until spd_index_destroy.  The work is enqueued on the creating handle's stream; use
 * the index with that handle (or, after synchronising its stream, with another handle on the same
 * device).  The planner options "split_len" and "window" are read at creation.
 * spd_index_destroy waits for the handle's stream before it frees the memory. */
spd_status spd_index_create(spd_handle *handle, const spd_csr *Index, spd_metric metric, float p,
                            spd_index **index);
spd_status spd_index_destroy(spd_handle *handle, spd_index *index);
spd_status spd_index_pairwise(spd_handle *handle, const spd_csr *A, const spd_index *index, float *out);
spd_status spd_index_knn(spd_handle *handle, const spd_csr *Q, const spd_index *index, int k,
                         int64_t *out_idx, float *out_dist);

/* Semirings (Section 2.2; the product and the sum that Section 4.2's interface passes to one
 * primitive).  A value between two rows is the sum() fold of product(x_c, y_c) over the columns c
 * both rows store, when 0 annihilates the product (the dot-product semiring is {TIMES, PLUS}; the
 * tropical semiring of Eq. 1 is {PLUS, MIN}); with `over_union` set, over the columns either row
 * stores, the missing side read as 0: the non-annihilating multiplicative monoid of Section 2.2
 * ({ABS_DIFF, PLUS} is the Manhattan distance, {ABS_DIFF, MAX} Chebyshev's).  A pair with no such
 * column gets the identity of sum(): 0, +infinity (MIN) or -infinity (MAX).  `transform` is applied
 * to every stored value first (a value it sends to 0 counts as absent), `epilogue` to the folded
 * value: together they spell every distance of Table 1, e.g.
 *   cosine          {TIMES, PLUS, 0, -, NONE, COSINE}        Hellinger  {TIMES, PLUS, 0, -, SQRT, HELLINGER}
 *   Jaccard         {TIMES, PLUS, 0, -, NONZERO, JACCARD}    Canberra   {CANBERRA, PLUS, 1, -, NONE, NONE}
 *   Minkowski       {ABS_DIFF_POW, PLUS, 1, p, NONE, ROOT_P} Hamming    {NOT_EQUAL, PLUS, 1, -, NONE, DIV_K}
 *   KL divergence   {X_LOG_X_OVER_Y, PLUS, 0, -, NONE, NONE} Jensen-Shannon {JS_TERM, PLUS, 1, -, NONE, SQRT_HALF}
 * A call that spells one of Table 1's distances runs on that distance's own kernels; any other
 * combination on kernels that take the product as a run-time choice.  Every product but
 * X_LOG_X_OVER_Y is commutative, as Section 2.2 asks of the union form. */
typedef enum {
    SPD_PRODUCT_TIMES = 0,  /* x * y     */
    SPD_PRODUCT_PLUS,       /* x + y     */
    SPD_PRODUCT_MIN,        /* min(x, y) */
    SPD_PRODUCT_MAX,        /* max(x, y) */
    SPD_PRODUCT_ABS_DIFF,   /* |x - y|   */
    SPD_PRODUCT_SQ_DIFF,    /* (x - y)^2 */
    SPD_PRODUCT_ABS_DIFF_POW,   /* |x - y|^p, p > 0 from the semiring                                   */
    SPD_PRODUCT_CANBERRA,       /* |x - y| / (|x| + |y|), 0 at (0, 0)                                   */
    SPD_PRODUCT_NOT_EQUAL,      /* 1 where x != y, else 0                                               */
    SPD_PRODUCT_X_LOG_X_OVER_Y, /* x log(x / y) where both are positive, else 0; over_union must be 0   */
    SPD_PRODUCT_JS_TERM,        /* x log(x/mu) + y log(y/mu), mu = (x + y)/2, 0 log 0 = 0; x, y >= 0    */
    SPD_PRODUCT_COUNT
} spd_product;

typedef enum { SPD_SUM_PLUS = 0, SPD_SUM_MIN, SPD_SUM_MAX, SPD_SUM_COUNT } spd_sum;

typedef enum { SPD_TRANSFORM_NONE = 0, SPD_TRANSFORM_SQRT, SPD_TRANSFORM_NONZERO /* 1 where the value is not 0 */,
               SPD_TRANSFORM_COUNT } spd_transform;

/* v: the folded value; x, y: the two rows after the transform; k: the number of columns. */
typedef enum {
    SPD_EPILOGUE_NONE = 0,      /* v                                                                    */
    SPD_EPILOGUE_ROOT_P,        /* v^(1/p)                                                              */
    SPD_EPILOGUE_DIV_K,         /* v / k                                                                */
    SPD_EPILOGUE_SQRT_HALF,     /* sqrt(v / 2)                                                          */
    /* The expansion functions over row norms (Table 1, Section 3.4) and the strict reading of the KL
     * divergence: each is accepted in the combination that makes it one of the library's distances
     * (the comment names product, sum, transform), and refused with SPD_ERR_BAD_METRIC otherwise.  */
    SPD_EPILOGUE_COSINE,        /* {TIMES, PLUS, NONE}: 1 - v/(|x|_2 |y|_2); 1 if one row is zero, 0 if both */
    SPD_EPILOGUE_L2,            /* {TIMES, PLUS, NONE}: sqrt(max(0, |x|_2^2 - 2v + |y|_2^2))              */
    SPD_EPILOGUE_CORRELATION,   /* {TIMES, PLUS, NONE}: 1 - Pearson correlation over k columns; 1 without variance */
    SPD_EPILOGUE_JACCARD,       /* {TIMES, PLUS, NONZERO or NONE}: 1 - v/(|x|_0 + |y|_0 - v); 0 if that is 0/0 */
    SPD_EPILOGUE_DICE,          /* {TIMES, PLUS, NONZERO}: 1 - 2v/(|x|_0 + |y|_0); 0 if both rows are empty */
    SPD_EPILOGUE_HELLINGER,     /* {TIMES, PLUS, SQRT}: sqrt(max(0, (|x|_2^2 + |y|_2^2)/2 - v))           */
    SPD_EPILOGUE_RUSSELL_RAO,   /* {TIMES, PLUS, NONZERO}: (k - v)/k                                      */
    SPD_EPILOGUE_STRICT,        /* {X_LOG_X_OVER_Y, PLUS, NONE}: v if y is positive wherever x is, else +infinity */
    SPD_EPILOGUE_COUNT
} spd_epilogue;

typedef struct {
    spd_product product;
    spd_sum sum;
    int over_union;         /* 0: columns stored in both rows; 1: in either row */
    float p;                /* degree of SPD_PRODUCT_ABS_DIFF_POW and SPD_EPILOGUE_ROOT_P (finite, > 0); ignored otherwise */
    spd_transform transform;
    spd_epilogue epilogue;
} spd_semiring;

/* out[i * B.n_rows + j] = the semiring's value between A_i and B_j, fp32, row-major, m x n.
 * An unknown product, sum, transform or epilogue, X_LOG_X_OVER_Y over the union, or an expansion
 * epilogue outside its combination returns SPD_ERR_BAD_METRIC; a degree that is needed and is
 * not a finite p > 0 returns SPD_ERR_BAD_P.  Scratch: the bound spd_workspace_bytes()
 * gives for SPD_MINKOWSKI covers every semiring. */
spd_status spd_semiring_pairwise(spd_handle *handle, const spd_csr *A, const spd_csr *B,
                                 const spd_semiring *semiring, float *out);

/* For each query row the k index rows with the smallest semiring value, ordered by (value,
 * index) ascending, selected inside the kernels like spd_knn's. */
spd_status spd_semiring_knn(spd_handle *handle, const spd_csr *Q, const spd_csr *Index,
                            const spd_semiring *semiring, int k, int64_t *out_idx, float *out_dist);

/* Device pass over a matrix that checks what the other calls assume: row pointers start
 * at 0, never decrease and end at nnz; columns ascend strictly inside a row and lie in
 * [0, n_cols); values are finite (and, if `require_nonnegative`, not negative).
 * Synchronises the stream.  Returns SPD_ERR_BAD_CSR if a check fails. */
spd_status spd_csr_validate(spd_handle *handle, const spd_csr *M, int require_nonnegative);

/* Planner knobs, mainly for tests that need to reach a particular staging path:
 *   "lds_budget"  bytes of LDS a workgroup may use (default: the device limit)
 *   "force_kind"  0 auto, 1 dense strip, 2 column-slot strip, 3 hash, 4 Bloom filter (every row of A
 *                 alone in a workgroup, its columns in a Bloom filter in LDS, its values looked up in
 *                 global memory by binary search: Section 3.3.2's alternative; not for Chebyshev or the
 *                 semirings whose sum() is min or max), 5 bitmap of the staged columns with running
 *                 counts (a column's slot is the number of staged columns below it)
 *   "bloom_long_rows" 1: a row of A too long to be staged whole gets a Bloom filter instead of being
 *                 cut into slices (default 0: measured slower than slices on every shape tried)
 *   "max_rows"    largest number of A rows staged together (1, 2, 4, 8 or 16; the set metrics,
 *                 whose rows take a byte each in the staged table, stage four times as many,
 *                 up to 32; with fused k-NN 16, or 32 for max_rows = 16)
 *   "split_len"   B rows at least this long are split over several lanes (0 = automatic: 256,
 *                 or 512 when B has 2^22 stored entries or more)
 *   "window"      rows of the streamed operand per degree-sorting window (0 = automatic: 2,048 for a
 *                 pairwise call that stages A, whose stores want the rows of a slab near each other;
 *                 and for an index, which serves such calls too; 65,536 for k-NN calls and for pairwise
 *                 calls with the operands' roles exchanged, where a wide window only means fewer idle lanes)
 *   "chunks"      number of B chunks (0 = automatic)
 *   "chunk_scale" the automatic number of chunks is the cost model's times this (1 to 8; 0 = automatic:
 *                 2 for k-NN calls, whose lists do better on shorter chunks, 1 for pairwise calls)
 *   "sort_slack"  1 (default): inside a window B's rows are sorted by their length in blocks of four
 *                 entries, and by row number among equals (neighbouring rows then share slabs and
 *                 their results share cache lines); 0: by their exact length
 *   "partial_groups" 1 (default): where 4 rows of A are too much for the LDS but 3 are not, they
 *                 are staged as a group of 4 with a place left empty instead of two groups of 2
 *                 (not for Chebyshev and the semirings with sum() = min or max; for the set
 *                 metrics at any group size, three quarters filled); 2: also 6 rows in a group
 *                 of 8 for the dot product, L1 and Hamming; 0: a group is full or halved
 *   "byte_counters" 1 (default): Jaccard, Dice and Russell-Rao count shared columns in byte lanes,
 *                 four staged rows to the 32-bit word; 0: through the dot product of 0/1 values
 *   "waves_per_cu" wavefronts a launch aims to keep on a compute unit: 8, 16 or 32 (0 = automatic: 32)
 *   "side_streams" how many internal streams (0 to 3; default 3) the launches that are small against
 *                 the call's largest one may use beside it, forked and joined with events so that
 *                 the handle's stream still orders the whole call (0: everything on the handle's stream);
 *                 they are used when the largest launch is short or the small ones hold a tenth of
 *                 the call's sweeps over B, and not otherwise
 *   "cuckoo_attempts" hash staging of a half-full table tries up to three pairs of hash functions
 *                 before it falls back to linear probing (3, the default); fewer, down to 0 (linear
 *                 probing at once), let a test reach that fall-back, which no input has needed so far
 *   "knn_seed"    fused top-k of the distances that grow with a row's mass (L1, Minkowski, Canberra,
 *                 Hamming, Jensen-Shannon, Chebyshev, expanded Euclidean, Hellinger): 1 (default) lets the wavefronts of a workgroup
 *                 agree on a first bound of the k-th distance from the shortest rows of their share
 *                 of B before any candidate is queued (the result does not depend on it); 0 starts
 *                 every list with no bound
 *   "swap_operands" spd_pairwise may stage B and stream A instead of the other way round (every distance
 *                 but the two KL divergences is symmetric in its rows): B's rows are then staged in
 *                 groups of consecutive rows, so that a lane's results are neighbours in the output
 *                 and are stored as whole 32-byte sectors.  1 (default): where it pays (A of 2^18 or
 *                 more stored entries and 1,024 or more rows, B's rows under 96 entries on average);
 *                 0: never; 2: wherever the distance allows it
 *   "check_plan"  1: verify every index the kernels will form from the plan before launching
 *   "profile"     1: bracket every kernel launch with HIP events (see spd_profile_read)
 * Unknown names or values out of range return SPD_ERR_UNSUPPORTED. */
spd_status spd_set_option(spd_handle *handle, const char *name, int64_t value);

/* Kernel timings of the last spd_pairwise / spd_knn call made with option "profile" = 1.
 * One record per launch, in launch order.  Waits for the call's kernels to finish. */
typedef struct {
    char name[24];        /* "pack_b", "scan", "finalize", "knn_merge"                   */
    int32_t rows_per_group; /* scan: R, the rows of A staged together; else 0            */
    int32_t staging_kind; /* scan: 1 dense strip, 2 column-slot strip, 3 hash, 4 Bloom, 5 bitmap; else 0 */
    int32_t block;        /* scan: threads per workgroup; else 0                          */
    int32_t lds_bytes;    /* scan: dynamic LDS per workgroup; else 0                      */
    int64_t a_rows;       /* scan: rows (or slices of rows) of A the launch covers        */
    int64_t workgroups;
    double ms;            /* HIP-event time of the launch on the handle's stream          */
} spd_kernel_time;
/* Writes at most `cap` records to `out`, returns how many the call produced (<0: error). */
int spd_profile_read(spd_handle *handle, spd_kernel_time *out, int cap);

const char *spd_last_error(const spd_handle *handle);
const char *spd_metric_name(spd_metric metric);
const char *spd_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPD_H */
