// C-ABI of the library (include/spd.h): argument checks, planning on the host, scratch
// layout, and the sequence of launches of one spd_pairwise / spd_knn call.
#include <hip/hip_runtime.h>

#include <chrono>
#include <cmath>
#include <cstdlib>
#include <cstdio>
#include <cstring>
#include <atomic>
#include <condition_variable>
#include <functional>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

#include "../../include/spd.h"
#include "spd_kernels.h"
#include "spd_plan.h"

using namespace spd;

// Scratch of the entry point that allocates nothing (spd_pairwise_static): one array per GPU, held
// from the moment the library's code is loaded on that GPU until the process ends.  In host code
// the array's name is only a stand-in for the symbol; the address a kernel can use is asked for
// once per device (spd_create, with that device current) and kept in g_static_scratch.
constexpr size_t kStaticScratchBytes = (size_t)SPD_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kStaticScratchDevices = 64;
static void *g_static_scratch[kStaticScratchDevices];
static std::mutex g_static_scratch_mutex;
// Pinned staging memory every handle holds from its creation, so that a call may not have to
// allocate any: three buffers of this size.
constexpr size_t kInitialPinnedBytes = (size_t)SPD_STATIC_STAGING_BYTES;

// A helper thread that runs one job at a time beside the caller's thread (the plan of A is
// made there while the caller plans B, uploads its plan and starts the repack).  A sleeping
// thread can take longer to wake than the job takes: when the caller comes to wait and the
// helper has not begun yet, the caller runs the job itself.
class Helper {
public:
    ~Helper() {
        if (!th_.joinable()) return;
        { std::lock_guard<std::mutex> g(m_); quit_ = true; }
        cv_.notify_all();
        th_.join();
    }
    void post(std::function<void()> job) {
        if (!th_.joinable()) th_ = std::thread([this] { loop(); });
        { std::lock_guard<std::mutex> g(m_); job_ = std::move(job); state_ = kPosted; posted_.store(true, std::memory_order_release); }
        cv_.notify_all();
    }
    void wait() {
        std::unique_lock<std::mutex> g(m_);
        if (state_ == kPosted) {                 // not begun: do it here
            state_ = kRunning;
            posted_.store(false, std::memory_order_relaxed);
            std::function<void()> job = std::move(job_);
            g.unlock();
            job();
            g.lock();
            state_ = kIdle;
            return;
        }
        cv_.wait(g, [this] { return state_ == kIdle; });
    }
private:
    enum State { kIdle, kPosted, kRunning };
    void loop() {
        std::unique_lock<std::mutex> g(m_);
        for (;;) {
            // calls tend to come back to back: look out for the next job for a little while
            // before going to sleep (waking a sleeping thread takes as long as a small plan)
            if (state_ != kPosted && !quit_) {
                g.unlock();
                const auto until = std::chrono::steady_clock::now() + std::chrono::microseconds(kSpinMicros);
                while (!posted_.load(std::memory_order_acquire) && std::chrono::steady_clock::now() < until) {
#if defined(__x86_64__)
                    __builtin_ia32_pause();
#endif
                }
                g.lock();
            }
            cv_.wait(g, [this] { return state_ == kPosted || quit_; });
            posted_.store(false, std::memory_order_relaxed);
            if (quit_) return;
            state_ = kRunning;
            std::function<void()> job = std::move(job_);
            g.unlock();
            job();
            g.lock();
            state_ = kIdle;
            cv_.notify_all();
        }
    }
    std::thread th_;
    std::mutex m_;
    std::condition_variable cv_;
    std::function<void()> job_;
    State state_ = kIdle;
    bool quit_ = false;
    std::atomic<bool> posted_{false};           // what the helper polls while it spins
    static constexpr int kSpinMicros = 300;
};

struct spd_handle {
    hipStream_t stream = nullptr;
    int device = 0;
    PlanOptions opt;
    std::string err;
    // Pinned staging memory: three buffers taken in turn, so that a call may fill one while the
    // copies of the calls before it are still waiting in the stream.  `pinned` is the one the
    // current call holds.
    struct PinnedSlot { void *ptr = nullptr; size_t bytes = 0; hipEvent_t done = nullptr; bool pending = false; };
    static constexpr int kPinnedSlots = 3;
    PinnedSlot pinned_slots[kPinnedSlots];
    int pinned_next = 0, pinned_held = -1;
    void *pinned = nullptr;
    size_t pinned_bytes = 0;
    void *ws = nullptr;          // device scratch in use
    size_t ws_bytes = 0;
    bool ws_external = false;
    void *own_ws = nullptr;      // the handle's own allocation
    size_t own_ws_bytes = 0;
    int32_t *flag = nullptr;     // device word for spd_csr_validate
    void *static_ws = nullptr;   // this device's copy of `scratch`
    bool no_alloc = false;       // inside spd_pairwise_static: nothing may be allocated
    bool profile = false;
    bool check_plan = false;
    bool no_byte_counters = false;   // option "byte_counters" 0: set metrics through the dot product
    int cuckoo_attempts = 3;     // option "cuckoo_attempts"
    int knn_seed = 1;            // option "knn_seed"
    int swap_operands = 1;       // option "swap_operands": 0 never, 1 where it pays, 2 wherever the distance allows it
    int side_streams = 3;        // option "side_streams": how many internal streams the small launches may use beside the large one
    static constexpr int kSideStreams = 3;
    hipStream_t side[kSideStreams] = {nullptr, nullptr, nullptr};
    hipEvent_t fork_event = nullptr, join_event[kSideStreams] = {nullptr, nullptr, nullptr};     // full consistency check of every plan before launching
    struct Timed { spd_kernel_time rec; hipEvent_t start, stop; };
    std::vector<Timed> timed;    // launches of the last call (profile mode)
    std::vector<hipEvent_t> event_pool;
    APlan plan_of_a;             // kept between calls: the planner reuses their buffers
    BPlan plan_of_b;
    Helper helper;
    std::vector<int64_t> knn_row_off;
    std::vector<int32_t> knn_row_lists;
};

// B of a distance, planned and repacked once (spd_index_create): the plan on the host, and on
// the device the plan's arrays, the packed slabs and the row norms in one allocation.
struct spd_index {
    spd_csr matrix;              // the caller's arrays (they must stay valid and unchanged)
    int metric = 0;
    float p = 1.0f;
    int device = 0;
    BPlan plan;
    void *dev = nullptr;
    size_t dev_bytes = 0;
    BDevice bd;
};

namespace {

const char *const kMetricNames[SPD_METRIC_COUNT] = {
    "inner_product", "cosine", "l2_expanded", "correlation", "jaccard", "dice", "hellinger", "l1",
    "chebyshev", "minkowski", "canberra", "hamming", "kl_divergence", "jensen_shannon", "russell_rao",
    "l2_unexpanded", "kl_divergence_strict", "jaccard_literal"};

spd_status fail(spd_handle *h, spd_status st, const std::string &msg) {
    if (h) h->err = msg;
    return st;
}

spd_status hip_fail(spd_handle *h, hipError_t e, const char *where) {
    return fail(h, SPD_ERR_HIP, std::string(where) + ": " + hipGetErrorString(e));
}

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// Sequential carving of the scratch buffer.
struct Carver {
    size_t off = 0;
    size_t take(size_t bytes) { size_t at = off; off = align256(off + bytes); return at; }
};

spd_status check_csr_args(spd_handle *h, const spd_csr *M, const char *name) {
    if (!M) return fail(h, SPD_ERR_NULL, std::string(name) + " is NULL");
    if (M->n_rows < 0 || M->n_cols < 0 || M->nnz < 0)
        return fail(h, SPD_ERR_DIM_MISMATCH, std::string(name) + " has a negative size");
    if (!M->indptr) return fail(h, SPD_ERR_NULL, std::string(name) + ".indptr is NULL");
    if (M->nnz > 0 && (!M->indices || !M->values))
        return fail(h, SPD_ERR_NULL, std::string(name) + ".indices / .values is NULL");
    if (M->n_rows >= ((int64_t)1 << 31) - 1 || M->n_cols >= ((int64_t)1 << 31) - 1)
        return fail(h, SPD_ERR_UNSUPPORTED, std::string(name) + ": more than 2^31-2 rows or columns");
    if (M->nnz >= ((int64_t)1 << 40))
        return fail(h, SPD_ERR_UNSUPPORTED, std::string(name) + ": more than 2^40 stored entries");
    return SPD_OK;
}

// The distance of Table 1 (or one of the library's variants of them) that a semiring call spells,
// or -1: such a call runs on the distance's own kernels.  The inner product is left out for k-NN
// (spd_knn returns its largest values, spd_semiring_knn the smallest), and so is Chebyshev, whose
// value between two empty rows is 0 where the semiring's is the identity of max.
int table1_metric(const spd_semiring &s, bool knn) {
    if (s.sum != SPD_SUM_PLUS) return -1;
    const int T = (int)s.transform, E = (int)s.epilogue;
    const bool U = s.over_union != 0;
    switch (s.product) {
    case SPD_PRODUCT_TIMES:          // (0 annihilates: the union adds nothing to the intersection)
        if (T == SPD_TRANSFORM_NONE) {
            if (E == SPD_EPILOGUE_NONE) return knn ? -1 : (int)SPD_INNER_PRODUCT;
            if (E == SPD_EPILOGUE_COSINE) return SPD_COSINE;
            if (E == SPD_EPILOGUE_L2) return SPD_L2_EXPANDED;
            if (E == SPD_EPILOGUE_CORRELATION) return SPD_CORRELATION;
            if (E == SPD_EPILOGUE_JACCARD) return SPD_JACCARD_LITERAL;
        } else if (T == SPD_TRANSFORM_NONZERO) {
            if (E == SPD_EPILOGUE_JACCARD) return SPD_JACCARD;
            if (E == SPD_EPILOGUE_DICE) return SPD_DICE;
            if (E == SPD_EPILOGUE_RUSSELL_RAO) return SPD_RUSSELL_RAO;
        } else if (T == SPD_TRANSFORM_SQRT) {
            if (E == SPD_EPILOGUE_HELLINGER) return SPD_HELLINGER;
        }
        return -1;
    case SPD_PRODUCT_ABS_DIFF: return (U && T == SPD_TRANSFORM_NONE && E == SPD_EPILOGUE_NONE) ? (int)SPD_L1 : -1;
    case SPD_PRODUCT_ABS_DIFF_POW: return (U && T == SPD_TRANSFORM_NONE && E == SPD_EPILOGUE_ROOT_P) ? (int)SPD_MINKOWSKI : -1;
    case SPD_PRODUCT_SQ_DIFF:
        return (U && T == SPD_TRANSFORM_NONE && E == SPD_EPILOGUE_ROOT_P && s.p == 2.0f) ? (int)SPD_L2_UNEXPANDED : -1;
    case SPD_PRODUCT_CANBERRA: return (U && T == SPD_TRANSFORM_NONE && E == SPD_EPILOGUE_NONE) ? (int)SPD_CANBERRA : -1;
    case SPD_PRODUCT_NOT_EQUAL: return (U && T == SPD_TRANSFORM_NONE && E == SPD_EPILOGUE_DIV_K) ? (int)SPD_HAMMING : -1;
    case SPD_PRODUCT_X_LOG_X_OVER_Y:
        if (U || T != SPD_TRANSFORM_NONE) return -1;
        return E == SPD_EPILOGUE_NONE ? (int)SPD_KL_DIVERGENCE : (E == SPD_EPILOGUE_STRICT ? (int)SPD_KL_STRICT : -1);
    case SPD_PRODUCT_JS_TERM: return (U && T == SPD_TRANSFORM_NONE && E == SPD_EPILOGUE_SQRT_HALF) ? (int)SPD_JENSEN_SHANNON : -1;
    default: return -1;
    }
}

spd_status check_call_args(spd_handle *h, const spd_csr *A, const spd_csr *B, spd_metric metric, float p, int knn_k,
                           bool is_knn, const void *o1, const void *o2, const spd_semiring *semiring = nullptr,
                           bool is_semiring = false) {
    if (!h) return SPD_ERR_NULL;
    h->err.clear();
    spd_status st = check_csr_args(h, A, is_knn ? "Q" : "A");
    if (st != SPD_OK) return st;
    st = check_csr_args(h, B, is_knn ? "Index" : "B");
    if (st != SPD_OK) return st;
    if (A->n_cols != B->n_cols) return fail(h, SPD_ERR_DIM_MISMATCH, "the two matrices differ in n_cols");
    if (is_semiring) {
        if (!semiring) return fail(h, SPD_ERR_NULL, "semiring is NULL");
        if ((int)semiring->product < 0 || (int)semiring->product >= SPD_PRODUCT_COUNT)
            return fail(h, SPD_ERR_BAD_METRIC, "unknown product");
        if ((int)semiring->sum < 0 || (int)semiring->sum >= SPD_SUM_COUNT) return fail(h, SPD_ERR_BAD_METRIC, "unknown sum");
        if ((int)semiring->transform < 0 || (int)semiring->transform >= SPD_TRANSFORM_COUNT)
            return fail(h, SPD_ERR_BAD_METRIC, "unknown transform");
        if ((int)semiring->epilogue < 0 || (int)semiring->epilogue >= SPD_EPILOGUE_COUNT)
            return fail(h, SPD_ERR_BAD_METRIC, "unknown epilogue");
        if (semiring->product == SPD_PRODUCT_X_LOG_X_OVER_Y && semiring->over_union)
            return fail(h, SPD_ERR_BAD_METRIC, "x log(x/y) has no value where y is absent: it is offered over the columns both rows store");
        if ((semiring->product == SPD_PRODUCT_ABS_DIFF_POW || semiring->epilogue == SPD_EPILOGUE_ROOT_P) &&
            !(semiring->p > 0.0f && std::isfinite(semiring->p)))
            return fail(h, SPD_ERR_BAD_P, "the semiring needs a finite degree p > 0");
        if (semiring->epilogue > SPD_EPILOGUE_SQRT_HALF && table1_metric(*semiring, false) < 0)
            return fail(h, SPD_ERR_BAD_METRIC, "this epilogue is an expansion over row norms: it is defined for the product, "
                                               "sum and transform of its own distance only");
    } else {
        if ((int)metric < 0 || (int)metric >= SPD_METRIC_COUNT) return fail(h, SPD_ERR_BAD_METRIC, "unknown metric");
        if (metric == SPD_MINKOWSKI && !(p > 0.0f && std::isfinite(p)))
            return fail(h, SPD_ERR_BAD_P, "Minkowski needs a finite p > 0");
    }
    if (is_knn) {
        if (knn_k < 1 || (int64_t)knn_k > B->n_rows || knn_k > SPD_KNN_MAX_K)
            return fail(h, SPD_ERR_BAD_K, "k must lie in [1, min(Index.n_rows, SPD_KNN_MAX_K)]");
        if (A->n_rows > 0 && (!o1 || !o2)) return fail(h, SPD_ERR_NULL, "out_idx / out_dist is NULL");
    } else {
        if (A->n_rows > 0 && B->n_rows > 0 && !o1) return fail(h, SPD_ERR_NULL, "out is NULL");
    }
    return SPD_OK;
}

// Holds one of the handle's pinned buffers for the length of a call: waits until the copies the
// buffer's last call enqueued have run, and on the way out marks the point in the stream after
// which it may be written again.
struct PinnedLease {
    spd_handle *h;
    explicit PinnedLease(spd_handle *hh) : h(hh) {
        const int i = h->pinned_next;
        h->pinned_next = (i + 1) % spd_handle::kPinnedSlots;
        spd_handle::PinnedSlot &s = h->pinned_slots[i];
        if (s.pending) { (void)hipEventSynchronize(s.done); s.pending = false; }
        h->pinned = s.ptr;
        h->pinned_bytes = s.bytes;
        h->pinned_held = i;
    }
    ~PinnedLease() {
        spd_handle::PinnedSlot &s = h->pinned_slots[h->pinned_held];
        s.ptr = h->pinned;
        s.bytes = h->pinned_bytes;
        if (!s.done && hipEventCreateWithFlags(&s.done, hipEventDisableTiming) != hipSuccess) s.done = nullptr;
        if (s.done && hipEventRecord(s.done, h->stream) == hipSuccess) s.pending = true;
        else (void)hipStreamSynchronize(h->stream);       // no event: fall back to waiting here
        h->pinned = nullptr;
        h->pinned_bytes = 0;
        h->pinned_held = -1;
    }
    PinnedLease(const PinnedLease &) = delete;
    PinnedLease &operator=(const PinnedLease &) = delete;
};

spd_status ensure_pinned(spd_handle *h, size_t bytes) {
    if (bytes <= h->pinned_bytes) return SPD_OK;
    if (h->no_alloc)
        return fail(h, SPD_ERR_WORKSPACE, "operands too large for the entry point that allocates nothing: the plan needs " +
                                              std::to_string(bytes) + " bytes of staging memory, a handle holds " +
                                              std::to_string(h->pinned_bytes));
    if (h->pinned) { hipError_t e = hipStreamSynchronize(h->stream); (void)e; (void)hipHostFree(h->pinned); h->pinned = nullptr; h->pinned_bytes = 0; }
    size_t want = align256(bytes + bytes / 4);
    hipError_t e = hipHostMalloc(&h->pinned, want, hipHostMallocDefault);
    if (e != hipSuccess) return hip_fail(h, e, "hipHostMalloc");
    h->pinned_bytes = want;
    return SPD_OK;
}

spd_status ensure_workspace(spd_handle *h, size_t bytes) {
    if (h->ws_external) {
        if (bytes > h->ws_bytes)
            return fail(h, SPD_ERR_WORKSPACE,
                        h->no_alloc ? "operands too large for the entry point that allocates nothing: they need " +
                                          std::to_string(bytes) + " bytes of scratch, the static array holds " +
                                          std::to_string(h->ws_bytes)
                                    : "caller workspace too small: need " + std::to_string(bytes) + " bytes");
        return SPD_OK;
    }
    if (bytes > h->own_ws_bytes) {
        if (h->own_ws) {
            hipError_t e = hipStreamSynchronize(h->stream);
            if (e != hipSuccess) return hip_fail(h, e, "hipStreamSynchronize");
            (void)hipFree(h->own_ws);
            h->own_ws = nullptr; h->own_ws_bytes = 0;
        }
        size_t want = align256(bytes + bytes / 8);
        hipError_t e = hipMalloc(&h->own_ws, want);
        if (e != hipSuccess) return fail(h, SPD_ERR_WORKSPACE, std::string("hipMalloc of scratch failed: ") + hipGetErrorString(e));
        h->own_ws_bytes = want;
    }
    h->ws = h->own_ws;
    h->ws_bytes = h->own_ws_bytes;
    return SPD_OK;
}

// Profile mode: events around one launch.
struct LaunchTimer {
    spd_handle *h;
    bool on;
    spd_handle::Timed t;
    hipStream_t stream;
    LaunchTimer(spd_handle *hh, const char *name, int R, int kind, int block, uint32_t lds, int64_t a_rows, int64_t wgs,
                hipStream_t st = nullptr)
        : h(hh), on(hh->profile), stream(st ? st : hh->stream) {
        if (!on) return;
        std::memset(&t.rec, 0, sizeof t.rec);
        std::snprintf(t.rec.name, sizeof t.rec.name, "%s", name);
        t.rec.rows_per_group = R; t.rec.staging_kind = kind; t.rec.block = block; t.rec.lds_bytes = (int32_t)lds;
        t.rec.a_rows = a_rows; t.rec.workgroups = wgs; t.rec.ms = -1.0;
        auto get = [&](hipEvent_t &e) {
            if (!h->event_pool.empty()) { e = h->event_pool.back(); h->event_pool.pop_back(); return true; }
            return hipEventCreate(&e) == hipSuccess;
        };
        if (!get(t.start) || !get(t.stop)) { on = false; return; }
        (void)hipEventRecord(t.start, stream);
    }
    void done() {
        if (!on) return;
        (void)hipEventRecord(t.stop, stream);
        h->timed.push_back(t);
    }
};

// Everything one call uploads, laid out in one pinned blob mirrored 1:1 in the scratch.
struct Upload {
    std::vector<std::pair<size_t, std::pair<const void *, size_t>>> parts;   // scratch offset, (src, bytes)
    void add(size_t off, const void *src, size_t bytes) { if (bytes) parts.push_back({off, {src, bytes}}); }
};

size_t workspace_bound(const spd_handle *h, const spd_csr *A, const spd_csr *B, int metric, int k_neighbors);

// Where B's plan, its packed slabs and its norms sit in a device buffer: the plan's arrays first,
// contiguous, so that one copy moves them.
struct BLayout {
    size_t slab_base, slab_steps, slab_split, seg_start, seg_len, seg_row, seg_glog, plan_end, packed, norms, end;
};

BLayout layout_b(const BPlan &bp, int64_t n, Carver &cv) {
    const size_t lanes = (size_t)bp.n_slabs * kWave;
    BLayout L;
    L.slab_base = cv.take(bp.slab_base.size() * 8);
    L.slab_steps = cv.take(bp.slab_steps.size() * 4);
    L.slab_split = cv.take(bp.slab_split.size());
    L.seg_start = cv.take(lanes * 8);
    L.seg_len = cv.take(lanes * 4);
    L.seg_row = cv.take(lanes * 4);
    L.seg_glog = cv.take(lanes);
    L.plan_end = cv.off;
    L.packed = cv.take((size_t)bp.slab_base[(size_t)bp.n_slabs] * 8);
    L.norms = cv.take((size_t)n * 16);
    L.end = cv.off;
    return L;
}

// Copies B's plan through the pinned buffer at `pin` into the device buffer `dev` (laid out by
// `L`) and starts the repack there.  Everything is enqueued on the handle's stream.
spd_status stage_b_into(spd_handle *h, const spd_csr *B, const BPlan &bp, const BLayout &L, unsigned char *dev,
                        unsigned char *pin, int metric, const MetricInfo &mi, const OpParams &q, uint32_t padcol,
                        BDevice &bd) {
    const size_t lanes = (size_t)bp.n_slabs * kWave;
    auto put = [&](size_t off, const void *src, size_t bytes) { if (bytes) std::memcpy(pin + off, src, bytes); };
    put(L.slab_base, bp.slab_base.data(), bp.slab_base.size() * 8);
    put(L.slab_steps, bp.slab_steps.data(), bp.slab_steps.size() * 4);
    put(L.slab_split, bp.slab_split.data(), bp.slab_split.size());
    put(L.seg_start, bp.seg_start.data(), lanes * 8);
    put(L.seg_len, bp.seg_len.data(), lanes * 4);
    put(L.seg_row, bp.seg_row.data(), lanes * 4);
    put(L.seg_glog, bp.seg_glog.data(), lanes);
    if (L.plan_end) {
        hipError_t err = hipMemcpyAsync(dev, pin, L.plan_end, hipMemcpyHostToDevice, h->stream);
        if (err != hipSuccess) return hip_fail(h, err, "upload of B's plan");
    }
    bd.packed = reinterpret_cast<const uint2 *>(dev + L.packed);
    bd.slab_base = reinterpret_cast<const int64_t *>(dev + L.slab_base);
    bd.slab_steps = reinterpret_cast<const int32_t *>(dev + L.slab_steps);
    bd.slab_split = dev + L.slab_split;
    bd.seg_start = reinterpret_cast<const int64_t *>(dev + L.seg_start);
    bd.seg_len = reinterpret_cast<const int32_t *>(dev + L.seg_len);
    bd.seg_row = reinterpret_cast<const int32_t *>(dev + L.seg_row);
    bd.seg_glog = dev + L.seg_glog;
    bd.norms = reinterpret_cast<const double *>(dev + L.norms);
    bd.n_slabs = bp.n_slabs;
    bd.n_rows = B->n_rows;
    LaunchTimer lt(h, "pack_b", 0, 0, 0, 0, 0, bp.n_slabs);
    hipError_t err = launch_pack_b(h->stream, B->indptr, B->indices, B->values, bd, reinterpret_cast<uint2 *>(dev + L.packed),
                                   reinterpret_cast<double *>(dev + L.norms), metric, mi.transform, mi.norm, q.p, q.k, padcol);
    if (err != hipSuccess) return hip_fail(h, err, "pack kernel");
    lt.done();
    return SPD_OK;
}

// The parameters of a metric's product as the kernels read them.
OpParams op_params(int metric, float p, int64_t n_cols, const spd_semiring *semiring) {
    OpParams q;
    q.p = p;
    if (metric == SPD_L2_UNEXPANDED) q.p = 2.0f;
    q.inv_p = (metric == SPD_MINKOWSKI) ? 1.0f / p : (metric == SPD_L2_UNEXPANDED ? 0.5f : 1.0f);
    q.k = (double)n_cols;
    q.metric = metric;
    if (metric != SPD_MINKOWSKI && metric != SPD_L2_UNEXPANDED) q.p = 1.0f;
    if (semiring) {
        q.product = (int)semiring->product;
        q.over_union = semiring->over_union != 0;
        q.sign = semiring->sum == SPD_SUM_MIN ? -1.0f : 1.0f;
        q.epilogue = (int)semiring->epilogue;          // (only the first four reach the kernels)
        if (semiring->product == SPD_PRODUCT_ABS_DIFF_POW || semiring->epilogue == SPD_EPILOGUE_ROOT_P) {
            q.p = semiring->p;
            q.inv_p = 1.0f / semiring->p;
        }
    }
    return q;
}

// The metric a call runs as (Minkowski of degree 1 is the Manhattan distance, whose product is
// a third of the work).
int effective_metric(int metric, float p) { return (metric == SPD_MINKOWSKI && p == 1.0f) ? (int)SPD_L1 : metric; }

// `metric` is a spd_metric, or, with `semiring` set, the internal id its sum() runs as.  With
// `index` set, B is that index's matrix and its plan, packed slabs and norms are taken from it.
// Whether a pairwise call stages B and streams A instead of the other way round.  A lane holds
// the results of one streamed row against the R staged rows; with A staged these are R different
// rows of the output and the 64 lanes of a store fall on 64 different cache lines (the streamed
// rows of a slab are the ones of similar length inside a window, not neighbours), which costs
// three times the output in write traffic.  With B staged in groups of consecutive rows a lane's
// R results are neighbours in its own output row: whole 32-byte sectors.  The roles can be
// exchanged for every distance that is symmetric in its two rows, and pay where the scan of a pair
// is short against its store (short rows of B) and A is large enough to be worth sweeping.
bool operands_may_swap(int metric, const spd_semiring *semiring) {
    if (semiring && semiring->product == SPD_PRODUCT_X_LOG_X_OVER_Y) return false;
    return metric != SPD_KL_DIVERGENCE && metric != SPD_KL_STRICT;
}
bool operands_swap_pays(const spd_csr *A, const spd_csr *B) {
    return A->nnz >= ((int64_t)1 << 18) && A->n_rows >= 1024 && B->nnz <= 96 * B->n_rows;
}

spd_status run(spd_handle *h, const spd_csr *A, const spd_csr *B, int metric, float p, const spd_semiring *semiring,
               int knn_k, float *out, int64_t *out_idx, float *out_dist, const spd_index *index = nullptr) {
    metric = effective_metric(metric, p);
    const bool swapped = knn_k == 0 && !index && operands_may_swap(metric, semiring) &&
                         (h->swap_operands == 2 || (h->swap_operands == 1 && operands_swap_pays(A, B)));
    if (swapped) std::swap(A, B);           // from here on A is the staged operand, B the streamed one
    const int64_t m = A->n_rows, n = B->n_rows;
    const int64_t out_stride_staged = swapped ? 1 : n, out_stride_streamed = swapped ? m : 1;
    static const bool host_times = std::getenv("SPD_HOST_TIMES") != nullptr;
    auto now = [] { return std::chrono::steady_clock::now(); };
    auto t_begin = now();
    auto lap = [&](const char *what) {
        if (!host_times) return;
        auto t = now();
        std::fprintf(stderr, "[spd host] %-12s %8.1f us\n", what, std::chrono::duration<double, std::micro>(t - t_begin).count());
        t_begin = t;
    };
    for (auto &t : h->timed) { h->event_pool.push_back(t.start); h->event_pool.push_back(t.stop); }
    h->timed.clear();
    if (m == 0 || n == 0) return SPD_OK;
    hipError_t e = hipSetDevice(h->device);
    if (e != hipSuccess) return hip_fail(h, e, "hipSetDevice");

    // ---- row pointers on the host: the caller's copies, or read back (the call's only
    //      synchronisation) ----------------------------------------------------------------
    PinnedLease lease(h);
    const bool same = !index && A->indptr == B->indptr && m == n;
    const int64_t *a_host = A->host_indptr ? A->host_indptr : (same ? B->host_indptr : nullptr);
    const int64_t *b_host = index ? nullptr : (B->host_indptr ? B->host_indptr : (same ? A->host_indptr : nullptr));
    const bool copy_a = !a_host;
    const bool copy_b = !index && !same && !b_host;
    const size_t ip_bytes = (copy_a ? (size_t)(m + 1) * 8 : 0) + (copy_b ? (size_t)(n + 1) * 8 : 0);
    // (sized for the two plan uploads as well, which follow the row pointers in the buffer)
    spd_status st = ensure_pinned(h, ip_bytes + (index ? 0 : 32 * ((size_t)n + 4096)) + 48 * ((size_t)m + 4096));
    if (st != SPD_OK) return st;
    // where the two arrays are read from: the caller's memory, or the start of the pinned buffer
    auto locate = [&](const int64_t *&a_at, const int64_t *&b_at) {
        int64_t *pin = reinterpret_cast<int64_t *>(h->pinned);
        a_at = a_host ? a_host : pin;
        b_at = b_host ? b_host : (same ? a_at : pin + (copy_a ? m + 1 : 0));
    };
    const int64_t *a_ip = nullptr, *b_ip = nullptr;
    locate(a_ip, b_ip);
    if (copy_a) {
        e = hipMemcpyAsync(const_cast<int64_t *>(a_ip), A->indptr, (size_t)(m + 1) * 8, hipMemcpyDeviceToHost, h->stream);
        if (e != hipSuccess) return hip_fail(h, e, "copy of A.indptr");
    }
    if (copy_b) {
        e = hipMemcpyAsync(const_cast<int64_t *>(b_ip), B->indptr, (size_t)(n + 1) * 8, hipMemcpyDeviceToHost, h->stream);
        if (e != hipSuccess) return hip_fail(h, e, "copy of B.indptr");
    }
    if (copy_a || copy_b) {
        e = hipStreamSynchronize(h->stream);
        if (e != hipSuccess) return hip_fail(h, e, "hipStreamSynchronize");
    }
    if (a_ip[m] != A->nnz || (!index && b_ip[n] != B->nnz)) return fail(h, SPD_ERR_BAD_CSR, "indptr[n_rows] != nnz");
    lap("indptr d2h");

    // ---- B first: plan it, upload its plan and start the repack, so that the device is
    //      busy while the host plans A (an index brings all of that with it) ---------------
    MetricInfo mi = metric_info(metric);
    if (semiring && mi.norm == NORM_SEMI) mi.norm = NORM_SEMI + (int)semiring->product;
    if (semiring) mi.transform = (int)semiring->transform;
    APlan &ap = h->plan_of_a;
    const BPlan &bp = index ? index->plan : h->plan_of_b;
    // the set metrics count shared columns in byte lanes, or (option) as a dot product of 0/1 values
    int op = mi.op;
    if (op == OP_CNT && (h->no_byte_counters || h->opt.force_kind == KIND_BLOOM)) op = OP_DOT;
    // Minkowski: the small integer degrees share one set of kernels, every other degree has its own
    if (op == OP_MINK && degree_class(metric == SPD_L2_UNEXPANDED ? 2.0f : p) == 0) op = OP_MINK_ANY;
    // A is planned on the helper thread meanwhile; every way out of this function waits for it
    std::string why_a;
    {
        const int64_t *a_rows_ptr = a_ip;
        PlanOptions opt_a = h->opt;
        opt_a.consecutive_groups = swapped ? 1 : 0;
        h->helper.post([&why_a, &ap, opt_a, a_rows_ptr, m, A, metric, op, knn_k] {
            try {
                why_a = plan_a(a_rows_ptr, m, A->n_cols, metric, op, knn_k, opt_a, ap);
            } catch (const std::exception &ex) {
                why_a = std::string("planning failed: ") + ex.what();
            }
        });
    }
    struct WaitForHelper { Helper &w; ~WaitForHelper() { w.wait(); } } wait_for_helper{h->helper};
    std::string why;
    if (!index) {
        PlanOptions opt_b = h->opt;
        opt_b.window = window_for(h->opt, knn_k > 0 || swapped ? WINDOW_NO_SCATTERED_STORES : WINDOW_SCATTERED_STORES);
        why = plan_b(b_ip, n, opt_b, h->plan_of_b);
        if (!why.empty()) return fail(h, why.find("pointers") != std::string::npos ? SPD_ERR_BAD_CSR : SPD_ERR_UNSUPPORTED, "B: " + why);
        lap("plan b");
    }
    int a_kind = 0, a_max_r = 1, a_min_r = 1;
    uint64_t a_dmax = 0;
    why = plan_staging(A->n_cols, metric, op, knn_k > 0, h->opt, a_kind, a_max_r, a_min_r, a_dmax);
    if (!why.empty()) return fail(h, SPD_ERR_UNSUPPORTED, "A: " + why);
    // The column an idle lane looks up: no row stores it, so every kind of map sends it to the
    // table's zero row.
    const uint32_t padcol = (uint32_t)A->n_cols;
    const OpParams q = op_params(metric, p, A->n_cols, semiring);

    const int planes = metric_planes(metric);
    Carver cv;
    // (1) B's plan, then what the repack produces (none of it with an index)
    BLayout bl{};
    if (!index) bl = layout_b(bp, n, cv);
    const size_t b_end = cv.off;
    if (!index) {
        // room for A's part as well, from the documented bound, so that the scratch does not
        // have to move once the repack has been started (checked again below)
        size_t guess = 0;
        if (!h->ws_external) guess = workspace_bound(h, A, B, metric, knn_k);
        st = ensure_workspace(h, std::max(b_end, guess));
        if (st != SPD_OK) return st;
    }
    // pinned staging: [row pointers | B's plan | A's plan]
    const size_t pin_b = align256(ip_bytes);
    const size_t pin_a = pin_b + align256(bl.plan_end);
    if (h->pinned_bytes < pin_a + (size_t)m * (sizeof(ARow) + 16) + (64 << 10)) {
        // growing the pinned buffer moves it: let the helper finish reading, keep the row pointers
        h->helper.wait();
        std::vector<unsigned char> keep(ip_bytes);
        std::memcpy(keep.data(), h->pinned, ip_bytes);
        st = ensure_pinned(h, pin_a + (size_t)m * (sizeof(ARow) + 16) + (64 << 10));
        if (st != SPD_OK) return st;
        std::memcpy(h->pinned, keep.data(), ip_bytes);
        locate(a_ip, b_ip);
    }
    BDevice bd;
    auto stage_b = [&]() -> spd_status {
        return stage_b_into(h, B, bp, bl, reinterpret_cast<unsigned char *>(h->ws),
                            reinterpret_cast<unsigned char *>(h->pinned) + pin_b, metric, mi, q, padcol, bd);
    };
    if (index) {
        bd = index->bd;
    } else {
        st = stage_b();
        if (st != SPD_OK) return st;
        lap("stage b");
    }

    // ---- A, while the repack runs -------------------------------------------------------
    h->helper.wait();
    why = why_a;
    if (!why.empty()) return fail(h, why.find("pointers") != std::string::npos ? SPD_ERR_BAD_CSR : SPD_ERR_UNSUPPORTED, "A: " + why);
    lap("wait for plan a");
    {
        PlanOptions opt_c = h->opt;
        opt_c.chunk_scale = chunk_scale_for(h->opt, knn_k > 0);
        for (AClass &c : ap.classes) plan_chunks(bp, c, opt_c);
    }
    lap("chunks");
    if (h->check_plan) {
        std::vector<int64_t> index_rows;
        const int64_t *b_rows_ptr = b_ip;
        if (index) {
            // the index keeps no host copy of the row pointers: rebuild them from its segments
            index_rows.assign((size_t)n + 1, 0);
            for (size_t l = 0; l < index->plan.seg_row.size(); ++l)
                if (index->plan.seg_row[l] >= 0) index_rows[(size_t)index->plan.seg_row[l] + 1] += index->plan.seg_len[l];
            for (int64_t j = 0; j < n; ++j) index_rows[(size_t)j + 1] += index_rows[(size_t)j];
            b_rows_ptr = index_rows.data();
        }
        why = plan_check(ap, bp, a_ip, b_rows_ptr, A->n_cols, metric, op, knn_k, h->opt);
        if (!why.empty()) return fail(h, SPD_ERR_UNSUPPORTED, "internal plan check failed: " + why);
    }
    for (const AClass &c : ap.classes)
        if ((int64_t)c.n_groups * c.n_chunks >= ((int64_t)1 << 31) || (int64_t)c.lds_bytes + kStaticLds > h->opt.lds_budget ||
            (c.kind != a_kind && c.kind != KIND_BLOOM))
            return fail(h, SPD_ERR_UNSUPPORTED, "internal: launch outside the device limits");
    lap("plan check");

    // (2) A's plan, contiguous again, then what the scans produce
    Upload up;
    const size_t a_plan_begin = cv.off;
    std::vector<size_t> o_rows(ap.classes.size()), o_sumlen(ap.classes.size()), o_chunks(ap.classes.size());
    for (size_t ci = 0; ci < ap.classes.size(); ++ci) {
        const AClass &c = ap.classes[ci];
        o_rows[ci] = cv.take(c.rows.size() * sizeof(ARow));
        o_sumlen[ci] = cv.take(c.sumlen.size() * 4);
        o_chunks[ci] = cv.take(c.chunk_begin.size() * 4);
        up.add(o_rows[ci], c.rows.data(), c.rows.size() * sizeof(ARow));
        up.add(o_sumlen[ci], c.sumlen.data(), c.sumlen.size() * 4);
        up.add(o_chunks[ci], c.chunk_begin.data(), c.chunk_begin.size() * 4);
    }
    const size_t o_spilled = cv.take(ap.spilled.size() * sizeof(SpilledRow));
    up.add(o_spilled, ap.spilled.data(), ap.spilled.size() * sizeof(SpilledRow));
    // k-NN: every (row, chunk of its launch) owns a list of k candidates
    std::vector<int64_t> &knn_row_off = h->knn_row_off;
    std::vector<int32_t> &knn_row_lists = h->knn_row_lists;
    size_t o_knn_off = 0, o_knn_lists = 0;
    int64_t knn_entries = 0;
    if (knn_k > 0) {
        knn_row_off.assign((size_t)m, 0);
        knn_row_lists.assign((size_t)m, 0);
        for (const AClass &c : ap.classes)
            for (const ARow &r : c.rows)
                if (r.out >= 0) {
                    knn_row_off[(size_t)r.out] = knn_entries;
                    knn_row_lists[(size_t)r.out] = c.n_chunks;
                    knn_entries += (int64_t)c.n_chunks * knn_k;
                }
        // a spilled row: one list per tile of columns its finalize kernel walks
        const int64_t tiles = (n + kFinalizeTile - 1) / kFinalizeTile;
        for (const SpilledRow &sr : ap.spilled) {
            knn_row_off[(size_t)sr.row] = knn_entries;
            knn_row_lists[(size_t)sr.row] = (int32_t)tiles;
            knn_entries += tiles * knn_k;
        }
        o_knn_off = cv.take((size_t)m * 8);
        o_knn_lists = cv.take((size_t)m * 4);
        up.add(o_knn_off, knn_row_off.data(), (size_t)m * 8);
        up.add(o_knn_lists, knn_row_lists.data(), (size_t)m * 4);
    }
    const size_t a_plan_end = cv.off;
    const size_t o_partial = cv.take((size_t)ap.n_partial_slots * planes * (size_t)n * 8);
    const size_t o_partial_norms = cv.take((size_t)ap.n_partial_slots * 16);
    const size_t o_knn_part = cv.take((size_t)knn_entries * sizeof(KnnEntry));
    if (cv.off > h->ws_bytes || pin_a + (a_plan_end - a_plan_begin) > h->pinned_bytes) {
        // the bound was too small after all (or, with an index, this is where the scratch is
        // sized): growing waits for the repack, discards it and runs it again in the new buffers
        st = ensure_workspace(h, cv.off);
        if (st != SPD_OK) return st;
        st = ensure_pinned(h, pin_a + (a_plan_end - a_plan_begin));
        if (st != SPD_OK) return st;
        if (!index) {
            if (h->profile && !h->timed.empty()) {
                h->event_pool.push_back(h->timed.back().start); h->event_pool.push_back(h->timed.back().stop);
                h->timed.pop_back();
            }
            st = stage_b();
            if (st != SPD_OK) return st;
        }
    }
    unsigned char *ws = reinterpret_cast<unsigned char *>(h->ws);
    if (a_plan_end > a_plan_begin) {
        unsigned char *pin = reinterpret_cast<unsigned char *>(h->pinned) + pin_a;
        for (auto &pt : up.parts) std::memcpy(pin + (pt.first - a_plan_begin), pt.second.first, pt.second.second);
        e = hipMemcpyAsync(ws + a_plan_begin, pin, a_plan_end - a_plan_begin, hipMemcpyHostToDevice, h->stream);
        if (e != hipSuccess) return hip_fail(h, e, "upload of A's plan");
    }
    lap("upload a");

    // The launch with the most work stays on the caller's stream; the others go round-robin
    // to side streams that fork after the repack and join before whatever follows, so that
    // launches too small to fill the chip overlap with the large one.
    size_t main_class = 0;
    std::vector<int> lane_of(ap.classes.size(), -1);        // -1: caller's stream
    int side_used = 0;
    {
        int64_t best = -1;
        for (size_t ci = 0; ci < ap.classes.size(); ++ci) {
            int64_t work = (int64_t)ap.classes[ci].n_groups * ap.classes[ci].R;
            if (work > best) { best = work; main_class = ci; }
        }
        // A launch goes beside the large one only if it is small against it: two large launches
        // side by side push each other's share of B out of the L2 caches.
        auto small = [&](size_t ci) {
            return ci != main_class && (int64_t)ap.classes[ci].n_groups * ap.classes[ci].R * 4 <= best;
        };
        // ... and only if the small launches are worth hiding.  Beside a long launch over a large B,
        // a few workgroups that sweep B in an order of their own cost more (config 3: 6 % of the
        // call, the pairwise calls of config 2: 13 %) than the time they would take in line.  They
        // are worth it when the large launch is short (by the planner's estimate: under some 2 ms),
        // so that what a launch costs beside its sweep counts, or when they hold a tenth or more of
        // the call's sweeps over B (a group's sweep weighed by its rows plus the column lookup).
        auto sweeps = [&](size_t ci) { return (double)ap.classes[ci].n_groups * (3.0 + ap.classes[ci].R); };
        int n_small = 0;
        double small_sweeps = 0.0;
        for (size_t ci = 0; ci < ap.classes.size(); ++ci)
            if (small(ci)) { ++n_small; small_sweeps += sweeps(ci); }
        const bool worth = !ap.classes.empty() &&
                           (ap.classes[main_class].cost < 8000.0 || small_sweeps * 10.0 >= sweeps(main_class));
        if (h->side_streams > 0 && n_small > 0 && worth) {
            const int want = std::min<int>(h->side_streams, n_small);
            for (int q = 0; q < want; ++q) {
                if (!h->side[q] && hipStreamCreateWithFlags(&h->side[q], hipStreamNonBlocking) != hipSuccess) { h->side[q] = nullptr; break; }
                if (!h->join_event[q] && hipEventCreateWithFlags(&h->join_event[q], hipEventDisableTiming) != hipSuccess) break;
                side_used = q + 1;
            }
            if (!h->fork_event && hipEventCreateWithFlags(&h->fork_event, hipEventDisableTiming) != hipSuccess) side_used = 0;
        }
        if (side_used > 0) {
            e = hipEventRecord(h->fork_event, h->stream);
            if (e != hipSuccess) return hip_fail(h, e, "hipEventRecord");
            for (int q = 0; q < side_used; ++q) {
                e = hipStreamWaitEvent(h->side[q], h->fork_event, 0);
                if (e != hipSuccess) return hip_fail(h, e, "hipStreamWaitEvent");
            }
            int next = 0;
            for (size_t ci = 0; ci < ap.classes.size(); ++ci)
                if (small(ci)) { lane_of[ci] = next; next = (next + 1) % side_used; }
        }
    }
    // the large launch goes first: every microsecond the host spends on the others would
    // otherwise delay it
    std::vector<size_t> launch_order;
    if (!ap.classes.empty()) launch_order.push_back(main_class);
    for (size_t ci = 0; ci < ap.classes.size(); ++ci) if (ci != main_class) launch_order.push_back(ci);
    for (size_t ci : launch_order) {
        hipStream_t st_launch = lane_of[ci] >= 0 ? h->side[lane_of[ci]] : h->stream;
        const AClass &c = ap.classes[ci];
        ScanArgs sa;
        sa.a_indices = A->indices;
        sa.a_values = A->values;
        sa.arows = reinterpret_cast<const ARow *>(ws + o_rows[ci]);
        sa.sumlen = reinterpret_cast<const int32_t *>(ws + o_sumlen[ci]);
        sa.n_groups = c.n_groups;
        sa.chunk_begin = reinterpret_cast<const int32_t *>(ws + o_chunks[ci]);
        sa.n_chunks = c.n_chunks;
        sa.b_indptr = B->indptr;
        sa.b_indices = B->indices;
        sa.b = bd;
        sa.q = q;
        sa.kind = c.kind;
        sa.hscale = c.hscale;
        sa.cuckoo_attempts = h->cuckoo_attempts;
        sa.knn_seed = h->knn_seed;
        sa.transform = mi.transform;
        sa.norm = mi.norm;
        sa.k = (uint32_t)A->n_cols;
        sa.padcol = padcol;
        sa.out = out;
        sa.out_stride_staged = out_stride_staged;
        sa.out_stride_streamed = out_stride_streamed;
        sa.partial = reinterpret_cast<double *>(ws + o_partial);
        sa.partial_norms = reinterpret_cast<double *>(ws + o_partial_norms);
        sa.planes = planes;
        sa.knn_k = knn_k;
        sa.knn_part = reinterpret_cast<KnnEntry *>(ws + o_knn_part);
        sa.knn_row_off = reinterpret_cast<const int64_t *>(ws + o_knn_off);
        int64_t live_rows = 0;
        for (const ARow &r : c.rows) live_rows += (r.out != -1);
        LaunchTimer lt(h, "scan", c.R, c.kind, c.block, c.lds_bytes, live_rows, (int64_t)c.n_groups * c.n_chunks,
                       st_launch);
        e = launch_scan(st_launch, op, c.R, c.block, c.lds_bytes, sa);
        if (e != hipSuccess) {
            // what already runs on the side streams still has to be ordered before the caller's next work
            for (int q = 0; q < side_used; ++q)
                if (hipEventRecord(h->join_event[q], h->side[q]) == hipSuccess) (void)hipStreamWaitEvent(h->stream, h->join_event[q], 0);
            return hip_fail(h, e, "scan kernel");
        }
        lt.done();
    }

    {
        hipError_t first_error = hipSuccess;
        for (int q = 0; q < side_used; ++q) {
            e = hipEventRecord(h->join_event[q], h->side[q]);
            if (e == hipSuccess) e = hipStreamWaitEvent(h->stream, h->join_event[q], 0);
            if (e != hipSuccess && first_error == hipSuccess) first_error = e;      // the other streams are still joined
        }
        if (first_error != hipSuccess) return hip_fail(h, first_error, "joining the side streams");
    }

    if (!ap.spilled.empty()) {
        FinalizeArgs fa;
        fa.spilled = reinterpret_cast<const SpilledRow *>(ws + o_spilled);
        fa.n_spilled = (int32_t)ap.spilled.size();
        fa.partial = reinterpret_cast<const double *>(ws + o_partial);
        fa.partial_norms = reinterpret_cast<const double *>(ws + o_partial_norms);
        fa.norms_b = bd.norms;
        fa.planes = planes;
        fa.n_b = n;
        fa.q = q;
        fa.out = out;
        fa.out_stride_staged = out_stride_staged;
        fa.out_stride_streamed = out_stride_streamed;
        fa.knn_k = knn_k;
        fa.knn_part = reinterpret_cast<KnnEntry *>(ws + o_knn_part);
        fa.knn_row_off = reinterpret_cast<const int64_t *>(ws + o_knn_off);
        LaunchTimer lt(h, "finalize", 0, 0, 0, 0, (int64_t)ap.spilled.size(), 0);
        e = launch_finalize(h->stream, fa);
        if (e != hipSuccess) return hip_fail(h, e, "finalize kernel");
        lt.done();
    }
    lap("launches");
    if (knn_k > 0) {
        LaunchTimer lt(h, "knn_merge", 0, 0, 0, 0, m, (m + 3) / 4);
        e = launch_knn_merge(h->stream, reinterpret_cast<const KnnEntry *>(ws + o_knn_part),
                             reinterpret_cast<const int64_t *>(ws + o_knn_off),
                             reinterpret_cast<const int32_t *>(ws + o_knn_lists), m, knn_k,
                             metric == SPD_INNER_PRODUCT ? 1 : 0, out_idx, out_dist);
        if (e != hipSuccess) return hip_fail(h, e, "k-NN merge kernel");
        lt.done();
    }
    return SPD_OK;
}

}  // namespace

extern "C" {

spd_status spd_create(spd_handle **handle, void *hip_stream) {
    if (!handle) return SPD_ERR_NULL;
    *handle = nullptr;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return SPD_ERR_HIP;
    spd_handle *h = new (std::nothrow) spd_handle();
    if (!h) return SPD_ERR_WORKSPACE;
    h->device = dev;
    h->stream = reinterpret_cast<hipStream_t>(hip_stream);
    int lds = 0, cus = 0;
    if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) == hipSuccess && lds > 0)
        h->opt.lds_budget = std::min<int64_t>(lds, 160 * 1024);
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
        h->opt.n_cus = cus;
    e = hipMalloc(reinterpret_cast<void **>(&h->flag), 256);
    if (e != hipSuccess) { delete h; return SPD_ERR_HIP; }
    // this device's copy of the static scratch array: its address is asked for once per device
    if (dev >= 0 && dev < kStaticScratchDevices) {
        std::lock_guard<std::mutex> g(g_static_scratch_mutex);
        if (!g_static_scratch[dev]) {
            void *ptr = nullptr;
            e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !ptr) { (void)hipFree(h->flag); delete h; return SPD_ERR_HIP; }
            g_static_scratch[dev] = ptr;
        }
        h->static_ws = g_static_scratch[dev];
    }
    // staging memory and the events that guard it, so that a call of modest size allocates nothing
    for (spd_handle::PinnedSlot &ps : h->pinned_slots) {
        if (hipHostMalloc(&ps.ptr, kInitialPinnedBytes, hipHostMallocDefault) != hipSuccess) { ps.ptr = nullptr; break; }
        ps.bytes = kInitialPinnedBytes;
        if (hipEventCreateWithFlags(&ps.done, hipEventDisableTiming) != hipSuccess) ps.done = nullptr;
    }
    *handle = h;
    return SPD_OK;
}

spd_status spd_destroy(spd_handle *h) {
    if (!h) return SPD_ERR_NULL;
    hipError_t e = hipStreamSynchronize(h->stream);
    (void)e;
    for (spd_handle::PinnedSlot &ps : h->pinned_slots) {
        if (ps.ptr) (void)hipHostFree(ps.ptr);
        if (ps.done) (void)hipEventDestroy(ps.done);
    }
    if (h->own_ws) (void)hipFree(h->own_ws);
    if (h->flag) (void)hipFree(h->flag);
    for (auto &t : h->timed) { (void)hipEventDestroy(t.start); (void)hipEventDestroy(t.stop); }
    for (hipEvent_t ev : h->event_pool) (void)hipEventDestroy(ev);
    for (int q = 0; q < spd_handle::kSideStreams; ++q) {
        if (h->side[q]) { (void)hipStreamSynchronize(h->side[q]); (void)hipStreamDestroy(h->side[q]); }
        if (h->join_event[q]) (void)hipEventDestroy(h->join_event[q]);
    }
    if (h->fork_event) (void)hipEventDestroy(h->fork_event);
    delete h;
    return SPD_OK;
}

spd_status spd_workspace_bytes(const spd_handle *h, const spd_csr *A, const spd_csr *B, spd_metric metric,
                               int k_neighbors, size_t *bytes) {
    if (!h || !A || !B || !bytes) return SPD_ERR_NULL;
    if ((int)metric < 0 || (int)metric >= SPD_METRIC_COUNT) return SPD_ERR_BAD_METRIC;
    if (A->n_rows < 0 || B->n_rows < 0 || A->nnz < 0 || B->nnz < 0 || A->n_cols != B->n_cols) return SPD_ERR_DIM_MISMATCH;
    *bytes = workspace_bound(h, A, B, (int)metric, k_neighbors);
    // (a pairwise call may exchange the roles of its operands)
    if (k_neighbors == 0 && h->swap_operands != 0 && operands_may_swap((int)metric, nullptr))
        *bytes = std::max(*bytes, workspace_bound(h, B, A, (int)metric, 0));
    return SPD_OK;
}

}  // extern "C"

namespace {
size_t workspace_bound(const spd_handle *h, const spd_csr *A, const spd_csr *B, int metric, int k_neighbors) {
    const PlanOptions &o = h->opt;
    const size_t m = (size_t)A->n_rows, n = (size_t)B->n_rows;
    const int split_len = split_len_for(o, B->nnz);
    const size_t seg_target = (size_t)std::max(1, std::max(2, split_len) / 2);
    const size_t window = (size_t)std::max(64, window_for(o, WINDOW_SCATTERED_STORES));   // the narrowest: the largest bound
    size_t slabs = n / 64 + n / window + (n + 4 * (size_t)B->nnz / seg_target) / 64 + 4;
    size_t lanes = slabs * 64;
    // at most 15 launches (5 group sizes x 3 occupancies), each cutting B at most 4096 times and
    // never into more than 4 workgroups per slot of the chip (times the chunk scale) plus one per group
    const size_t launches = 15;
    const size_t chunk_words = launches * 4097;
    // rows of A that do not fit alone are cut into slices of at least 1/2 of the largest
    // slice the budget admits; 512 entries is a floor for any budget the planner accepts
    size_t slices = 2 * (size_t)A->nnz / 512 + 2;
    slices = std::min(slices, (size_t)A->nnz / 64 + 2);
    size_t planes = (size_t)metric_planes(metric);
    size_t total = 0;
    auto add = [&](size_t b) { total += align256(b); };
    // padded slabs: at most 64 idle entries per step of the longest row of each window, one per
    // lane of a split row, and the rounding of each group of split rows
    size_t padded = (size_t)B->nnz + (size_t)B->nnz * 64 / (size_t)std::max(2, split_len) +
                    64 * (size_t)std::max(2, split_len) * (n / window + 8) + 64 * (size_t)kScanUnroll * slabs;
    add(padded * 8); add(n * 16); add((slabs + 1) * 8); add(slabs * 4); add(slabs);
    add(lanes * 8); add(lanes * 4); add(lanes * 4); add(lanes); add(chunk_words * 4); total += launches * 256;
    // (a group may leave a quarter of its places empty: up to a third more places than rows)
    const size_t places = m + slices + (m + slices) / 3 + 32 * 6;
    add(places * sizeof(ARow)); add((m + slices + 6) * 4); total += 12 * 256;
    add(slices * sizeof(SpilledRow));
    // partial results exist only for sliced rows; a row needs slicing only above ~9,000 entries
    size_t sliced_rows_max = (size_t)A->nnz / 4096 + 1;
    size_t partial_slots = std::min(slices, 2 * sliced_rows_max + (size_t)A->nnz / 4096);
    add(partial_slots * planes * n * 8); add(partial_slots * 16);
    if (k_neighbors > 0) {
        size_t lists = o.chunks > 0 ? (m + m / 3 + 16 * launches) * (size_t)o.chunks
                                    : launches * 16 * (16 * (size_t)o.n_cus * (size_t)chunk_scale_for(o, true) + 1) + m + m / 3 + 16 * launches;
        lists += std::min(sliced_rows_max, m) * (n / (size_t)kFinalizeTile + 1);     // the tiles of spilled rows
        add(lists * (size_t)k_neighbors * sizeof(KnnEntry)); add(m * 8); add(m * 4);
    }
    return total;
}
}  // namespace

extern "C" {

spd_status spd_set_workspace(spd_handle *h, void *device_ptr, size_t bytes) {
    if (!h) return SPD_ERR_NULL;
    h->err.clear();
    if (!device_ptr || bytes == 0) {
        h->ws_external = false;
        h->ws = h->own_ws;
        h->ws_bytes = h->own_ws_bytes;
        return SPD_OK;
    }
    if ((reinterpret_cast<uintptr_t>(device_ptr) & 255u) != 0) return fail(h, SPD_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    h->ws_external = true;
    h->ws = device_ptr;
    h->ws_bytes = bytes;
    return SPD_OK;
}

spd_status spd_pairwise(spd_handle *h, const spd_csr *A, const spd_csr *B, spd_metric metric, float p, float *out) {
    spd_status st = check_call_args(h, A, B, metric, p, 0, false, out, nullptr);
    if (st != SPD_OK) return st;
    return run(h, A, B, (int)metric, p, nullptr, 0, out, nullptr, nullptr);
}

spd_status spd_pairwise_static(spd_handle *h, const spd_csr *A, const spd_csr *B, spd_metric metric, float p,
                               float *out) {
    spd_status st = check_call_args(h, A, B, metric, p, 0, false, out, nullptr);
    if (st != SPD_OK) return st;
    if (!A->host_indptr || !B->host_indptr)
        return fail(h, SPD_ERR_NULL, "spd_pairwise_static needs host_indptr of both operands (it neither copies the row "
                                     "pointers back nor waits for the stream)");
    if (!h->static_ws) return fail(h, SPD_ERR_HIP, "no static scratch on this device");
    for (const spd_handle::PinnedSlot &ps : h->pinned_slots)
        if (!ps.ptr || !ps.done) return fail(h, SPD_ERR_WORKSPACE, "the handle holds no staging memory");
    // the call runs as spd_pairwise does, with the static array as its scratch, on the handle's
    // stream alone and without launch timers (internal streams and events would have to be created)
    struct Saved {
        spd_handle *h; void *ws; size_t ws_bytes; bool ws_external; int side_streams; bool profile;
        ~Saved() { h->ws = ws; h->ws_bytes = ws_bytes; h->ws_external = ws_external; h->side_streams = side_streams;
                   h->profile = profile; h->no_alloc = false; }
    } saved{h, h->ws, h->ws_bytes, h->ws_external, h->side_streams, h->profile};
    h->ws = h->static_ws;
    h->ws_bytes = kStaticScratchBytes;
    h->ws_external = true;
    h->side_streams = 0;
    h->profile = false;
    h->no_alloc = true;
    return run(h, A, B, (int)metric, p, nullptr, 0, out, nullptr, nullptr);
}

spd_status spd_knn(spd_handle *h, const spd_csr *Q, const spd_csr *Index, spd_metric metric, float p, int k,
                   int64_t *out_idx, float *out_dist) {
    spd_status st = check_call_args(h, Q, Index, metric, p, k, true, out_idx, out_dist);
    if (st != SPD_OK) return st;
    return run(h, Q, Index, (int)metric, p, nullptr, k, nullptr, out_idx, out_dist);
}

spd_status spd_semiring_pairwise(spd_handle *h, const spd_csr *A, const spd_csr *B, const spd_semiring *semiring,
                                 float *out) {
    spd_status st = check_call_args(h, A, B, SPD_INNER_PRODUCT, 0.0f, 0, false, out, nullptr, semiring, true);
    if (st != SPD_OK) return st;
    const int as_metric = table1_metric(*semiring, false);
    if (as_metric >= 0) return run(h, A, B, as_metric, semiring->p, nullptr, 0, out, nullptr, nullptr);
    return run(h, A, B, semiring->sum == SPD_SUM_PLUS ? MT_SEMI_SUM : MT_SEMI_EXT, 1.0f, semiring, 0, out, nullptr, nullptr);
}

spd_status spd_semiring_knn(spd_handle *h, const spd_csr *Q, const spd_csr *Index, const spd_semiring *semiring, int k,
                            int64_t *out_idx, float *out_dist) {
    spd_status st = check_call_args(h, Q, Index, SPD_INNER_PRODUCT, 0.0f, k, true, out_idx, out_dist, semiring, true);
    if (st != SPD_OK) return st;
    const int as_metric = table1_metric(*semiring, true);
    if (as_metric >= 0) return run(h, Q, Index, as_metric, semiring->p, nullptr, k, nullptr, out_idx, out_dist);
    return run(h, Q, Index, semiring->sum == SPD_SUM_PLUS ? MT_SEMI_SUM : MT_SEMI_EXT, 1.0f, semiring, k, nullptr, out_idx,
               out_dist);
}

spd_status spd_index_create(spd_handle *h, const spd_csr *Index, spd_metric metric, float p, spd_index **out) {
    if (!h) return SPD_ERR_NULL;
    h->err.clear();
    if (!out) return fail(h, SPD_ERR_NULL, "index is NULL");
    *out = nullptr;
    spd_status st = check_csr_args(h, Index, "Index");
    if (st != SPD_OK) return st;
    if ((int)metric < 0 || (int)metric >= SPD_METRIC_COUNT) return fail(h, SPD_ERR_BAD_METRIC, "unknown metric");
    if (metric == SPD_MINKOWSKI && !(p > 0.0f && std::isfinite(p))) return fail(h, SPD_ERR_BAD_P, "Minkowski needs a finite p > 0");
    for (auto &t : h->timed) { h->event_pool.push_back(t.start); h->event_pool.push_back(t.stop); }
    h->timed.clear();
    hipError_t e = hipSetDevice(h->device);
    if (e != hipSuccess) return hip_fail(h, e, "hipSetDevice");
    const int64_t n = Index->n_rows;
    spd_index *ix = new (std::nothrow) spd_index();
    if (!ix) return fail(h, SPD_ERR_WORKSPACE, "out of host memory");
    struct Guard { spd_index *p; ~Guard() { if (p) { if (p->dev) (void)hipFree(p->dev); delete p; } } } guard{ix};
    ix->matrix = *Index;
    ix->metric = (int)metric;
    ix->p = p;
    ix->device = h->device;
    PinnedLease lease(h);
    st = ensure_pinned(h, (size_t)(n + 1) * 8 + 32 * ((size_t)n + 4096));
    if (st != SPD_OK) return st;
    const int64_t *b_ip = Index->host_indptr;
    if (!b_ip) {
        int64_t *pin = reinterpret_cast<int64_t *>(h->pinned);
        e = hipMemcpyAsync(pin, Index->indptr, (size_t)(n + 1) * 8, hipMemcpyDeviceToHost, h->stream);
        if (e != hipSuccess) return hip_fail(h, e, "copy of Index.indptr");
        e = hipStreamSynchronize(h->stream);
        if (e != hipSuccess) return hip_fail(h, e, "hipStreamSynchronize");
        b_ip = pin;
    }
    if (b_ip[n] != Index->nnz) return fail(h, SPD_ERR_BAD_CSR, "indptr[n_rows] != nnz");
    std::string why;
    try {
        PlanOptions opt_b = h->opt;
        opt_b.window = window_for(h->opt, WINDOW_SCATTERED_STORES);      // an index serves pairwise calls that stage A as well
        why = plan_b(b_ip, n, opt_b, ix->plan);
    } catch (const std::exception &ex) {
        why = std::string("planning failed: ") + ex.what();
    }
    if (!why.empty()) return fail(h, why.find("pointers") != std::string::npos ? SPD_ERR_BAD_CSR : SPD_ERR_UNSUPPORTED, "Index: " + why);
    Carver cv;
    const BLayout bl = layout_b(ix->plan, n, cv);
    ix->dev_bytes = std::max<size_t>(cv.off, 256);
    e = hipMalloc(&ix->dev, ix->dev_bytes);
    if (e != hipSuccess) { ix->dev = nullptr; return fail(h, SPD_ERR_WORKSPACE, std::string("hipMalloc of the index failed: ") + hipGetErrorString(e)); }
    // (the row pointers have served: the plan's arrays may overwrite them in the pinned buffer)
    st = ensure_pinned(h, bl.plan_end + 256);
    if (st != SPD_OK) return st;
    const int run_as = effective_metric((int)metric, p);
    const MetricInfo mi = metric_info(run_as);
    const OpParams q = op_params(run_as, p, Index->n_cols, nullptr);
    if (n > 0) {
        st = stage_b_into(h, Index, ix->plan, bl, reinterpret_cast<unsigned char *>(ix->dev),
                          reinterpret_cast<unsigned char *>(h->pinned), run_as, mi, q, (uint32_t)Index->n_cols, ix->bd);
        if (st != SPD_OK) return st;
    }
    guard.p = nullptr;
    *out = ix;
    return SPD_OK;
}

spd_status spd_index_destroy(spd_handle *h, spd_index *index) {
    if (!h) return SPD_ERR_NULL;
    h->err.clear();
    if (!index) return SPD_OK;
    hipError_t e = hipStreamSynchronize(h->stream);      // calls that read the index may still be running
    (void)e;
    if (index->dev) (void)hipFree(index->dev);
    delete index;
    return SPD_OK;
}

spd_status spd_index_pairwise(spd_handle *h, const spd_csr *A, const spd_index *index, float *out) {
    if (!h) return SPD_ERR_NULL;
    if (!index) { h->err = "index is NULL"; return SPD_ERR_NULL; }
    spd_status st = check_call_args(h, A, &index->matrix, (spd_metric)index->metric, index->p, 0, false, out, nullptr);
    if (st != SPD_OK) return st;
    if (index->device != h->device) return fail(h, SPD_ERR_UNSUPPORTED, "the index lives on another device");
    return run(h, A, &index->matrix, index->metric, index->p, nullptr, 0, out, nullptr, nullptr, index);
}

spd_status spd_index_knn(spd_handle *h, const spd_csr *Q, const spd_index *index, int k, int64_t *out_idx,
                         float *out_dist) {
    if (!h) return SPD_ERR_NULL;
    if (!index) { h->err = "index is NULL"; return SPD_ERR_NULL; }
    spd_status st = check_call_args(h, Q, &index->matrix, (spd_metric)index->metric, index->p, k, true, out_idx, out_dist);
    if (st != SPD_OK) return st;
    if (index->device != h->device) return fail(h, SPD_ERR_UNSUPPORTED, "the index lives on another device");
    return run(h, Q, &index->matrix, index->metric, index->p, nullptr, k, nullptr, out_idx, out_dist, index);
}

spd_status spd_csr_validate(spd_handle *h, const spd_csr *M, int require_nonnegative) {
    if (!h) return SPD_ERR_NULL;
    h->err.clear();
    spd_status st = check_csr_args(h, M, "M");
    if (st != SPD_OK) return st;
    if (M->n_rows == 0) return M->nnz == 0 ? SPD_OK : fail(h, SPD_ERR_BAD_CSR, "no rows but nnz > 0");
    hipError_t e = hipMemsetAsync(h->flag, 0, 4, h->stream);
    if (e != hipSuccess) return hip_fail(h, e, "hipMemsetAsync");
    e = launch_validate(h->stream, M->indptr, M->indices, M->values, M->n_rows, M->n_cols, M->nnz,
                        require_nonnegative, h->flag);
    if (e != hipSuccess) return hip_fail(h, e, "validate kernel");
    int32_t flag = 0;
    e = hipMemcpyAsync(&flag, h->flag, 4, hipMemcpyDeviceToHost, h->stream);
    if (e != hipSuccess) return hip_fail(h, e, "hipMemcpyAsync");
    e = hipStreamSynchronize(h->stream);
    if (e != hipSuccess) return hip_fail(h, e, "hipStreamSynchronize");
    if (flag) {
        std::string what;
        if (flag & 1) what += " row pointers;";
        if (flag & 2) what += " column order or range;";
        if (flag & 4) what += " values;";
        return fail(h, SPD_ERR_BAD_CSR, "invalid CSR:" + what);
    }
    return SPD_OK;
}

spd_status spd_set_option(spd_handle *h, const char *name, int64_t value) {
    if (!h || !name) return SPD_ERR_NULL;
    h->err.clear();
    std::string s(name);
    PlanOptions &o = h->opt;
    if (s == "lds_budget") {
        if (value < 8192 || value > 160 * 1024) return fail(h, SPD_ERR_UNSUPPORTED, "lds_budget must lie in [8192, 163840]");
        o.lds_budget = value;
    } else if (s == "force_kind") {
        if (value < 0 || value > 5) return fail(h, SPD_ERR_UNSUPPORTED, "force_kind must be 0..5");
        o.force_kind = (int)value;
    } else if (s == "max_rows") {
        if (value != 1 && value != 2 && value != 4 && value != 8 && value != 16)
            return fail(h, SPD_ERR_UNSUPPORTED, "max_rows must be 1, 2, 4, 8 or 16");
        o.max_rows = (int)value;
    } else if (s == "split_len") {
        if (value != 0 && (value < 2 || value > (1 << 20)))
            return fail(h, SPD_ERR_UNSUPPORTED, "split_len must be 0 (automatic) or lie in [2, 2^20]");
        o.split_len = (int)value;
    } else if (s == "window") {
        if (value != 0 && (value < 64 || value > (1 << 24)))
            return fail(h, SPD_ERR_UNSUPPORTED, "window must be 0 (automatic) or lie in [64, 2^24]");
        o.window = (int)value;
    } else if (s == "chunk_scale") {
        if (value < 0 || value > 8) return fail(h, SPD_ERR_UNSUPPORTED, "chunk_scale must lie in [0, 8]");
        o.chunk_scale = (int)value;
    } else if (s == "chunks") {
        if (value < 0 || value > 4096) return fail(h, SPD_ERR_UNSUPPORTED, "chunks must lie in [0, 4096]");
        o.chunks = (int)value;
    } else if (s == "byte_counters") {
        if (value != 0 && value != 1) return fail(h, SPD_ERR_UNSUPPORTED, "byte_counters must be 0 or 1");
        h->no_byte_counters = value == 0;
    } else if (s == "waves_per_cu") {
        if (value != 0 && value != 8 && value != 16 && value != 32)
            return fail(h, SPD_ERR_UNSUPPORTED, "waves_per_cu must be 0 (automatic), 8, 16 or 32");
        o.waves_per_cu = (int)value;
    } else if (s == "sort_slack") {
        if (value != 0 && value != 1) return fail(h, SPD_ERR_UNSUPPORTED, "sort_slack must be 0 or 1");
        o.sort_slack = (int)value;
    } else if (s == "partial_groups") {
        if (value < 0 || value > 2) return fail(h, SPD_ERR_UNSUPPORTED, "partial_groups must be 0, 1 or 2");
        o.partial_groups = (int)value;
    } else if (s == "bloom_long_rows") {
        if (value != 0 && value != 1) return fail(h, SPD_ERR_UNSUPPORTED, "bloom_long_rows must be 0 or 1");
        o.bloom_long_rows = (int)value;
    } else if (s == "side_streams") {
        if (value < 0 || value > spd_handle::kSideStreams) return fail(h, SPD_ERR_UNSUPPORTED, "side_streams must lie in [0, 3]");
        h->side_streams = (int)value;
    } else if (s == "knn_seed") {
        if (value < 0 || value > 1) return fail(h, SPD_ERR_UNSUPPORTED, "knn_seed must be 0 or 1");
        h->knn_seed = (int)value;
    } else if (s == "cuckoo_attempts") {
        if (value < 0 || value > 3) return fail(h, SPD_ERR_UNSUPPORTED, "cuckoo_attempts must lie in [0, 3]");
        h->cuckoo_attempts = (int)value;
    } else if (s == "swap_operands") {
        if (value < 0 || value > 2) return fail(h, SPD_ERR_UNSUPPORTED, "swap_operands must be 0, 1 or 2");
        h->swap_operands = (int)value;
    } else if (s == "check_plan") {
        if (value != 0 && value != 1) return fail(h, SPD_ERR_UNSUPPORTED, "check_plan must be 0 or 1");
        h->check_plan = value != 0;
    } else if (s == "profile") {
        if (value != 0 && value != 1) return fail(h, SPD_ERR_UNSUPPORTED, "profile must be 0 or 1");
        h->profile = value != 0;
    } else {
        return fail(h, SPD_ERR_UNSUPPORTED, "unknown option " + s);
    }
    return SPD_OK;
}

int spd_profile_read(spd_handle *h, spd_kernel_time *out, int cap) {
    if (!h || (cap > 0 && !out)) return -1;
    if (h->timed.empty()) return 0;
    if (hipEventSynchronize(h->timed.back().stop) != hipSuccess) return -2;
    int n = 0;
    for (auto &t : h->timed) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, t.start, t.stop) == hipSuccess) t.rec.ms = (double)ms;
        if (n < cap) out[n] = t.rec;
        ++n;
    }
    return n;
}

const char *spd_last_error(const spd_handle *h) { return h ? h->err.c_str() : "null handle"; }

const char *spd_metric_name(spd_metric metric) {
    return ((int)metric >= 0 && (int)metric < SPD_METRIC_COUNT) ? kMetricNames[(int)metric] : "unknown";
}

const char *spd_version(void) { return "spd 0.1 (gfx950)"; }

}  // extern "C"
