// The staged-scan kernel: one workgroup stages R rows of A in LDS and sweeps a chunk of
// B's slabs over them (the hot loop of the paper's Algorithm 3, re-cut for 64-wide
// wavefronts: one row of B per lane instead of one non-zero per thread, so the segmented
// scan and the atomic writes of that algorithm disappear).
//
// Included once per product (OP) by the spd_scan_op_*.hip translation units.
#pragma once
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>

#include "spd_kernels.h"

namespace spd {

// ------------------------------------------------------------------------------------
// wavefront helpers (gfx950: 64 lanes)
// ------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t lane_rank_in(uint64_t mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}
__device__ __forceinline__ int wave_uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ double wave_uniform_f64(double v) {
    const int lo = __builtin_amdgcn_readfirstlane(__double2loint(v)), hi = __builtin_amdgcn_readfirstlane(__double2hiint(v));
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ bool lex_less(float d1, int j1, float d2, int j2) {
    return d1 < d2 || (d1 == d2 && j1 < j2);
}

// Order-preserving map float -> uint32 (for an LDS atomicMin over distances of any sign).
__device__ __forceinline__ uint32_t float_order_key(float f) {
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float float_from_order_key(uint32_t u) {
    return __uint_as_float((u & 0x80000000u) ? (u & 0x7fffffffu) : ~u);
}

// Lane l receives lane l-1's value (lane 0 keeps its own): DPP wavefront shift right by one.
__device__ __forceinline__ int wave_shr1(int v) { return __builtin_amdgcn_update_dpp(v, v, 0x138, 0xf, 0xf, false); }

// (distance, index) as one integer whose order is the lexicographic order of the pair.
__device__ __forceinline__ uint64_t knn_key(float d, int j) {
    return ((uint64_t)float_order_key(d + 0.0f) << 32) | (uint32_t)j;     // -0 counts as +0
}
constexpr int kKnnBulkFrom = 8;     // candidates in one offer from which they are sorted rather than inserted one by one

// Lanes whose bit is set keep the smaller key of a compare-exchange at distance J while
// blocks of K lanes are being merged (K = 128: every block ascending).
constexpr uint64_t bitonic_keep_min(int K, int J, bool descending) {
    uint64_t m = 0;
    for (int l = 0; l < 64; ++l) {
        bool up = ((l & K) == 0) != descending;
        if (((l & J) == 0) == up) m |= (uint64_t)1 << l;
    }
    return m;
}

// Value of lane l ^ J.  Within a row of 16 lanes the exchange is a DPP move (no trip through
// the LDS crossbar): quad permutes for 1 and 2, a rotation by 8, and for 4 two shifts that
// each write the banks of four lanes they are right for.
template <int J> __device__ __forceinline__ uint32_t lane_xor(uint32_t v) {
    const int x = (int)v;
    if constexpr (J == 1) return (uint32_t)__builtin_amdgcn_mov_dpp(x, 0xB1, 0xf, 0xf, false);        // quad_perm [1,0,3,2]
    else if constexpr (J == 2) return (uint32_t)__builtin_amdgcn_mov_dpp(x, 0x4E, 0xf, 0xf, false);   // quad_perm [2,3,0,1]
    else if constexpr (J == 4) {
        int t = __builtin_amdgcn_mov_dpp(x, 0x104, 0xf, 0x5, false);             // row_shl:4 -> lanes 0-3, 8-11 read l+4
        return (uint32_t)__builtin_amdgcn_update_dpp(t, x, 0x114, 0xf, 0xA, false);   // row_shr:4 -> lanes 4-7, 12-15 read l-4
    } else if constexpr (J == 8) return (uint32_t)__builtin_amdgcn_mov_dpp(x, 0x128, 0xf, 0xf, false);  // row_ror:8
    else return (uint32_t)__shfl_xor(x, J);
}

template <int K, int J, bool DESC> __device__ __forceinline__ uint64_t bitonic_step(uint64_t mine, int lane) {
    constexpr uint64_t keep = bitonic_keep_min(K, J, DESC);
    const uint32_t lo = lane_xor<J>((uint32_t)mine);
    const uint32_t hi = lane_xor<J>((uint32_t)(mine >> 32));
    const uint64_t other = ((uint64_t)hi << 32) | lo;
    // take the other key where (other < mine) == keep: the lane pattern is a constant mask
    (void)lane;
    const bool take = __builtin_amdgcn_inverse_ballot_w64(__builtin_amdgcn_ballot_w64(other < mine) ^ ~keep);
    return take ? other : mine;
}

// Sorts one key per lane over the wavefront, descending (bitonic network, 21 steps).
__device__ __forceinline__ uint64_t wave_sort_desc(uint64_t x, int lane) {
    x = bitonic_step<2, 1, true>(x, lane);
    x = bitonic_step<4, 2, true>(x, lane);  x = bitonic_step<4, 1, true>(x, lane);
    x = bitonic_step<8, 4, true>(x, lane);  x = bitonic_step<8, 2, true>(x, lane);  x = bitonic_step<8, 1, true>(x, lane);
    x = bitonic_step<16, 8, true>(x, lane); x = bitonic_step<16, 4, true>(x, lane); x = bitonic_step<16, 2, true>(x, lane);
    x = bitonic_step<16, 1, true>(x, lane);
    x = bitonic_step<32, 16, true>(x, lane); x = bitonic_step<32, 8, true>(x, lane); x = bitonic_step<32, 4, true>(x, lane);
    x = bitonic_step<32, 2, true>(x, lane);  x = bitonic_step<32, 1, true>(x, lane);
    x = bitonic_step<64, 32, true>(x, lane); x = bitonic_step<64, 16, true>(x, lane); x = bitonic_step<64, 8, true>(x, lane);
    x = bitonic_step<64, 4, true>(x, lane);  x = bitonic_step<64, 2, true>(x, lane);  x = bitonic_step<64, 1, true>(x, lane);
    return x;
}
// Sorts a bitonic sequence of 64 keys ascending (6 steps).
__device__ __forceinline__ uint64_t wave_merge_asc(uint64_t x, int lane) {
    x = bitonic_step<128, 32, false>(x, lane); x = bitonic_step<128, 16, false>(x, lane);
    x = bitonic_step<128, 8, false>(x, lane);  x = bitonic_step<128, 4, false>(x, lane);
    x = bitonic_step<128, 2, false>(x, lane);  x = bitonic_step<128, 1, false>(x, lane);
    return x;
}

// Sorted list of the k best (distance, index) pairs of one query row, entry t in lane t (the kernels that
// merge lists from memory keep theirs this way; the scan kernel's lists live in LDS, below).
// Entry k-1 is the bar a candidate has to beat; it is read from its lane when needed (scalar
// registers), so a list costs two vector registers.
struct KnnList {
    float d;
    int j;
    __device__ __forceinline__ void reset() {
        d = __builtin_huge_valf();
        j = 0x7fffffff;
    }
    __device__ __forceinline__ float bar_d(int k) const {
        return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(d), k - 1));
    }
    __device__ __forceinline__ int bar_j(int k) const { return __builtin_amdgcn_readlane(j, k - 1); }
    __device__ __forceinline__ bool full(int k) const { return bar_j(k) != 0x7fffffff; }
    // Every lane may offer one candidate; the list stays sorted by (d, j).  `bound` is any
    // upper bound of the final k-th distance known from elsewhere (candidates above it are
    // dropped unseen).  Returns true if the list changed.
    __device__ __forceinline__ bool offer(float dv, int jv, bool valid, int k, float bound) {
        float tau_d = bar_d(k);
        int tau_j = bar_j(k);
        const bool pass = valid && dv <= bound && lex_less(dv, jv, tau_d, tau_j);
        uint64_t m = __ballot(pass);
        if (m == 0) return false;
        const int lane = (int)__lane_id();
        if (__popcll(m) >= kKnnBulkFrom) {
            // many candidates: sort them descending, take the lane-wise minimum with the
            // ascending list (the 64 smallest of both, a bitonic sequence), sort that
            const uint64_t unused = knn_key(__builtin_huge_valf(), 0x7fffffff);
            uint64_t c = wave_sort_desc(pass ? knn_key(dv, jv) : unused, lane);
            const uint64_t mine = knn_key(d, j);
            c = wave_merge_asc(c < mine ? c : mine, lane);
            if (lane >= k) c = unused;
            d = float_from_order_key((uint32_t)(c >> 32));
            j = (int)(uint32_t)c;
            return true;
        }
        bool changed = false;
        do {
            const int src = (int)__builtin_ctzll(m);                 // wavefront-uniform
            m &= m - 1;
            const float x = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(dv), src));
            const int xj = __builtin_amdgcn_readlane(jv, src);
            if (!lex_less(x, xj, tau_d, tau_j)) continue;            // the list improved meanwhile
            const int pos = (int)__popcll(__ballot(lex_less(d, j, x, xj)));   // sorted: a prefix
            const float sd = __int_as_float(wave_shr1(__float_as_int(d)));
            const int sj = wave_shr1(j);
            if (lane > pos) { d = sd; j = sj; }
            else if (lane == pos) { d = x; j = xj; }
            tau_d = bar_d(k);
            tau_j = bar_j(k);
            changed = true;
        } while (m);
        return changed;
    }
};

// ------------------------------------------------------------------------------------
// fused k-NN inside the scan kernel: one list per staged row and workgroup, in LDS
// ------------------------------------------------------------------------------------
// The key no candidate reaches: (+infinity, the largest index).
constexpr uint64_t kKnnUnused = 0xFF8000007FFFFFFFull;
constexpr int kKnnQueue = 64;             // candidates a row's queue holds (one wavefront's offer always fits an empty queue)
constexpr int kKnnLockSpins = 1 << 24;    // bound of the wait for a row's lock (never reached: the holder does not wait for anyone)

// A staged row's selection state: `list` holds the best keys so far in ascending order (entry
// t at position t, kKnnUnused beyond the k-th), `queue` the candidates that passed the bound
// since the list was last brought up to date.
struct KnnRowArea { uint64_t list[kWave]; uint64_t queue[kKnnQueue]; };
static_assert(sizeof(KnnRowArea) == kKnnAreaBytes, "the planner sizes the launch with kKnnAreaBytes per row");

// Merges the first `cnt` queued candidates into the list (the whole wavefront takes part: the
// queue is sorted descending, its lane-wise minimum with the ascending list is a bitonic
// sequence of the 64 smallest keys of both) and returns the list's new k-th key.
__device__ __forceinline__ uint64_t knn_merge_queue(KnnRowArea *area, int cnt, int k, int lane) {
    uint64_t c = lane < cnt ? area->queue[lane] : kKnnUnused;
    c = wave_sort_desc(c, lane);
    const uint64_t mine = area->list[lane];
    c = wave_merge_asc(c < mine ? c : mine, lane);
    if (lane >= k) c = kKnnUnused;
    area->list[lane] = c;
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)c, k - 1);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(c >> 32), k - 1);
    return ((uint64_t)hi << 32) | lo;
}

// The largest / the t-th smallest of the wavefront's 64 values (t >= 1; equal values count once each).
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
    uint32_t o;
    o = lane_xor<1>(v); v = o > v ? o : v;   o = lane_xor<2>(v); v = o > v ? o : v;
    o = lane_xor<4>(v); v = o > v ? o : v;   o = lane_xor<8>(v); v = o > v ? o : v;
    o = lane_xor<16>(v); v = o > v ? o : v;  o = lane_xor<32>(v); v = o > v ? o : v;
    return v;
}
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
    uint32_t o;
    o = lane_xor<1>(v); v = o < v ? o : v;   o = lane_xor<2>(v); v = o < v ? o : v;
    o = lane_xor<4>(v); v = o < v ? o : v;   o = lane_xor<8>(v); v = o < v ? o : v;
    o = lane_xor<16>(v); v = o < v ? o : v;  o = lane_xor<32>(v); v = o < v ? o : v;
    return v;
}
__device__ __forceinline__ uint32_t wave_kth_smallest_u32(uint32_t v, int t, int lane) {
    uint64_t out = 0;                            // lanes whose value was counted already (wavefront-uniform)
    uint32_t least = 0;
    for (int round = 0; round < t; ++round) {
        const uint32_t x = ((out >> lane) & 1u) ? 0xFFFFFFFFu : v;
        least = wave_min_u32(x);
        const uint64_t holders = __ballot(x == least);
        out |= holders & (0 - holders);          // one of them leaves
    }
    return least;
}

// Every lane may offer one candidate key for the staged row whose state is (area, tau, count,
// lock).  Candidates below the row's bound are appended to its queue under the row's lock; a
// queue that cannot take them is merged into the list first, which tightens the bound.  The
// lock is held for a few dozen instructions by a wavefront that waits for nothing meanwhile.
__device__ __forceinline__ void knn_offer(KnnRowArea *area, unsigned long long *tau_p, int *count_p, int *lock_p,
                                          uint64_t key, bool valid, uint64_t tau, int k, int lane) {
    bool pass = valid && key < tau;
    uint64_t m = __ballot(pass);
    if (m == 0) return;
    if (lane == 0) {
        int spins = 0;
        while (atomicCAS(lock_p, 0, 1) != 0 && ++spins < kKnnLockSpins) __builtin_amdgcn_s_sleep(1);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    int cnt = wave_uniform(__atomic_load_n(count_p, __ATOMIC_RELAXED));
    int n = (int)__popcll(m);
    if (cnt + n > kKnnQueue) {
        const uint64_t now = knn_merge_queue(area, cnt, k, lane);
        if (lane == 0) atomicMin(tau_p, (unsigned long long)now);   // (never above a bar that was seeded)
        cnt = 0;
        pass = pass && key < now;               // the merge may have ruled some of them out
        m = __ballot(pass);
        n = (int)__popcll(m);
    }
    if (pass) area->queue[cnt + (int)lane_rank_in(m)] = key;
    if (lane == 0) __atomic_store_n(count_p, cnt + n, __ATOMIC_RELAXED);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    if (lane == 0) __atomic_store_n(lock_p, 0, __ATOMIC_RELAXED);
}

// c ? b : a on any plain struct, word by word (selects, no branch).
template <typename T> __device__ __forceinline__ T select_words(bool c, const T &a, const T &b) {
    static_assert(sizeof(T) % 4 == 0, "whole words");
    constexpr int N = (int)(sizeof(T) / 4);
    uint32_t wa[N], wb[N];
    __builtin_memcpy(wa, &a, sizeof(T));
    __builtin_memcpy(wb, &b, sizeof(T));
#pragma unroll
    for (int i = 0; i < N; ++i) wa[i] = c ? wb[i] : wa[i];
    T out;
    __builtin_memcpy(&out, wa, sizeof(T));
    return out;
}

template <typename T> __device__ __forceinline__ T shfl_xor_any(T v, int mask);
template <> __device__ __forceinline__ double shfl_xor_any<double>(double v, int mask) { return __shfl_xor(v, mask); }
template <> __device__ __forceinline__ float shfl_xor_any<float>(float v, int mask) { return __shfl_xor(v, mask); }
template <> __device__ __forceinline__ int shfl_xor_any<int>(int v, int mask) { return __shfl_xor(v, mask); }

template <int OP> __device__ __forceinline__ typename Op<OP>::Acc acc_shfl_xor(const typename Op<OP>::Acc &a, int m);
#define SPD_ACC_SHFL1(OPID, FIELD)                                                              \
    template <> __device__ __forceinline__ Op<OPID>::Acc acc_shfl_xor<OPID>(const Op<OPID>::Acc &a, int m) { \
        Op<OPID>::Acc r; r.FIELD = shfl_xor_any(a.FIELD, m); return r; }
SPD_ACC_SHFL1(OP_DOT, v)
SPD_ACC_SHFL1(OP_L1, v)
SPD_ACC_SHFL1(OP_CANB, v)
SPD_ACC_SHFL1(OP_HAMM, c)
SPD_ACC_SHFL1(OP_CNT, c)
SPD_ACC_SHFL1(OP_CHEB, m)
SPD_ACC_SHFL1(OP_SEMI_EXT, m)
template <> __device__ __forceinline__ Op<OP_MINK>::Acc acc_shfl_xor<OP_MINK>(const Op<OP_MINK>::Acc &a, int m) {
    Op<OP_MINK>::Acc r; r.d = __shfl_xor(a.d, m); r.s = __shfl_xor(a.s, m); r.hits = __shfl_xor(a.hits, m); return r;
}
template <> __device__ __forceinline__ Op<OP_SEMI_SUM>::Acc acc_shfl_xor<OP_SEMI_SUM>(const Op<OP_SEMI_SUM>::Acc &a, int m) {
    Op<OP_SEMI_SUM>::Acc r; r.d = __shfl_xor(a.d, m); r.s = __shfl_xor(a.s, m); r.hits = __shfl_xor(a.hits, m); return r;
}
template <> __device__ __forceinline__ Op<OP_MINK_ANY>::Acc acc_shfl_xor<OP_MINK_ANY>(const Op<OP_MINK_ANY>::Acc &a, int m) {
    return acc_shfl_xor<OP_MINK>(a, m);
}
template <> __device__ __forceinline__ Op<OP_KL>::Acc acc_shfl_xor<OP_KL>(const Op<OP_KL>::Acc &a, int m) {
    Op<OP_KL>::Acc r; r.v = __shfl_xor(a.v, m); r.hits = __shfl_xor(a.hits, m); return r;
}
template <> __device__ __forceinline__ Op<OP_JS>::Acc acc_shfl_xor<OP_JS>(const Op<OP_JS>::Acc &a, int m) {
    Op<OP_JS>::Acc r; r.f = __shfl_xor(a.f, m); r.s = __shfl_xor(a.s, m); return r;
}

// ------------------------------------------------------------------------------------
// column -> slot of the staged value table
// ------------------------------------------------------------------------------------
// The hash table is an array of buckets of two {column, slot} entries, read with one
// 16-byte LDS load.  A lookup reads a fixed number of buckets, the same in every lane, with no
// branch (a column that was never staged, and the idle column, which is the empty key, come
// out as slot 0).  Two ways of filling it:
//  * sparse tables (a quarter full or less): an entry is claimed in the first free place of
//    its home bucket, else of the next bucket; the longest such walk is recorded and is the
//    number of buckets a lookup reads (one or two, rarely three);
//  * denser tables: every column has two candidate buckets (two hash functions) and an
//    insertion that finds both full moves an older entry to its other bucket (cuckoo
//    hashing): a lookup reads exactly the two.  Half full, linear probing would walk 8 to 13
//    buckets for its unluckiest entry, and every lookup would have to read as many.
//
// KIND_BITMAP replaces the table by one bit per column of the matrix and, per word of 32 bits,
// the number of staged columns before it: one 8-byte read at a place the column number gives
// directly, no multiplication, no comparison of keys (it fits while the column count stays
// under some 200,000).
//
// KIND_BLOOM keeps no table at all: the row's columns set two bits each of a Bloom filter in
// LDS, and a column that finds both of its bits set is searched for in the row itself (global
// memory, ascending columns: a binary search of a fixed number of steps).  The "slot" is the
// entry's position in the row plus one, 0 for a column the row does not store.
template <int KIND> struct ColumnMap {
    const uint32_t *bits;     // KIND_BLOOM: the filter, `mask` + 1 bits
    const int32_t *row_cols;  // KIND_BLOOM: the staged row's columns (global memory)
    int row_len, search_steps;
    const uint16_t *slot16;   // KIND_SLOT: k+1 entries
    const uint2 *words;       // KIND_BITMAP: per 32 columns {their bits, staged columns below the word + 1}
    const uint4 *table;       // KIND_HASH: buckets {column, slot, column, slot}, empty = {kEmptyKey, 0}
    uint32_t mask, shift;     // over buckets
    uint32_t mult1, mult2;    // odd multipliers of the two hash functions
    bool two_choice;          // KIND_HASH: the second way
    int reach;                // KIND_HASH: buckets a lookup reads (at least 1)
    __device__ __forceinline__ uint32_t home(uint32_t c) const { return (c * mult1) >> shift; }
    __device__ __forceinline__ uint32_t other(uint32_t c) const { return (c * mult2) >> shift; }
    __device__ __forceinline__ static uint32_t match(uint32_t c, uint4 e, uint32_t slot) {
        slot = (e.x == c) ? e.y : slot;
        return (e.z == c) ? e.w : slot;
    }
    // The i-th bucket (i >= 1) a lookup of column c reads after its home bucket h.
    __device__ __forceinline__ uint32_t next_bucket(uint32_t c, uint32_t h, int i) const {
        return two_choice ? other(c) : ((h + (uint32_t)i) & mask);
    }
    // the two filter bits of column c
    __device__ __forceinline__ uint32_t bit1(uint32_t c) const { return ((c * mult1) >> shift) & mask; }
    __device__ __forceinline__ uint32_t bit2(uint32_t c) const { return ((c * mult2) >> shift) & mask; }
    __device__ __forceinline__ uint32_t lookup(uint32_t c) const {
        if constexpr (KIND == KIND_STRIP) return c;
        else if constexpr (KIND == KIND_SLOT) return slot16[c];
        else if constexpr (KIND == KIND_BITMAP) {
            // the slot of a staged column is its rank among the staged columns (plus one): the
            // count the word carries plus the bits below the column's own; 0 if its bit is clear
            // (the bit-field extract takes its offset and its width from the low five bits of
            // the operand: the column number serves as it is)
            const uint2 e = words[c >> 5];
            const uint32_t rank = (uint32_t)__builtin_popcount(__builtin_amdgcn_ubfe(e.x, 0u, c)) + e.y;
            return __builtin_amdgcn_ubfe(e.x, c, 1u) ? rank : 0u;
        }
        else if constexpr (KIND == KIND_BLOOM) {
            const uint32_t b1 = bit1(c), b2 = bit2(c);
            const bool maybe = ((bits[b1 >> 5] >> (b1 & 31u)) & (bits[b2 >> 5] >> (b2 & 31u)) & 1u) != 0u;
            uint32_t pos = 0u;
            if (maybe) {
                // first entry not below c: every probe stays inside [0, row_len)
                int lo = 0, hi = row_len;
                for (int it = 0; it < search_steps; ++it) {
                    if (lo < hi) {
                        const int mid = (lo + hi) >> 1;
                        if ((uint32_t)row_cols[mid] < c) lo = mid + 1; else hi = mid;
                    }
                }
                if (lo < row_len && (uint32_t)row_cols[lo] == c) pos = (uint32_t)lo + 1u;
            }
            return pos;
        } else {
            const uint32_t h = home(c);
            uint32_t slot = match(c, table[h], 0u);
            for (int i = 1; i < reach; ++i) slot = match(c, table[next_bucket(c, h, i)], slot);
            return slot;
        }
    }
};

constexpr int kCuckooKicks = 96;          // moves after which an insertion gives up
constexpr int kCuckooAttempts = 3;        // pairs of hash functions tried before linear probing takes over
__device__ __constant__ const uint32_t kHashMult[kCuckooAttempts][2] = {
    {0x9E3779B1u, 0x85EBCA77u}, {0xC2B2AE3Du, 0x27D4EB2Fu}, {0x165667B1u, 0xD3A2646Du}};

template <int R> struct RowVals { float v[R]; };

// Four floats stored with one instruction at an address that is only known to be 4-byte aligned.
struct __attribute__((packed, aligned(4))) Float4Unaligned { float x, y, z, w; };

// The value table is kept in planes of four staged rows: plane q holds, for every slot, the
// values of rows 4q .. 4q+3 in 16 bytes.  A wavefront's 16-byte reads at random slots then
// fall on all LDS banks alike (rows of 32 or 64 bytes would start on every other or every
// fourth bank group only and halve or quarter the rate).
template <int R> __device__ __forceinline__ uint32_t vals_index(uint32_t slot, int r, uint32_t nslots) {
    if constexpr (R <= 4) return slot * R + (uint32_t)r;
    else return ((uint32_t)(r >> 2) * nslots + slot) * 4u + (uint32_t)(r & 3);
}

template <int R> __device__ __forceinline__ RowVals<R> load_vals(const float *vals, uint32_t slot, uint32_t nslots) {
    RowVals<R> out;
    if constexpr (R == 1) {
        out.v[0] = vals[slot];
    } else if constexpr (R == 2) {
        float2 t = *reinterpret_cast<const float2 *>(vals + (size_t)slot * 2);
        out.v[0] = t.x; out.v[1] = t.y;
    } else {
#pragma unroll
        for (int q = 0; q < R / 4; ++q) {
            float4 t = *reinterpret_cast<const float4 *>(vals + ((size_t)q * nslots + slot) * 4);
            out.v[4 * q] = t.x; out.v[4 * q + 1] = t.y; out.v[4 * q + 2] = t.z; out.v[4 * q + 3] = t.w;
        }
    }
    return out;
}

// ------------------------------------------------------------------------------------
// the kernel
// ------------------------------------------------------------------------------------
template <int OP, int R, int KIND, bool KNN>
__global__ void __launch_bounds__(scan_max_block(OP, R, KNN))
    __attribute__((amdgpu_waves_per_eu(scan_min_waves(OP, R, KIND, KNN)))) spd_scan_kernel(const ScanArgs args) {
    using O = Op<OP>;
    using Acc = typename O::Acc;
    // sum() = max: a column that only the staged row stores still counts, and is completed from
    // the row's ranked entries (Chebyshev, and the semirings whose sum() is min or max)
    constexpr bool kCheb = (OP == OP_CHEB || OP == OP_SEMI_EXT);
    constexpr bool kSemi = (OP == OP_SEMI_SUM || OP == OP_SEMI_EXT);   // product() picked at run time
    constexpr bool kCnt = (OP == OP_CNT);          // set metrics: one byte of the table per staged row
    constexpr int W = table_words(OP, R);          // 4-byte words per slot of the value table
    static_assert(!kCnt || (R % 4 == 0), "byte counters come four to the word");
    static_assert(kTopRanks == 32, "a pair's visited ranks are the bits of one 32-bit word");
    static_assert(KIND != KIND_BLOOM || (R == 1 && bloom_serves(OP)), "a Bloom-staged row is alone in its workgroup");
    constexpr int U = kScanUnroll;
    // the instances compiled for 64 registers per lane (eight wavefronts per SIMD) keep the short pipeline, and so
    // do those behind the 16-bit strip, whose lookup is one LDS read and an address (the compiler carries their
    // slots through the long pipeline as 16 bits and clears the upper half again at every use: 65,536 x 26,000
    // rows, four rows per group, L1: 56.2 ms with the long pipeline, 54.1 with the short one)
    constexpr bool kDeepPipeline = KIND != KIND_BLOOM && KIND != KIND_SLOT && scan_min_waves(OP, R, KIND, KNN) < 8 && !kSemi;
    extern __shared__ __align__(16) unsigned char dyn[];
    __shared__ ARow s_rows[R];
    __shared__ uint32_t s_prefix[R + 1];
    __shared__ double s_na[R][2];
    __shared__ int s_ctr;
    __shared__ int s_reach;                      // hash staging: buckets the longest insertion walked
    __shared__ uint32_t s_scan[KIND == KIND_BITMAP ? 16 : 1];   // bitmap staging: the wavefronts' totals of the scan
    __shared__ unsigned long long s_knn_tau[KNN ? R : 1];   // k-NN: the k-th key of the row's list (the bar a candidate has to beat)
    __shared__ int s_knn_count[KNN ? R : 1];                // k-NN: candidates waiting in the row's queue
    __shared__ int s_knn_lock[KNN ? R : 1];                 // k-NN: 1 while a wavefront works on the row's queue
    __shared__ float s_top[kCheb ? R * kTopRanks : 1];
    __shared__ int s_topn[R];
    __shared__ uint32_t s_clo[kCheb ? R : 1], s_cspan[kCheb ? R : 1];   // column range a slice answers for

    const int tid = (int)threadIdx.x, nthr = (int)blockDim.x;
    const int lane = tid & 63, wave = tid >> 6, nw = nthr >> 6;

    // Consecutive workgroups are consecutive groups of rows on one chunk of B: whatever runs at the
    // same time, on any XCD, sweeps the same stretch of B, which the memory-side cache then serves
    // to all of them (giving each XCD a chunk of its own, so that its L2 alone is shared, measured
    // slower on every configuration: eight stretches of B in flight instead of one or two).
    const int chunk = (int)blockIdx.x / args.n_groups, g = (int)blockIdx.x % args.n_groups;
    const int slab_begin = args.chunk_begin[chunk], slab_end = args.chunk_begin[chunk + 1];
    if (slab_begin >= slab_end) {
        if constexpr (KNN) {
            // an empty chunk still owns its place in the candidate lists: mark it unused
            for (int e = tid; e < R * args.knn_k; e += nthr) {
                const int out = args.arows[(size_t)g * R + e / args.knn_k].out;
                if (out >= 0)
                    args.knn_part[args.knn_row_off[out] + (size_t)chunk * args.knn_k + e % args.knn_k] =
                        KnnEntry{__builtin_huge_valf(), 0x7fffffff};
            }
        }
        return;
    }

    if (tid < R) s_rows[tid] = args.arows[(size_t)g * R + tid];
    const uint32_t sumlen = (uint32_t)args.sumlen[g];
    const LdsLayout L = lds_layout(KIND, W, sumlen, args.k, kCheb, args.hscale);
    float *vals = reinterpret_cast<float *>(dyn + L.off_vals);
    uint16_t *slot16 = reinterpret_cast<uint16_t *>(dyn + L.off_map);
    uint4 *table = reinterpret_cast<uint4 *>(dyn + L.off_map);
    unsigned char *rank8 = dyn + L.off_rank;
    ColumnMap<KIND> cmap;
    cmap.slot16 = slot16;
    cmap.words = reinterpret_cast<const uint2 *>(dyn + L.off_map);
    cmap.table = table;
    cmap.mask = L.cap ? L.cap / 2u - 1u : 0u;
    cmap.shift = L.cap ? 33u - (uint32_t)__builtin_ctz(L.cap) : 0u;
    cmap.reach = 1;
    cmap.mult1 = 0x9E3779B1u;
    cmap.mult2 = 0x85EBCA77u;
    cmap.two_choice = false;
    cmap.bits = reinterpret_cast<const uint32_t *>(dyn + L.off_map);
    cmap.row_cols = args.a_indices;
    cmap.row_len = 0;
    cmap.search_steps = 0;
    if constexpr (KIND == KIND_BLOOM) {
        cmap.mask = L.cap - 1u;
        cmap.shift = 32u - (uint32_t)__builtin_ctz(L.cap);        // the high bits of the product
    }

    // ---- stage ------------------------------------------------------------------------
    // 1. clear the value table and the column map
    {
        uint32_t nv4 = (L.nslots * W + 3u) / 4u;
        float4 *v4 = reinterpret_cast<float4 *>(vals);
        for (uint32_t i = tid; i < nv4; i += nthr) v4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        if constexpr (KIND == KIND_SLOT) {
            uint32_t nw32 = (args.k + 2u) / 2u;
            uint32_t *m32 = reinterpret_cast<uint32_t *>(slot16);
            for (uint32_t i = tid; i < nw32; i += nthr) m32[i] = 0u;
        } else if constexpr (KIND == KIND_BITMAP) {
            uint2 *w2 = reinterpret_cast<uint2 *>(dyn + L.off_map);
            for (uint32_t i = tid; i < bitmap_words(args.k); i += nthr) w2[i] = make_uint2(0u, 0u);
        } else if constexpr (KIND == KIND_HASH) {
            for (uint32_t i = tid; i < L.cap / 2u; i += nthr) table[i] = make_uint4(kEmptyKey, 0u, kEmptyKey, 0u);
        } else if constexpr (KIND == KIND_BLOOM) {
            uint32_t *bits = reinterpret_cast<uint32_t *>(dyn + L.off_map);
            for (uint32_t i = tid; i < L.cap / 32u; i += nthr) bits[i] = 0u;
        }
        if constexpr (kCheb) {
            uint32_t nr4 = (L.nslots * R + 3u) / 4u;
            uint32_t *r32 = reinterpret_cast<uint32_t *>(rank8);
            for (uint32_t i = tid; i < nr4; i += nthr) r32[i] = 0xFFFFFFFFu;
        }
    }
    __syncthreads();
    if (tid == 0) {
        uint32_t acc = 0;
        for (int r = 0; r < R; ++r) { s_prefix[r] = acc; acc += (uint32_t)s_rows[r].len; }
        s_prefix[R] = acc;
        s_ctr = slab_begin;
        s_reach = 1;
    }
    KnnRowArea *knn_rows = reinterpret_cast<KnnRowArea *>(dyn + L.off_knn);
    if constexpr (KNN) {
        if (tid < R) { s_knn_tau[tid] = kKnnUnused; s_knn_count[tid] = 0; s_knn_lock[tid] = 0; }
        for (int e = tid; e < R * kWave; e += nthr) knn_rows[e / kWave].list[e % kWave] = kKnnUnused;
    }
    // 2. row norms: one wavefront per row, summed in a fixed order (Section 3.4)
    for (int r = wave; r < R; r += nw) {
        const int64_t start = s_rows[r].start;
        const int len = s_rows[r].len;
        double s0 = 0.0, s1 = 0.0;
        for (int qi = lane; qi < len; qi += 64)
            norm_accumulate(args.norm, transform_value(args.transform, args.a_values[start + qi]), args.q.p, s0, s1);
        for (int m = 32; m >= 1; m >>= 1) { s0 += __shfl_xor(s0, m); s1 += __shfl_xor(s1, m); }
        if (lane == 0) {
            double d0, d1;
            norm_derive(args.q.metric, args.q.k, s0, s1, d0, d1);
            s_na[r][0] = d0; s_na[r][1] = d1;
            const int out = s_rows[r].out;
            if (out <= -2 && chunk == 0) {
                args.partial_norms[(size_t)(-2 - out) * 2] = s0;
                args.partial_norms[(size_t)(-2 - out) * 2 + 1] = s1;
            }
        }
    }
    __syncthreads();
    // 3. every stored entry of the R rows claims a slot for its column.  Two rows that share
    //    a column may both write: either slot id will do, the fill below reads the winner.
    const uint32_t total = s_prefix[R];
    if constexpr (KIND != KIND_STRIP) {
        // inserts every stored entry's column (the slot id is the entry's position + 1)
        auto for_each_entry = [&](auto &&insert) {
            for (uint32_t e = tid; e < total; e += nthr) {
                int r = 0;
#pragma unroll
                for (int q = 1; q < R; ++q) r += (e >= s_prefix[q]) ? 1 : 0;
                const int64_t at = s_rows[r].start + (e - s_prefix[r]);
                const float t = transform_value(args.transform, args.a_values[at]);
                if (t != 0.0f) insert((uint32_t)args.a_indices[at], e + 1u);     // a stored zero is absent
            }
        };
        if constexpr (KIND == KIND_SLOT) {
            for_each_entry([&](uint32_t c, uint32_t id) { if (slot16[c] == 0) slot16[c] = (uint16_t)id; });
            __syncthreads();
        } else if constexpr (KIND == KIND_BITMAP) {
            // every stored column sets its bit; then the words' running counts: each thread sums
            // the bits of its run of consecutive words, the runs' sums are scanned over the
            // workgroup (inside the wavefronts, then over the wavefronts' totals), and each
            // thread walks its run again
            uint2 *w2 = reinterpret_cast<uint2 *>(dyn + L.off_map);
            for_each_entry([&](uint32_t c, uint32_t) { atomicOr(&w2[c >> 5].x, 1u << (c & 31u)); });
            __syncthreads();
            const uint32_t nwords = bitmap_words(args.k);
            const uint32_t per = (nwords + (uint32_t)nthr - 1u) / (uint32_t)nthr;
            const uint32_t w_begin = min((uint32_t)tid * per, nwords), w_end = min(w_begin + per, nwords);
            uint32_t mine = 0u;
            for (uint32_t w = w_begin; w < w_end; ++w) mine += (uint32_t)__builtin_popcount(w2[w].x);
            uint32_t incl = mine;                        // inclusive scan over the wavefront's lanes
#pragma unroll
            for (int d = 1; d < kWave; d <<= 1) {
                const uint32_t up = (uint32_t)__shfl_up((int)incl, d);
                if (lane >= d) incl += up;
            }
            if (lane == kWave - 1) s_scan[wave] = incl;
            __syncthreads();
            uint32_t before = 1u;                        // slot ids start at 1
            for (int w = 0; w < wave; ++w) before += s_scan[w];
            before += incl - mine;
            for (uint32_t w = w_begin; w < w_end; ++w) {
                const uint32_t bits = w2[w].x;
                w2[w].y = before;
                before += (uint32_t)__builtin_popcount(bits);
            }
            __syncthreads();
        } else if constexpr (KIND == KIND_BLOOM) {
            uint32_t *bits = reinterpret_cast<uint32_t *>(dyn + L.off_map);
            for_each_entry([&](uint32_t c, uint32_t) {
                const uint32_t b1 = cmap.bit1(c), b2 = cmap.bit2(c);
                atomicOr(&bits[b1 >> 5], 1u << (b1 & 31u));
                atomicOr(&bits[b2 >> 5], 1u << (b2 & 31u));
            });
            cmap.row_cols = args.a_indices + s_rows[0].start;
            cmap.row_len = s_rows[0].len;
            cmap.search_steps = 32 - __builtin_clz((uint32_t)cmap.row_len | 1u);   // halvings that empty [0, len)
            __syncthreads();
        } else {
            unsigned long long *t64 = reinterpret_cast<unsigned long long *>(table);   // entry = column | slot << 32
            const unsigned long long kEmpty64 = (unsigned long long)kEmptyKey;
            bool built = false;
            if (args.hscale == 1) {
                // dense table: two candidate buckets per column
                for (int attempt = 0; attempt < min(kCuckooAttempts, args.cuckoo_attempts) && !built; ++attempt) {
                    cmap.mult1 = kHashMult[attempt][0];
                    cmap.mult2 = kHashMult[attempt][1];
                    if (attempt > 0) {
                        for (uint32_t i = tid; i < L.cap / 2u; i += nthr) table[i] = make_uint4(kEmptyKey, 0u, kEmptyKey, 0u);
                        if (tid == 0) s_reach = 1;
                        __syncthreads();
                    }
                    for_each_entry([&](uint32_t c, uint32_t id) {
                        unsigned long long item = (unsigned long long)c | ((unsigned long long)id << 32);
                        uint32_t bkt = cmap.home(c);
                        for (int kick = 0; kick < kCuckooKicks; ++kick) {
                            unsigned long long *pair = t64 + 2u * bkt;
                            unsigned long long old = atomicCAS(&pair[0], kEmpty64, item);
                            if (old == kEmpty64 || (uint32_t)old == (uint32_t)item) return;
                            old = atomicCAS(&pair[1], kEmpty64, item);
                            if (old == kEmpty64 || (uint32_t)old == (uint32_t)item) return;
                            // both places taken: take one over and carry its entry to its other bucket
                            item = atomicExch(&pair[(kick ^ (int)(c >> 7)) & 1], item);
                            const uint32_t moved = (uint32_t)item;
                            const uint32_t b1 = cmap.home(moved), b2 = cmap.other(moved);
                            bkt = (b1 == bkt) ? b2 : b1;
                        }
                        atomicExch(&s_reach, -1);              // gave up: this pair of functions fails
                    });
                    __syncthreads();
                    built = wave_uniform(s_reach) > 0;
                    __syncthreads();
                }
                if (built) { cmap.two_choice = true; cmap.reach = 2; }
            }
            if (!built) {
                cmap.mult1 = kHashMult[0][0];
                cmap.two_choice = false;
                if (args.hscale == 1 && args.cuckoo_attempts > 0) {       // (what the failed attempts left behind)
                    for (uint32_t i = tid; i < L.cap / 2u; i += nthr) table[i] = make_uint4(kEmptyKey, 0u, kEmptyKey, 0u);
                    if (tid == 0) s_reach = 1;
                    __syncthreads();
                }
                for_each_entry([&](uint32_t c, uint32_t id) {
                    uint32_t h = cmap.home(c);
                    int walked = 1;
                    for (;; ++walked) {
                        uint32_t old = atomicCAS(&table[h].x, kEmptyKey, c);
                        if (old == kEmptyKey) { table[h].y = id; break; }
                        if (old == c) break;
                        old = atomicCAS(&table[h].z, kEmptyKey, c);
                        if (old == kEmptyKey) { table[h].w = id; break; }
                        if (old == c) break;
                        h = (h + 1u) & cmap.mask;
                    }
                    if (walked > 1) atomicMax(&s_reach, walked);
                });
                __syncthreads();
                cmap.reach = wave_uniform(s_reach);
            }
        }
    }
    // 4. fill the value table (a Bloom-staged row keeps its values where they are)
    for (uint32_t e = tid; e < (KIND == KIND_BLOOM ? 0u : total); e += nthr) {
        int r = 0;
#pragma unroll
        for (int q = 1; q < R; ++q) r += (e >= s_prefix[q]) ? 1 : 0;
        const int64_t at = s_rows[r].start + (e - s_prefix[r]);
        const float t = transform_value(args.transform, args.a_values[at]);
        if (t != 0.0f) {
            const uint32_t slot = cmap.lookup((uint32_t)args.a_indices[at]);
            if constexpr (kCnt)      // byte r & 3 of word r >> 2 of the slot
                reinterpret_cast<unsigned char *>(vals)[(size_t)vals_index<W>(slot, r >> 2, L.nslots) * 4 + (r & 3)] = 1;
            else vals[vals_index<R>(slot, r, L.nslots)] = t;
        }
    }
    if constexpr (kCheb) {
        // With sum() = max a column that a slice of a row does not store still counts
        // (|0 - b|), so each slice answers only for the columns from its first entry up to
        // the next slice's first entry (the partition membership test of Section 3.3.3).
        if (tid < R) {
            const ARow rw = s_rows[tid];
            uint32_t lo = (rw.flags & kRowFirst) ? 0u : (uint32_t)args.a_indices[rw.start];
            uint32_t hi = (rw.flags & kRowLast) ? 0xFFFFFFFFu : (uint32_t)args.a_indices[rw.start + rw.len] - 1u;
            s_clo[tid] = lo;
            s_cspan[tid] = hi - lo;
        }
    }
    __syncthreads();

    if constexpr (kCheb) {
        // The kTopRanks largest one-sided contributions (Chebyshev: |values|) of each staged
        // row, in order, and their ranks beside the value table: what a row of B leaves
        // unvisited is completed from them.  A product over the intersection has none.
        constexpr uint32_t kNone = 0xFFFFFFFFu;             // no column: columns stay below 2^31
        const bool one_sided = (OP == OP_CHEB) || args.q.over_union != 0;
        for (int r = wave; r < R; r += nw) {
            const int64_t start = s_rows[r].start;
            const int len = one_sided ? s_rows[r].len : 0;
            float prev_v = __builtin_huge_valf();
            uint32_t prev_c = 0u;
            bool first = true;
            int found = 0;
            for (int round = 0; round < kTopRanks; ++round) {
                float best_v = 0.0f;
                uint32_t best_c = kNone;
                for (int qi = lane; qi < len; qi += 64) {
                    const float a = args.a_values[start + qi];
                    const float v = one_sided_key<OP>(a, args.q);
                    uint32_t c = (uint32_t)args.a_indices[start + qi];
                    bool after_prev = first || v < prev_v || (v == prev_v && c > prev_c);
                    bool better = best_c == kNone || v > best_v || (v == best_v && c < best_c);
                    if (a != 0.0f && after_prev && better) { best_v = v; best_c = c; }
                }
                for (int m = 32; m >= 1; m >>= 1) {
                    float ov = __shfl_xor(best_v, m);
                    uint32_t oc = (uint32_t)__shfl_xor((int)best_c, m);
                    if (oc != kNone && (best_c == kNone || ov > best_v || (ov == best_v && oc < best_c))) { best_v = ov; best_c = oc; }
                }
                if (best_c == kNone) break;
                if (lane == 0) {
                    s_top[r * kTopRanks + round] = best_v;
                    rank8[(size_t)cmap.lookup(best_c) * R + r] = (unsigned char)round;
                }
                prev_v = best_v; prev_c = best_c; first = false;
                found = round + 1;
            }
            if (lane == 0) s_topn[r] = found;
        }
        __syncthreads();
    }

    // what the epilogue of every slab needs of the staged rows, once, in scalar registers
    int row_out[R];
    double row_na0[R], row_na1[R];
    uint32_t row_clo[kCheb ? R : 1], row_cspan[kCheb ? R : 1];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        row_out[r] = wave_uniform(s_rows[r].out);
        row_na0[r] = wave_uniform_f64(s_na[r][0]);
        row_na1[r] = wave_uniform_f64(s_na[r][1]);
        if constexpr (kCheb) {
            row_clo[r] = (uint32_t)wave_uniform((int)s_clo[r]);
            row_cspan[r] = (uint32_t)wave_uniform((int)s_cspan[r]);
        }
    }

    // The rows are finished eight at a time, or four (all at once would keep the sums and
    // distances of up to 32 rows in registers together).
    constexpr bool kThreeSums = (OP == OP_MINK || OP == OP_MINK_ANY || OP == OP_SEMI_SUM);
    constexpr int RB = R < 8 ? R : ((KNN && R >= 16) || kThreeSums ? 4 : 8);
    // Pairwise, with the staged operand along the output's rows (stride 1): a block of staged rows
    // that are consecutive rows of that operand is stored by each lane as 16-byte pieces of its
    // own output row.  Bit b: block b qualifies.
    uint32_t out_vector_blocks = 0u;
    if constexpr (!KNN && RB % 4 == 0) {
        if (args.out_stride_staged == 1) {
#pragma unroll
            for (int r0 = 0; r0 < R; r0 += RB) {
                bool ok = row_out[r0] >= 0;
#pragma unroll
                for (int i = 1; i < RB; ++i) ok = ok && row_out[r0 + i] == row_out[r0] + i;
                out_vector_blocks |= ok ? (1u << (r0 / RB)) : 0u;
            }
        }
    }

    // ---- scan: every wavefront takes slabs of the chunk until none is left -----------
    const int64_t n_b = args.b.n_rows;
    const float *bloom_values = args.a_values + (KIND == KIND_BLOOM ? s_rows[0].start : 0);

    // k-NN where the distance grows with the mass of B's row (L1, Minkowski, Canberra, Hamming,
    // Jensen-Shannon, Chebyshev): the lists meet the rows of B longest first, so the distances fall
    // from slab to slab and every slab brings a new set of candidates, on top of the first slabs,
    // which pass in full because the lists start empty.  Where the chunk has slabs enough, each
    // wavefront takes one of the chunk's last (shortest) slabs first and publishes, per staged row,
    // the t-th smallest of its 64 distances, t = ceil(k / wavefronts): the largest of these has k
    // distances of the chunk at or below it, so no key of the final list exceeds it, and it is known
    // before the first candidate is queued (10,000 x 10,000 rows, L1, k = 32: 0.87 -> 0.68 ms).  Not in
    // a chunk of a few slabs per wavefront (the short slabs are what evens out the wavefronts' shares
    // at the end), and not for cosine, correlation, the inner product and the set metrics, whose near
    // rows are the long ones: the short slabs' distances say nothing there, and the exchange costs 2-3 %.
    // (the dot product serves both kinds: the expanded Euclidean and Hellinger distances grow with the
    // row's mass, cosine, correlation and the inner product do not)
    constexpr bool kSeedPays = OP == OP_L1 || OP == OP_MINK || OP == OP_MINK_ANY || OP == OP_CANB || OP == OP_HAMM ||
                               OP == OP_JS || OP == OP_CHEB || OP == OP_DOT;
    bool seeding = false;
    int seed_rank = 1;
    if constexpr (KNN && kSeedPays) {
        seed_rank = (args.knn_k + nw - 1) / nw;
        seeding = args.knn_seed != 0 && slab_end - slab_begin >= 8 * nw && seed_rank <= 8 &&      // the same in every wavefront
                  (OP != OP_DOT || args.q.metric == MT_L2 || args.q.metric == MT_HELLINGER);
    }
    const int taken_end = seeding ? slab_end - nw : slab_end;    // slabs [slab_begin, taken_end) go to whoever comes first
    for (;;) {
        int s = 0;
        if (seeding) {
            s = slab_end - 1 - wave;
        } else {
            if (lane == 0) s = atomicAdd(&s_ctr, 1);
            s = wave_uniform(s);
            if (s >= taken_end) break;
        }
        const size_t at = (size_t)s * kWave + lane;
        const int row = args.b.seg_row[at];
        const int steps = wave_uniform(args.b.slab_steps[s]);
        const int split_depth = wave_uniform((int)args.b.slab_split[s]);   // deepest split of a row in the slab
        const uint2 *__restrict__ pk = args.b.packed + args.b.slab_base[s] + lane;
        Acc acc[R];
        uint32_t hit[kCheb ? R : 1];
        uint32_t counts[kCnt ? W : 1];            // set metrics: four byte counters to the word
#pragma unroll
        for (int r = 0; r < R; ++r) { O::init(acc[r]); if constexpr (kCheb) hit[r] = 0u; }
        if constexpr (kCnt) {
#pragma unroll
            for (int w = 0; w < W; ++w) counts[w] = 0u;
        }

        // Entry t of lane l sits at pk[t*64 + l]: one coalesced load per step, fetched a block
        // of U steps ahead of its use.  The plan pads every slab to whole blocks (with the
        // column that stages nothing), so the loop has no tail.
        auto fetch_block = [&](uint2 (&into)[U], int t_first) {
            const uint2 *__restrict__ src = pk + (size_t)t_first * kWave;
#pragma unroll
            for (int u = 0; u < U; ++u) into[u] = src[u * kWave];
        };
        auto visit_step = [&](const uint2 entry, const uint32_t slot) {
            if constexpr (kCnt) {
                // the slot's R bytes are 0 or 1: adding its words counts the shared columns of all
                // R rows at once
                const RowVals<W> a = load_vals<W>(vals, slot, L.nslots);
#pragma unroll
                for (int w = 0; w < W; ++w) counts[w] += __float_as_uint(a.v[w]);
            } else {
                const typename O::Bv bv = O::prep(__uint_as_float(entry.y), args.q);
                RowVals<R> a;
                if constexpr (KIND == KIND_BLOOM) {
                    // slot = position in the row + 1 (0: not stored)
                    a.v[0] = slot ? transform_value(args.transform, bloom_values[slot - 1u]) : 0.0f;
                } else {
                    a = load_vals<R>(vals, slot, L.nslots);
                }
                // (a semiring's product and Minkowski's degree are run-time choices: they are
                // switched on once per step, not once per visit)
                auto visit_rows = [&](auto product_tag) {
                    constexpr int P = decltype(product_tag)::value;
                    constexpr bool kUnion = decltype(product_tag)::over_union;
                    // (over the intersection a slice meets only its own columns and nothing is
                    // one-sided: no range to check, no ranks to mark)
                    if constexpr (kCheb && (kUnion || !kSemi)) {
                        const unsigned char *rk = rank8 + (size_t)slot * R;
#pragma unroll
                        for (int r = 0; r < R; ++r) {
                            if (entry.x - row_clo[r] <= row_cspan[r]) visit_with<OP, P, kUnion>(acc[r], a.v[r], bv, args.q);
                            // a ranked entry's byte is its rank (below 32), any other byte is 255: a
                            // 64-bit one shifted by the byte's low six bits lands beyond bit 31 for those
                            const uint32_t q = rk[r];
                            hit[r] |= (uint32_t)(1ull << (q & 63u));
                        }
                    } else {
#pragma unroll
                        for (int r = 0; r < R; ++r) visit_with<OP, P, kUnion>(acc[r], a.v[r], bv, args.q);
                    }
                };
                if constexpr (kSemi) for_product(args.q.product, args.q.over_union != 0, visit_rows);
                else if constexpr (OP == OP_MINK) for_degree(args.q.p, visit_rows);
                else visit_rows(ProductTag<0>{});
            }
        };
        // Byte counters hold up to 255: they are folded into the pairs' 32-bit counts before a
        // byte can overflow, and at the end of the slab.
        int unfolded = 0;
        auto fold_counts = [&]() {
            if constexpr (kCnt) {
#pragma unroll
                for (int r = 0; r < R; ++r) acc[r].c += (int)((counts[r >> 2] >> (8 * (r & 3))) & 0xffu);
#pragma unroll
                for (int w = 0; w < W; ++w) counts[w] = 0u;
                unfolded = 0;
            }
        };
        // the slots of a block's columns (the LDS reads of a block are issued together)
        auto lookup_block = [&](const uint2 (&cur)[U], uint32_t (&slot)[U]) {
            if constexpr (KIND == KIND_HASH) {
                uint32_t h[U];
                uint4 e[U];
#pragma unroll
                for (int u = 0; u < U; ++u) { h[u] = cmap.home(cur[u].x); e[u] = table[h[u]]; }
#pragma unroll
                for (int u = 0; u < U; ++u) slot[u] = ColumnMap<KIND>::match(cur[u].x, e[u], 0u);
                for (int i = 1; i < cmap.reach; ++i) {
#pragma unroll
                    for (int u = 0; u < U; ++u) e[u] = table[cmap.next_bucket(cur[u].x, h[u], i)];
#pragma unroll
                    for (int u = 0; u < U; ++u) slot[u] = ColumnMap<KIND>::match(cur[u].x, e[u], slot[u]);
                }
            } else {
#pragma unroll
                for (int u = 0; u < U; ++u) slot[u] = cmap.lookup(cur[u].x);
            }
        };
        auto visit_block = [&](const uint2 (&cur)[U], const uint32_t (&slot)[U]) {
            if constexpr (kCnt) {
                if (unfolded > kCntMaxSteps - U) fold_counts();
                unfolded += U;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) visit_step(cur[u], slot[u]);
        };
        // first step of the block that follows the one at t (past the slab's end the last block is
        // simply read again)
        auto block_after = [&](int t, int ahead) { return min(t + ahead * U, steps - U); };
        if (steps > 0) {
            if constexpr (kDeepPipeline) {
                // Three register sets take turns: while block t is worked on, the columns of block
                // t + 1 are being looked up in LDS and block t + 2 is in flight from memory.  (A
                // launch that the LDS holds to a few wavefronts per SIMD has nobody else to hide the
                // two dependent LDS reads of a step behind.)
                uint2 e0[U], e1[U], e2[U];
                uint32_t s0[U], s1[U], s2[U];
                fetch_block(e0, 0);
                fetch_block(e1, block_after(0, 1));
                lookup_block(e0, s0);
                for (int t0 = 0;;) {
                    fetch_block(e2, block_after(t0, 2));
                    lookup_block(e1, s1);
                    __builtin_amdgcn_sched_barrier(0);    // keep the loads and lookups ahead of the arithmetic
                    visit_block(e0, s0);
                    t0 += U;
                    if (t0 >= steps) break;
                    fetch_block(e0, block_after(t0, 2));
                    lookup_block(e2, s2);
                    __builtin_amdgcn_sched_barrier(0);
                    visit_block(e1, s1);
                    t0 += U;
                    if (t0 >= steps) break;
                    fetch_block(e1, block_after(t0, 2));
                    lookup_block(e0, s0);
                    __builtin_amdgcn_sched_barrier(0);
                    visit_block(e2, s2);
                    t0 += U;
                    if (t0 >= steps) break;
                }
            } else {
                // two register sets take turns: while one block is worked on, the next one is in flight
                uint2 even[U], odd[U];
                uint32_t slot[U];
                fetch_block(even, 0);
                for (int t0 = 0;;) {
                    fetch_block(odd, block_after(t0, 1));
                    __builtin_amdgcn_sched_barrier(0);        // keep the loads ahead of the arithmetic
                    lookup_block(even, slot);
                    visit_block(even, slot);
                    t0 += U;
                    if (t0 >= steps) break;
                    fetch_block(even, block_after(t0, 1));
                    __builtin_amdgcn_sched_barrier(0);
                    lookup_block(odd, slot);
                    visit_block(odd, slot);
                    t0 += U;
                    if (t0 >= steps) break;
                }
            }
        }

        if constexpr (kCnt) fold_counts();
        const int glog = args.b.seg_glog[at];
        if (split_depth > 0) {
            // rows cut over 2^glog adjacent lanes: sum (max) the lanes of each group
#pragma unroll
            for (int step = 0; step < 6; ++step) {
                if (step >= split_depth) break;
                const bool mine = step < glog;
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    Acc merged = acc[r];
                    O::combine(merged, acc_shfl_xor<OP>(acc[r], 1 << step));
                    acc[r] = select_words(mine, acc[r], merged);
                    if constexpr (kCheb) {
                        const uint32_t oh = (uint32_t)__shfl_xor((int)hit[r], 1 << step);
                        hit[r] |= mine ? oh : 0u;
                    }
                }
            }
        }
        const bool leader = row >= 0 && (lane & ((1 << glog) - 1)) == 0;
        double nb0 = 0.0, nb1 = 0.0;
        if (leader) { nb0 = args.b.norms[(size_t)row * 2]; nb1 = args.b.norms[(size_t)row * 2 + 1]; }

#pragma unroll
        for (int r0 = 0; r0 < R; r0 += RB) {
            double v0[RB], v1[RB], v2[RB];
#pragma unroll
            for (int i = 0; i < RB; ++i) { v0[i] = O::v0(acc[r0 + i]); v1[i] = O::v1(acc[r0 + i]); v2[i] = O::v2(acc[r0 + i]); }
            if constexpr (kCheb) {
#pragma unroll
                for (int i = 0; i < RB; ++i) {
                    const int r = r0 + i;
                    if (row_out[r] == -1) continue;
                    if (leader) {
                        const int topn = s_topn[r];
                        uint32_t tracked = topn >= 32 ? 0xFFFFFFFFu : ((1u << topn) - 1u);
                        uint32_t unhit = ~hit[r] & tracked;
                        float extra = -__builtin_huge_valf();
                        if (unhit) {
                            extra = s_top[r * kTopRanks + __builtin_ctz(unhit)];
                        } else if (topn == kTopRanks) {
                            // every tracked entry was visited: walk the two sorted rows
                            const int64_t a0 = s_rows[r].start, a1 = a0 + s_rows[r].len;
                            int64_t bj = args.b_indptr[row];
                            const int64_t be = args.b_indptr[row + 1];
                            for (int64_t ai = a0; ai < a1; ++ai) {
                                int32_t c = args.a_indices[ai];
                                while (bj < be && args.b_indices[bj] < c) ++bj;
                                const float av = args.a_values[ai];
                                if ((bj >= be || args.b_indices[bj] != c) && av != 0.0f)
                                    extra = fmaxf(extra, one_sided_key<OP>(av, args.q));
                            }
                        }
                        v0[i] = fmax(v0[i], (double)extra);
                    }
                }
            }
            // the expansion function is picked once per eight rows, not once per pair
            float dist[RB];
            for_metric_of<OP>(args.q.metric, [&](auto metric_tag) {
                constexpr int MT = decltype(metric_tag)::value;
#pragma unroll
                for (int i = 0; i < RB; ++i) {
                    dist[i] = finish_as<MT>(args.q, v0[i], v1[i], v2[i], row_na0[r0 + i], row_na1[r0 + i], nb0, nb1);
                    if constexpr (KNN && MT == MT_INNER) dist[i] = 0.0f - dist[i];   // largest first; never -0: keys order by bit pattern
                }
            });
            if constexpr (!KNN) {
                if (leader) {
                    bool stored = false;
                    if constexpr (RB % 4 == 0) {
                        // the staged rows of this block are neighbours in the lane's output row: 16-byte stores
                        if ((out_vector_blocks >> (r0 / RB)) & 1u) {
                            float *dst = args.out + ((size_t)row * (size_t)args.out_stride_streamed + (size_t)row_out[r0]);
#pragma unroll
                            for (int i = 0; i < RB; i += 4)
                                *reinterpret_cast<Float4Unaligned *>(dst + i) = Float4Unaligned{dist[i], dist[i + 1], dist[i + 2], dist[i + 3]};
                            stored = true;
                        }
                    }
                    if (!stored) {
#pragma unroll
                        for (int i = 0; i < RB; ++i) {
                            const int out = row_out[r0 + i];
                            if (out >= 0)
                                args.out[(size_t)out * (size_t)args.out_stride_staged + (size_t)row * (size_t)args.out_stride_streamed] = dist[i];
                        }
                    }
                }
            } else {
                if (kSeedPays && seeding) {
                    // (every wavefront of the workgroup is here, on its first slab: the rows' queues are still
                    // empty and lend their first places to the exchange)
#pragma unroll
                    for (int i = 0; i < RB; ++i) {
                        const int r = r0 + i;
                        if (row_out[r] < 0) continue;
                        const uint32_t mine = leader ? (uint32_t)(knn_key(dist[i], row) >> 32) : (uint32_t)(kKnnUnused >> 32);
                        const uint32_t kth = wave_kth_smallest_u32(mine, seed_rank, lane);
                        if (lane == 0) knn_rows[r].queue[wave] = kth;
                    }
                    __syncthreads();
                    if (wave == 0) {
#pragma unroll
                        for (int i = 0; i < RB; ++i) {
                            const int r = r0 + i;
                            if (row_out[r] < 0) continue;
                            const uint32_t theirs = wave_max_u32(lane < nw ? (uint32_t)knn_rows[r].queue[lane] : 0u);
                            // (any index passes at that distance)
                            if (lane == 0) atomicMin(&s_knn_tau[r], ((unsigned long long)theirs << 32) | 0x7FFFFFFFull);
                        }
                    }
                    __syncthreads();          // the bars are set, and read, before the first candidate is queued
                }
#pragma unroll
                for (int i = 0; i < RB; ++i) {
                    const int r = r0 + i;
                    if (row_out[r] < 0) continue;
                    // (the bound may be out of date: then it is only looser)
                    const uint64_t tau = (uint64_t)__atomic_load_n(&s_knn_tau[r], __ATOMIC_RELAXED);
                    const float bound = float_from_order_key((uint32_t)(tau >> 32));
                    if (__ballot(leader && dist[i] <= bound) == 0) continue;      // the usual case once the list is warm
                    knn_offer(&knn_rows[r], &s_knn_tau[r], &s_knn_count[r], &s_knn_lock[r], knn_key(dist[i], row), leader, tau,
                              args.knn_k, lane);
                }
            }
            if (leader) {
#pragma unroll
                for (int i = 0; i < RB; ++i) {
                    const int out = row_out[r0 + i];
                    if (out > -2) continue;
                    const size_t slot = (size_t)(-2 - out);
                    args.partial[(slot * args.planes) * (size_t)n_b + (size_t)row] = v0[i];
                    if (args.planes >= 2) args.partial[(slot * args.planes + 1) * (size_t)n_b + (size_t)row] = v1[i];
                    if (args.planes == 3) args.partial[(slot * 3 + 2) * (size_t)n_b + (size_t)row] = v2[i];
                }
            }
        }
        seeding = false;                              // from the second slab on: first come, first served
    }

    // ---- k-NN: what is still queued joins the lists, which go to the chunk's place in memory --
    if constexpr (KNN) {
        const int kk = args.knn_k;
        __syncthreads();                              // every wavefront has left the scan
        for (int r = wave; r < R; r += nw) {
            const int out = s_rows[r].out;
            if (out < 0) continue;
            knn_merge_queue(&knn_rows[r], s_knn_count[r], kk, lane);
            const uint64_t key = knn_rows[r].list[lane];
            if (lane < kk)
                args.knn_part[args.knn_row_off[out] + (size_t)chunk * kk + lane] =
                    KnnEntry{float_from_order_key((uint32_t)(key >> 32)), (int)(uint32_t)key};
        }
    }
}

template <int OP, int R, int KIND, bool KNN>
static hipError_t launch_scan_rkk(hipStream_t st, int block, uint32_t lds_bytes, const ScanArgs &args) {
    if (block > scan_max_block(OP, R, KNN) || block < kWave || (block & (kWave - 1))) return hipErrorInvalidValue;
    auto kern = spd_scan_kernel<OP, R, KIND, KNN>;
    // the instance's LDS limit is raised once per device (to the most a launch may ask for), not
    // at every launch
    constexpr int kMaxDevices = 64;
    static std::atomic<uint32_t> allowed[kMaxDevices];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices || allowed[dev].load(std::memory_order_acquire) < lds_bytes) {
        const uint32_t want = std::max<uint32_t>(lds_bytes, 160u * 1024u - kStaticLds);
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)want);
        if (e != hipSuccess) {
            // a device with less LDS: ask for what this launch needs
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
            if (e != hipSuccess) return e;
        } else if (dev >= 0 && dev < kMaxDevices) {
            allowed[dev].store(want, std::memory_order_release);
        }
    }
    dim3 grid((unsigned)((size_t)args.n_groups * (size_t)args.n_chunks));
    hipLaunchKernelGGL(kern, grid, dim3((unsigned)block), lds_bytes, st, args);
    return hipGetLastError();
}

// WHICH: 0 = pairwise instances only, 1 = fused k-NN instances only, 2 = both (a product whose
// instances take long to compile is spread over two translation units).
template <int OP, int R, int WHICH>
static hipError_t launch_scan_r(hipStream_t st, int block, uint32_t lds_bytes, const ScanArgs &args) {
    const bool knn = args.knn_k > 0;
    if ((knn && WHICH == 0) || (!knn && WHICH == 1)) return hipErrorInvalidValue;
    if constexpr (WHICH != 0) {
        if (knn) {
            switch (args.kind) {
            case KIND_STRIP: return launch_scan_rkk<OP, R, KIND_STRIP, true>(st, block, lds_bytes, args);
            case KIND_SLOT: return launch_scan_rkk<OP, R, KIND_SLOT, true>(st, block, lds_bytes, args);
            case KIND_HASH: return launch_scan_rkk<OP, R, KIND_HASH, true>(st, block, lds_bytes, args);
            case KIND_BITMAP: return launch_scan_rkk<OP, R, KIND_BITMAP, true>(st, block, lds_bytes, args);
            case KIND_BLOOM:
                if constexpr (R == 1 && bloom_serves(OP)) return launch_scan_rkk<OP, R, KIND_BLOOM, true>(st, block, lds_bytes, args);
                else return hipErrorInvalidValue;
            default: return hipErrorInvalidValue;
            }
        }
    }
    if constexpr (WHICH != 1) {
        switch (args.kind) {
        case KIND_STRIP: return launch_scan_rkk<OP, R, KIND_STRIP, false>(st, block, lds_bytes, args);
        case KIND_SLOT: return launch_scan_rkk<OP, R, KIND_SLOT, false>(st, block, lds_bytes, args);
        case KIND_HASH: return launch_scan_rkk<OP, R, KIND_HASH, false>(st, block, lds_bytes, args);
        case KIND_BITMAP: return launch_scan_rkk<OP, R, KIND_BITMAP, false>(st, block, lds_bytes, args);
        case KIND_BLOOM:
            if constexpr (R == 1 && bloom_serves(OP)) return launch_scan_rkk<OP, R, KIND_BLOOM, false>(st, block, lds_bytes, args);
            else return hipErrorInvalidValue;
        default: return hipErrorInvalidValue;
        }
    }
    return hipErrorInvalidValue;
}

template <int OP, int WHICH = 2>
static hipError_t launch_scan_op(hipStream_t st, int R, int block, uint32_t lds_bytes, const ScanArgs &args) {
    if constexpr (OP == OP_CNT) {
        // four rows to the word of the table; 32 rows only without the k-NN lists
        switch (R) {
        case 4: return launch_scan_r<OP, 4, WHICH>(st, block, lds_bytes, args);
        case 8: return launch_scan_r<OP, 8, WHICH>(st, block, lds_bytes, args);
        case 16: return launch_scan_r<OP, 16, WHICH>(st, block, lds_bytes, args);
        case 32: return launch_scan_r<OP, 32, WHICH>(st, block, lds_bytes, args);
        default: return hipErrorInvalidValue;
        }
    } else {
        switch (R) {
        case 1: return launch_scan_r<OP, 1, WHICH>(st, block, lds_bytes, args);
        case 2: return launch_scan_r<OP, 2, WHICH>(st, block, lds_bytes, args);
        case 4: return launch_scan_r<OP, 4, WHICH>(st, block, lds_bytes, args);
        case 8:
            if constexpr (OP == OP_MINK || OP == OP_MINK_ANY || OP == OP_SEMI_SUM || OP == OP_SEMI_EXT) return hipErrorInvalidValue;
            else return launch_scan_r<OP, 8, WHICH>(st, block, lds_bytes, args);
        case 16:
            if constexpr (OP == OP_JS || OP == OP_MINK || OP == OP_MINK_ANY || OP == OP_SEMI_SUM || OP == OP_SEMI_EXT) return hipErrorInvalidValue;
            else return launch_scan_r<OP, 16, WHICH>(st, block, lds_bytes, args);
        default: return hipErrorInvalidValue;
        }
    }
}

}  // namespace spd
