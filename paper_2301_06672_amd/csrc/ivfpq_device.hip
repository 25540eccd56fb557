// Device half of libivfpq: upload of the index image and the HIP kernels of the IVFPQ search phase
// (arXiv 2301.06672, Sec. I-C second enumeration, Sec. I-D, Sec. II) for gfx950 (MI355X, wave64).
//
// Kernels, in the order one search call runs them (per tile of queries):
//   coarse_rank_*_kernel step 1a: ranking values |c|^2 - 2 q.c of every (query, cluster) pair on the
//                        matrix cores: bf16 instructions on operands split in two for large problems,
//                        fp32 otherwise; stored as all keys (few clusters) or as the three smallest
//                        tagged keys of every strip of 32 / 64 clusters
//   select_probes_kernel step 1b: candidates by ranking value with a rigorous error bound, exact
//                        direct-form distances for them, exact selection of the n_probes nearest
//                        clusters; per-pair descriptors and R offsets
//   scan_kernel (mode 1) steps 2-4 for the nearest probe of every query: query residual, lookup table F
//                        built in LDS as fp32 / half / e5m3 / e4m4, then every wave streams 64-vector
//                        groups of PQ codes from HBM and accumulates R = sum_j F(y_j) (Eq. 1)
//   bound_kernel         the k-th smallest R of that nearest cluster: an upper bound of the final
//                        k-th distance of the query; the cluster's values under it start the survivor list
//   pair_count / pair_offsets / pair_scatter   the other (query, probe) pairs grouped by cluster
//                        (counts per workgroup in LDS first when there are few clusters)
//   scan_kernel (mode 2) steps 2-4 for the other probes, in cluster-grouped, XCD-aware order (a
//                        cluster's codes then come from one XCD's L2); only R values under the bound
//                        are kept
//   scan_group_kernel    the same for up to four neighbouring pairs of one cluster per workgroup (8- and 4-bit codes):
//                        their tables are interleaved entry by entry, so one LDS read serves one lookup of
//                        every query of the group; codebooks and codes are read once for all of them
//   topk_kernel          step 5: the k smallest R among the survivors of a query, ordered by
//                        (R, id), and the map from (cluster, position) to the caller's ids
// Beside the path: dump_lut_kernel (steps 2-3 of one pair, for inspection) and refine_kernel (exact
// re-ranking of candidates with the stored vectors).
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <algorithm>
#include <cstring>
#include <thread>
#include <type_traits>
#include <utility>

#include "ivfpq_internal.hpp"
#include "ivfpq_rank.hpp"
#include "ivfpq_lds_util.hpp"

using namespace ivfpq;

// The workspace of ivfpq_search_static: a fixed device array, so that callers who cannot allocate (HIP graph
// capture, serving loops, harnesses that forbid hipMalloc) need bring none.  Each GPU the library runs on holds
// its own copy at its own address until the process ends.  In host code this name is only a stand-in for the
// symbol: the array's device address comes from hipGetSymbolAddress (static_scratch_ptr), and only that pointer
// is ever handed to kernels.
static __device__ __align__(256) unsigned char scratch[IVFPQ_STATIC_SCRATCH_BYTES];

namespace {

constexpr size_t kStaticScratchBytes = IVFPQ_STATIC_SCRATCH_BYTES;

// Device address of `scratch` on the current device, looked up once per device.
int static_scratch_ptr(void** out) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void* ptr[kMaxDevices] = {};
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(IVFPQ_EUNSUPPORTED, "device ordinal %d outside [0, %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void* p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(IVFPQ_EHIP, "hipGetSymbolAddress gave a null address for the static scratch");
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return IVFPQ_OK;
}

constexpr uint32_t kPadKey = 0xFFFFFFFFu;      // R of a padding lane: sorts after every real distance

// ================================================================================================
// Exact selection of the k smallest of n keyed elements by one workgroup.
// Keys are the bit patterns of non-negative floats (order-preserving as unsigned integers); equal
// keys are ordered by a signed 64-bit tie key, then by position.  MSB-first radix select with 8-bit
// digits finds the k-th smallest key; everything below it and the needed share of the ties is
// collected into LDS records and sorted there (bitonic).
// ================================================================================================
// (the helpers below are force-inlined: left to the inliner, a few lines more in one of them turned it into a
// real call with its arguments on the stack, and the probe-selection kernel took twice as long)
constexpr int SEL_THREADS = 256;
constexpr int SEL_CAP = 1024;      // record capacity = IVFPQ_MAX_K: the selected elements always fit

// what block_kth_key alone needs
struct KthShared {
    uint32_t hist[256];
    uint32_t digit, need, count;
    uint32_t n_rec;
};

// CAP: how many records the selection can return (>= k); kernels whose k is small take a small CAP, so that more of
// their workgroups share a compute unit (they wait on barriers and memory most of the time: the top-k kernel with
// k = 100 took 0.25 ms at six workgroups per compute unit and 0.21 ms at eight)
template <int CAP>
struct SelectSharedT {
    static constexpr int kCap = CAP;
    uint32_t hist[256];
    uint32_t rec_key[CAP];
    uint32_t rec_pos[CAP];
    long long rec_tie[CAP];
    uint32_t digit, need, count;   // broadcast slots of the digit search
    uint32_t n_rec, n_eq;
};
using SelectShared = SelectSharedT<SEL_CAP>;
constexpr int SEL_CAP_SMALL = 256;  // >= 2 * kFewMax: block_select_few parks tie keys in the upper half of the records

// The sum of a value over every aligned group of 8 lanes, left in all 8: neighbours, then pairs inside a quad, then
// the other quad of the group (whose four lanes hold the same value by then, so the mirrored order does not matter).
// Each step adds the same two numbers in both partners: all 8 lanes end with the same bits.
__device__ inline float sum_over_8_lanes(float v) {
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true));     // quad_perm [1,0,3,2]
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true));     // quad_perm [2,3,0,1]
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, true));    // row_half_mirror
    return v;
}

// Sum over this lane and the lanes below it, by data-parallel permutes (no trip through the LDS): a scan inside
// every row of 16 lanes, then the last lane of a row added to the rows above.  (A lane a permute has no source
// for, or whose row is masked out, receives 0.)
template <int CTRL, int ROWS>
__device__ inline uint32_t dpp_or_zero(uint32_t v) { return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROWS, 0xF, true); }
__device__ inline uint32_t wave_inclusive_scan(uint32_t v) {
    v += dpp_or_zero<0x111, 0xF>(v);       // row_shr:1
    v += dpp_or_zero<0x112, 0xF>(v);       // row_shr:2
    v += dpp_or_zero<0x114, 0xF>(v);       // row_shr:4
    v += dpp_or_zero<0x118, 0xF>(v);       // row_shr:8
    v += dpp_or_zero<0x142, 0xA>(v);       // row_bcast:15 into rows 1 and 3
    v += dpp_or_zero<0x143, 0xC>(v);       // row_bcast:31 into rows 2 and 3
    return v;
}

// hist holds digit counts; finds the digit that contains the `need`-th smallest element
// (1-based).  Result in s.digit (the digit), s.need (rank inside that digit), s.count (its count).
// Called by all threads; contains barriers.
template <class Shared>
__device__ __forceinline__ void find_digit(Shared& s, uint32_t need) {
    __syncthreads();
    if (threadIdx.x < kWave) {
        const int t = threadIdx.x;
        uint32_t c0 = s.hist[4 * t], c1 = s.hist[4 * t + 1], c2 = s.hist[4 * t + 2], c3 = s.hist[4 * t + 3];
        uint32_t sum = c0 + c1 + c2 + c3;
        uint32_t incl = wave_inclusive_scan(sum);
        uint32_t excl = incl - sum;
        if (excl < need && need <= incl) {
            uint32_t r = need - excl, dsel = 0, cnt = c0;
            if (r > c0) { r -= c0; dsel = 1; cnt = c1;
                if (r > c1) { r -= c1; dsel = 2; cnt = c2;
                    if (r > c2) { r -= c2; dsel = 3; cnt = c3; } } }
            s.digit = 4 * t + dsel;
            s.need = r;
            s.count = cnt;
        }
    }
    __syncthreads();
}

__device__ inline bool rec_less(uint32_t ka, long long ta, uint32_t pa, uint32_t kb, long long tb, uint32_t pb) {
    if (ka != kb) return ka < kb;
    if (ta != tb) return ta < tb;
    return pa < pb;
}

// sorts records [0, np2) ascending by (key, tie, pos); np2 is a power of two <= the record capacity
template <class S>
__device__ __forceinline__ void sort_records(S& s, int np2) {
    for (int size = 2; size <= np2; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            for (int t = threadIdx.x; t < (np2 >> 1); t += blockDim.x) {
                int lo = ((t / stride) * stride * 2) + (t % stride);
                int hi = lo + stride;
                bool up = ((lo & size) == 0);
                uint32_t ka = s.rec_key[lo], kb = s.rec_key[hi];
                long long ta = s.rec_tie[lo], tb = s.rec_tie[hi];
                uint32_t pa = s.rec_pos[lo], pb = s.rec_pos[hi];
                bool b_lt_a = rec_less(kb, tb, pb, ka, ta, pa);
                if (b_lt_a == up) {
                    s.rec_key[lo] = kb; s.rec_key[hi] = ka;
                    s.rec_tie[lo] = tb; s.rec_tie[hi] = ta;
                    s.rec_pos[lo] = pb; s.rec_pos[hi] = pa;
                }
            }
        }
    }
    __syncthreads();
}

// One histogram increment per active lane, with the increments of a wave folded into a single
// LDS atomic when all its active lanes hit the same bin (the usual case for the leading digit of
// distances of similar magnitude, where per-lane atomics on one address would serialise).
__device__ __forceinline__ void hist_add(uint32_t* hist, uint32_t digit, bool active) {
    const unsigned long long act = ballot64(active);
    if (act == 0) return;
    const int first = __ffsll((long long)act) - 1;
    const uint32_t d0 = (uint32_t)__builtin_amdgcn_readlane((int)digit, first);      // `first` is the same for the whole wave
    const unsigned long long same = ballot64(active && digit == d0);
    if (same == act) {
        if ((int)(threadIdx.x & (kWave - 1)) == first) atomicAdd(&hist[d0], (uint32_t)__popcll(act));
    } else if (active) {
        atomicAdd(&hist[digit], 1u);
    }
}

// The kk-th smallest (1-based, 1 <= kk <= n) of n keys, by four 8-bit digits from the top.
// *rank_in_ties = how many elements equal to the result rank at or below kk (1..*n_ties),
// *n_ties = number of elements equal to the result.  Called by every thread of the workgroup.
template <class Shared, class KeyFn>
__device__ __forceinline__ uint32_t block_kth_key(Shared& s, uint32_t n, uint32_t kk, KeyFn key_of,
                                  uint32_t* rank_in_ties, uint32_t* n_ties) {
    const int tid = threadIdx.x, nth = blockDim.x;
    uint32_t prefix = 0, need = kk, n_eq = 0;
    for (int pass = 3; pass >= 0; --pass) {
        const int shift = pass * 8;
        __syncthreads();
        for (int b = tid; b < 256; b += nth) s.hist[b] = 0;
        __syncthreads();
        for (uint32_t base = 0; base < n; base += nth) {
            const uint32_t i = base + tid;
            const bool valid = i < n;
            const uint32_t key = valid ? key_of(i) : 0u;
            const bool in = valid && ((pass == 3) || ((key >> (shift + 8)) == (prefix >> (shift + 8))));
            hist_add(s.hist, (key >> shift) & 255u, in);
        }
        find_digit(s, need);
        prefix |= s.digit << shift;
        need = s.need;
        n_eq = s.count;
    }
    *rank_in_ties = need;
    *n_ties = n_eq;
    return prefix;
}

// KeyFn(i) -> uint32 key of element i; TieFn(i) -> long long tie key of element i.
// On return records [0, min(k, n)) hold the selected elements in ascending (key, tie, pos) order.
// Returns min(k, n).  Must be called by every thread of the workgroup.
template <class S, class KeyFn, class TieFn>
__device__ __forceinline__ int block_select_smallest(S& s, uint32_t n, uint32_t k, KeyFn key_of, TieFn tie_of) {
    const uint32_t kk = k < n ? k : n;
    if (kk == 0) return 0;
    const int tid = threadIdx.x, nth = blockDim.x;

    uint32_t need = 0, n_eq = 0;
    const uint32_t T = block_kth_key(s, n, kk, key_of, &need, &n_eq);
    const uint32_t n_less = kk - need;     // elements strictly below T: all selected

    // ---- collect
    __syncthreads();
    if (tid == 0) { s.n_rec = 0; s.n_eq = 0; }
    __syncthreads();
    const bool all_fit = (n_less + n_eq) <= (uint32_t)S::kCap;
    if (all_fit) {
        // everything <= T goes into the records; the sort decides which ties stay
        for (uint32_t i = tid; i < n; i += nth) {
            uint32_t key = key_of(i);
            if (key <= T) {
                uint32_t slot = atomicAdd(&s.n_rec, 1u);
                s.rec_key[slot] = key; s.rec_pos[slot] = i; s.rec_tie[slot] = tie_of(i);
            }
        }
    } else {
        // too many elements equal to T: pick the `need` smallest tie keys among them with a second,
        // 64-bit radix select (tie keys mapped to unsigned order by flipping the sign bit)
        unsigned long long uprefix = 0;
        uint32_t uneed = need;
        for (int pass = 7; pass >= 0; --pass) {
            const int shift = pass * 8;
            __syncthreads();
            for (int b = tid; b < 256; b += nth) s.hist[b] = 0;
            __syncthreads();
            for (uint32_t base = 0; base < n; base += nth) {
                const uint32_t i = base + tid;
                bool in = i < n && key_of(i) == T;
                unsigned long long u = 0;
                if (in) {
                    u = (unsigned long long)tie_of(i) ^ 0x8000000000000000ull;
                    in = (pass == 7) || ((u >> (shift + 8)) == (uprefix >> (shift + 8)));
                }
                hist_add(s.hist, (uint32_t)(u >> shift) & 255u, in);
            }
            find_digit(s, uneed);
            uprefix |= (unsigned long long)s.digit << shift;
            uneed = s.need;
        }
        // uprefix = the need-th smallest tie key; uneed = how many copies of it to take
        __syncthreads();
        for (uint32_t i = tid; i < n; i += nth) {
            uint32_t key = key_of(i);
            if (key > T) continue;
            bool take = key < T;
            long long tie = tie_of(i);
            if (!take) {
                unsigned long long u = (unsigned long long)tie ^ 0x8000000000000000ull;
                if (u < uprefix) take = true;
                else if (u == uprefix) take = atomicAdd(&s.n_eq, 1u) < uneed;
            }
            if (take) {
                uint32_t slot = atomicAdd(&s.n_rec, 1u);
                s.rec_key[slot] = key; s.rec_pos[slot] = i; s.rec_tie[slot] = tie;
            }
        }
    }
    __syncthreads();
    const uint32_t n_rec = s.n_rec;
    int np2 = 1;
    while ((uint32_t)np2 < n_rec) np2 <<= 1;
    for (int i = n_rec + tid; i < np2; i += nth) {
        s.rec_key[i] = 0xFFFFFFFFu; s.rec_pos[i] = 0xFFFFFFFFu; s.rec_tie[i] = 0x7FFFFFFFFFFFFFFFll;
    }
    sort_records(s, np2);
    return (int)kk;
}

// The same selection for few elements (n <= kFewMax <= blockDim.x; key_of must be cheap, every thread
// calls it n times): thread i ranks element i by counting the elements that precede it in (key, tie,
// index) order, three barriers in all.  It costs about n instructions per thread where the radix select
// and the sort cost several hundred whatever n is.  Tie keys are fetched only for elements with fewer than
// k smaller keys, and wait in the upper half of the record array while the ranks are settled.
constexpr uint32_t kFewMax = 128;
template <class S, class KeyFn, class TieFn>
__device__ __forceinline__ int block_select_few(S& s, uint32_t n, uint32_t k, KeyFn key_of, TieFn tie_of) {
    static_assert(S::kCap >= 2 * (int)kFewMax, "tie keys wait in the upper half of the records");
    const uint32_t kk = k < n ? k : n;
    if (kk == 0) return 0;
    const uint32_t e = threadIdx.x;
    constexpr uint32_t SCR = S::kCap / 2;
    __syncthreads();
    const uint32_t key = e < n ? key_of(e) : 0xFFFFFFFFu;
    uint32_t less = 0, same = 0;
    if (e < n)
        for (uint32_t j = 0; j < n; ++j) {
            const uint32_t kj = key_of(j);
            less += kj < key ? 1u : 0u;
            same += kj == key ? 1u : 0u;
        }
    const bool cand = e < n && less < kk;
    long long tie = 0;
    if (cand) { tie = tie_of(e); s.rec_tie[SCR + e] = tie; }
    __syncthreads();
    if (cand) {
        uint32_t r = less;
        if (same > 1)                        // elements with the same key all have their tie key in place
            for (uint32_t j = 0; j < n; ++j) {
                if (j == e || key_of(j) != key) continue;
                const long long tj = s.rec_tie[SCR + j];
                r += (tj < tie || (tj == tie && j < e)) ? 1u : 0u;
            }
        if (r < kk) { s.rec_key[r] = key; s.rec_tie[r] = tie; s.rec_pos[r] = e; }
    }
    __syncthreads();
    return (int)kk;
}

// ------------------------------------------------------------------------------------------------
// The k smallest of a long row of keys in global memory (tens of thousands per query).
// The k-th smallest key among the first CAND_CAP elements is an upper bound of the k-th smallest
// of the whole row, so one streaming pass that keeps only keys not above that bound compacts the
// row into LDS (typically a few times k elements); the exact selection then runs on that small
// set.  If the compacted set overflows LDS the routine falls back to exact selection over the
// whole row in global memory.  tie_of_pos(pos, key) gives the tie key of the element at row
// position pos.  On return records [0, got) hold key, tie and row position in ascending
// (key, tie) order.
// ------------------------------------------------------------------------------------------------
constexpr int CAND_CAP = 1024;   // >= IVFPQ_MAX_K

template <int CAP>
struct RowSelectSharedT {
    SelectSharedT<CAP> sel;
    uint32_t cand_key[CAND_CAP];
    uint32_t cand_pos[CAND_CAP];
    uint32_t n_cand;
};
using RowSelectShared = RowSelectSharedT<SEL_CAP>;

// pos_of(i): logical position of row element i (what the records report and what tie_of_pos
// takes); have_bound/bound: an upper bound of the k-th smallest key that the caller already knows
// (at least k elements of the row are <= it).
// Hooks for rows whose keys are only approximate (probe selection): widen(bound) is applied to every
// bound before it filters (it must return a key that no element the exact selection could need
// exceeds); refine(n_cand) runs once the candidates sit in LDS, may replace their keys by exact ones and
// drop candidates (it returns how many remain, at the front of the candidate arrays); whole_row() is the
// fallback when compaction fails and must return the selection itself.
struct NoWiden { __device__ uint32_t operator()(uint32_t b) const { return b; } };
struct NoRefine { __device__ uint32_t operator()(uint32_t n) const { return n; } };

template <class T, class PosFn, class TieFn, class WidenFn, class RefineFn, class WholeRowFn>
__device__ __forceinline__ int block_select_row_ex(T& t, const uint32_t* __restrict__ row, uint32_t n, uint32_t k,
                                   bool have_bound, uint32_t bound, PosFn pos_of, TieFn tie_of_pos,
                                   WidenFn widen, RefineFn refine, WholeRowFn whole_row) {
    auto& s = t.sel;
    const int tid = threadIdx.x, nth = blockDim.x;
    const uint32_t kk = k < (uint32_t)CAND_CAP ? k : (uint32_t)CAND_CAP;
    bool compact = true;
    uint32_t n_cand = n;
    __syncthreads();
    if (n > (uint32_t)CAND_CAP) {
        uint32_t r0, r1;
        if (!have_bound) {
            // the k-th smallest of the first S keys bounds the k-th smallest of the row; about k n / S keys
            // pass it, so S grows with k n until half the LDS buffer is the expectation (a second pass
            // over the whole row costs more than a longer sample)
            const unsigned long long want = (unsigned long long)kk * n / (CAND_CAP / 2);
            const uint32_t S = want <= (unsigned long long)CAND_CAP ? (uint32_t)CAND_CAP : (want < n ? (uint32_t)want : n);
            if (S == (uint32_t)CAND_CAP) {
                for (int i = tid; i < CAND_CAP; i += nth) t.cand_key[i] = row[i];
                bound = block_kth_key(s, (uint32_t)CAND_CAP, kk, [&](uint32_t i) { return t.cand_key[i]; }, &r0, &r1);
            } else {
                bound = block_kth_key(s, S, kk, [&](uint32_t i) { return row[i]; }, &r0, &r1);
            }
        }
        bound = widen(bound);
        const bool vec = (reinterpret_cast<uintptr_t>(row) & 15u) == 0;      // 16-byte loads, the last n % 4 keys one by one
        compact = false;
        // Each pass keeps the elements not above the bound.  If they overflow the LDS buffer, the
        // k-th smallest of the ones that were kept is a tighter valid bound (they are all members
        // of the row): the survivor count shrinks by about CAND_CAP / k per pass.
        for (int pass = 0; pass < 8; ++pass) {
            __syncthreads();
            if (tid == 0) t.n_cand = 0;
            __syncthreads();
            auto keep = [&](uint32_t key, uint32_t i) {
                if (key <= bound) {
                    uint32_t slot = atomicAdd(&t.n_cand, 1u);
                    if (slot < (uint32_t)CAND_CAP) { t.cand_key[slot] = key; t.cand_pos[slot] = pos_of(i); }
                }
            };
            if (vec) {
                const uint4* row4 = reinterpret_cast<const uint4*>(row);
                for (uint32_t i4 = tid; i4 < n / 4; i4 += nth) {
                    const uint4 v = row4[i4];
                    keep(v.x, i4 * 4); keep(v.y, i4 * 4 + 1); keep(v.z, i4 * 4 + 2); keep(v.w, i4 * 4 + 3);
                }
                for (uint32_t i = (n & ~3u) + tid; i < n; i += nth) keep(row[i], i);
            } else {
                for (uint32_t i = tid; i < n; i += nth) keep(row[i], i);
            }
            __syncthreads();
            n_cand = t.n_cand;
            if (n_cand <= (uint32_t)CAND_CAP) { compact = true; break; }
            const uint32_t tighter = widen(block_kth_key(s, (uint32_t)CAND_CAP, kk, [&](uint32_t i) { return t.cand_key[i]; }, &r0, &r1));
            if (tighter >= bound) break;      // a plateau of equal keys: no progress possible this way
            bound = tighter;
        }
    } else {
        for (uint32_t i = tid; i < n; i += nth) { t.cand_key[i] = row[i]; t.cand_pos[i] = pos_of(i); }
        __syncthreads();
    }
    int got;
    if (compact) {
        n_cand = refine(n_cand);
        auto key_of = [&](uint32_t i) { return t.cand_key[i]; };
        auto tie_of = [&](uint32_t i) -> long long { return tie_of_pos(t.cand_pos[i], t.cand_key[i]); };
        got = n_cand <= kFewMax ? block_select_few(s, n_cand, k, key_of, tie_of)
                                : block_select_smallest(s, n_cand, k, key_of, tie_of);
        for (int j = tid; j < got; j += nth) s.rec_pos[j] = t.cand_pos[s.rec_pos[j]];   // back to logical positions
    } else {
        got = whole_row();
    }
    __syncthreads();
    return got;
}

template <class T, class PosFn, class TieFn>
__device__ __forceinline__ int block_select_row(T& t, const uint32_t* __restrict__ row, uint32_t n, uint32_t k,
                                bool have_bound, uint32_t bound, PosFn pos_of, TieFn tie_of_pos) {
    auto& s = t.sel;
    return block_select_row_ex(t, row, n, k, have_bound, bound, pos_of, tie_of_pos, NoWiden{}, NoRefine{},
        [&]() -> int {
            const int got = block_select_smallest(s, n, k,
                [&](uint32_t i) { return row[i]; },
                [&](uint32_t i) -> long long { return tie_of_pos(pos_of(i), row[i]); });
            for (int j = threadIdx.x; j < got; j += blockDim.x) s.rec_pos[j] = pos_of(s.rec_pos[j]);
            return got;
        });
}

// ================================================================================================
// Step 1b: probe selection for one query per workgroup: short-list by the ranking values of step
// 1a (with their error bound), exact distances for the short list, exact selection among those.
// Also lays out the query's slice of the R scratch: roff[p] = first slot of probe p, roff[n_probes]
// = padded candidate count (every cluster padded to a multiple of 64 vectors), and writes one
// descriptor per (query, probe) pair -- {cluster, length, first 64-vector group, R offset} -- so
// that a scan workgroup starts from a single 16-byte load.
// S (may be null): instead of the keys, the ranking kernel's summary of every strip of strip_w clusters
// (its three smallest keys, tagged with the cluster's position in the strip), strip-major
// [n_strips][gridDim.x]; the host passes it when there are at least 2 n_probes strips.  The n_probes-th
// smallest strip minimum then bounds the n_probes-th smallest key; a strip whose minimum passes the
// (widened) bound yields its best cluster, its best two if the second key passes too, or all its clusters if
// the third does as well, and all of
// these get their exact distance.  A is then only scratch for the whole-row fallback.
// ================================================================================================
// CAP: record capacity, >= n_probes.  The small one serves selections from strip summaries only (S given): the path
// that streams all keys short-lists up to CAND_CAP indices in the record arrays.
template <int CAP>
__global__ void __launch_bounds__(SEL_THREADS)
select_probes_kernel(uint32_t* __restrict__ A, const StripSummary* __restrict__ S, int strip_w,
                     const float* __restrict__ queries,
                     const float* __restrict__ centroids, float centroid_norm_max, int d,
                     int n_lists, int n_probes,
                     const uint32_t* __restrict__ list_sizes, const int64_t* __restrict__ group_offsets,
                     uint32_t* __restrict__ probes, float* __restrict__ probe_dists,
                     uint32_t* __restrict__ roff, uint4* __restrict__ pairs, int k_hint) {
    __shared__ RowSelectSharedT<CAP> t;
    __shared__ float s_part[SEL_THREADS / kWave];
    auto& s = t.sel;
    // Workgroup b runs on XCD b % 8.  Inside every block of 64 queries the eight workgroups of one XCD take eight
    // consecutive queries: their strip summaries (16 bytes per query and strip, strip-major) share 128-byte lines,
    // so a line is fetched into one XCD's L2 instead of all eight.
    const int b = blockIdx.x;
    const int q = b < (int)(gridDim.x & ~63u) ? (b & ~63) + ((b & 7) << 3) + ((b >> 3) & 7) : b;
    const int tid = threadIdx.x, nth = blockDim.x;
    const int lane = tid & (kWave - 1), wave = tid >> 6, n_waves = nth >> 6;
    const float* qv = queries + (size_t)q * d;
    uint32_t* row = A + (size_t)q * n_lists;       // ranking keys of a(q, c) = |c|^2 - 2 q.c

    auto wave_sum = [&](float v) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
        return v;
    };
    // |q|^2, for the error bound of a()
    float part = 0.f;
    for (int c = tid; c < d; c += nth) part = __builtin_fmaf(qv[c], qv[c], part);
    part = wave_sum(part);
    if (lane == 0) s_part[wave] = part;
    __syncthreads();
    float qn = 0.f;
    for (int w = 0; w < n_waves; ++w) qn += s_part[w];
    // |a_computed - a_exact| <= delta
    const float delta = rank_error_bound(d, qn, centroid_norm_max);
    // keys up to this one can belong to a cluster whose exact rank is within the bound's rank
    auto widen = [&](uint32_t key) {
        const float f = ordered_key_value(key);
        float g = f + 2.f * delta;
        g += __builtin_fabsf(g) * 2.3841858e-07f;          // the addition above rounds: stay on the safe side
        return (g == g) ? ordered_key(g) : 0xFFFFFFFFu;     // NaN (from infinite inputs): admit everything
    };
    // exact squared distance to cluster l (direct form) by a group of 8 adjacent lanes: each lane sums
    // every 8th component, then three exchange steps; the order is fixed, so the value of a cluster
    // does not depend on which path computes it.  Every lane of the group gets the result.
    auto exact8 = [&](uint32_t l, bool valid) {
        float acc = 0.f;
        if (valid) {
            const float* c = centroids + (size_t)l * d;
            for (int u = tid & 7; u < d; u += 8) { const float diff = qv[u] - c[u]; acc = __builtin_fmaf(diff, diff, acc); }
        }
        acc = sum_over_8_lanes(acc);
        return acc;
    };
    // candidates in LDS: keep those whose a() is within 2 delta of the n_probes-th smallest a() among
    // them (every cluster of the exact answer is among these), give them their exact distance
    auto refine = [&](uint32_t n_cand) -> uint32_t {
        const uint32_t kk = (uint32_t)n_probes < n_cand ? (uint32_t)n_probes : n_cand;
        if (kk == 0) return n_cand;
        uint32_t r0, r1;
        const uint32_t limit = widen(block_kth_key(s, n_cand, kk, [&](uint32_t i) { return t.cand_key[i]; }, &r0, &r1));
        __syncthreads();
        if (tid == 0) s.n_rec = 0;
        __syncthreads();
        // the short list, as indices into the candidate arrays (the record array is free at this point)
        for (uint32_t i = tid; i < n_cand; i += nth) {
            if (t.cand_key[i] <= limit) s.rec_pos[atomicAdd(&s.n_rec, 1u)] = i;
            else t.cand_key[i] = 0xFFFFFFFFu;
        }
        __syncthreads();
        const uint32_t n_short = s.n_rec;
        for (uint32_t base = 0; base < n_short; base += nth / 8) {
            const uint32_t j = base + (tid >> 3);
            const bool valid = j < n_short;
            const uint32_t i = valid ? s.rec_pos[j] : 0u;
            const float dist = exact8(valid ? t.cand_pos[i] : 0u, valid);
            if (valid && (tid & 7) == 0) t.cand_key[i] = __float_as_uint(dist);
        }
        __syncthreads();
        if (n_short > kFewMax) return n_cand;        // the others keep the all-ones key and are never selected
        // few enough for the counting selection: move the short list to the front
        const uint32_t i = (uint32_t)tid < n_short ? s.rec_pos[tid] : 0u;
        const uint32_t mk = t.cand_key[i], mp = t.cand_pos[i];
        __syncthreads();
        if ((uint32_t)tid < n_short) { t.cand_key[tid] = mk; t.cand_pos[tid] = mp; }
        __syncthreads();
        return n_short;
    };
    // compaction failed (a plateau of equal ranking values): exact distances of all clusters
    auto whole_row = [&]() -> int {
        __syncthreads();
        for (uint32_t base = 0; base < (uint32_t)n_lists; base += nth / 8) {
            const uint32_t l = base + (tid >> 3);
            const bool valid = l < (uint32_t)n_lists;
            const float dist = exact8(valid ? l : 0u, valid);
            if (valid && (tid & 7) == 0) row[l] = __float_as_uint(dist);
        }
        __threadfence_block();
        __syncthreads();
        return block_select_smallest(s, (uint32_t)n_lists, (uint32_t)n_probes,
            [&](uint32_t i) { return row[i]; }, [&](uint32_t i) { return (long long)i; });
    };
    int got;
    if (S) {
        const uint32_t n_strips = ((uint32_t)n_lists + strip_w - 1) / strip_w, sw = (uint32_t)strip_w;
        const size_t stride = gridDim.x;
        const StripSummary* mine = S + q;
        // the strip minima are read several times: from the (still unused) candidate-key array if they fit; the
        // second and third keys are needed only for the few strips whose minimum passes the bound
        const bool in_lds = n_strips <= (uint32_t)CAND_CAP;
        if (in_lds)
            for (uint32_t i = tid; i < n_strips; i += nth) t.cand_key[i] = mine[i * stride].x;
        __syncthreads();
        auto low1 = [&](uint32_t i) { return in_lds ? t.cand_key[i] : mine[i * stride].x; };
        auto low2 = [&](uint32_t i) { return mine[i * stride].y; };
        auto low3 = [&](uint32_t i) { return mine[i * stride].z; };
        uint32_t r0, r1;
        const uint32_t kk = (uint32_t)n_probes < n_strips ? (uint32_t)n_probes : n_strips;
        // kk strips hold a key not above this, so it bounds the kk-th smallest key of the row
        const uint32_t bound = widen(block_kth_key(s, n_strips, kk, [&](uint32_t i) { return low1(i) | 63u; }, &r0, &r1));
        __syncthreads();
        if (tid == 0) t.n_cand = 0;
        __syncthreads();
        for (uint32_t i = tid; i < n_strips; i += nth) {
            const uint32_t a1 = low1(i), first = i * sw;
            if ((a1 & ~63u) > bound) continue;
            const uint32_t a2 = low2(i);
            if ((a2 & ~63u) > bound || (low3(i) & ~63u) > bound) {
                // only its best cluster can pass, or its best two
                const uint32_t n_take = (a2 & ~63u) > bound ? 1u : 2u;
                for (uint32_t u = 0; u < n_take; ++u) {
                    const uint32_t c = first + ((u == 0 ? a1 : a2) & 63u);
                    if (c < (uint32_t)n_lists) {
                        const uint32_t slot = atomicAdd(&t.n_cand, 1u);
                        if (slot < (uint32_t)CAND_CAP) t.cand_pos[slot] = c;
                    }
                }
            } else {                                   // more may: all its clusters
                const uint32_t cnt = (uint32_t)n_lists - first < sw ? (uint32_t)n_lists - first : sw;
                const uint32_t slot = atomicAdd(&t.n_cand, cnt);
                for (uint32_t c = 0; c < cnt; ++c)
                    if (slot + c < (uint32_t)CAND_CAP) t.cand_pos[slot + c] = first + c;
            }
        }
        __syncthreads();
        const uint32_t n_cand = t.n_cand;
        if (n_cand >= (uint32_t)n_probes && n_cand <= (uint32_t)CAND_CAP) {
            for (uint32_t base = 0; base < n_cand; base += nth / 8) {
                const uint32_t j = base + (tid >> 3);
                const bool valid = j < n_cand;
                const float dist = exact8(valid ? t.cand_pos[j] : 0u, valid);
                if (valid && (tid & 7) == 0) t.cand_key[j] = __float_as_uint(dist);
            }
            __syncthreads();
            auto key_of = [&](uint32_t i) { return t.cand_key[i]; };
            auto tie_of = [&](uint32_t i) { return (long long)t.cand_pos[i]; };
            got = n_cand <= kFewMax ? block_select_few(s, n_cand, (uint32_t)n_probes, key_of, tie_of)
                                    : block_select_smallest(s, n_cand, (uint32_t)n_probes, key_of, tie_of);
            for (int j = tid; j < got; j += nth) s.rec_pos[j] = t.cand_pos[s.rec_pos[j]];
        } else {
            got = whole_row();       // a plateau of equal ranking values (or not-a-number keys)
        }
        __syncthreads();
    } else if constexpr (CAP == SEL_CAP) {
        got = block_select_row_ex(t, row, (uint32_t)n_lists, (uint32_t)n_probes, false, 0u,
                                  [](uint32_t i) { return i; },
                                  [](uint32_t pos, uint32_t) { return (long long)pos; },
                                  widen, refine, whole_row);
    } else {
        return;              // not launched: the host gives the small capacity strip summaries
    }
    if (!roff) {             // the caller's probe lists: nearest first
        for (int p = tid; p < got; p += nth) {
            probes[(size_t)q * n_probes + p] = s.rec_pos[p];
            if (probe_dists) probe_dists[(size_t)q * n_probes + p] = __uint_as_float(s.rec_key[p]);
        }
        return;
    }
    // The search's own lists.  Slot 0 is the cluster that is scanned unfiltered and whose k-th smallest R
    // bounds the rest: the nearest one that holds at least k_hint vectors (a smaller one gives no bound, and
    // then every vector of every other probe would be kept); the others follow in order of distance.
    // (lengths and first groups of all probes are fetched in parallel; got <= 1024 = the candidate buffer)
    for (int p = tid; p < got; p += nth) {
        const uint32_t l = s.rec_pos[p];
        t.cand_key[p] = list_sizes[l];
        t.cand_pos[p] = (uint32_t)group_offsets[l];
    }
    uint32_t* slot_of = reinterpret_cast<uint32_t*>(s.rec_tie);          // 2 CAP words: slot of probe p, then offsets
    uint32_t* offs = slot_of + CAP;
    __syncthreads();
    if (tid == 0) {
        int pivot = 0;
        if (k_hint > 0)
            for (int p = 0; p < got; ++p)
                if (t.cand_key[p] >= (uint32_t)k_hint) { pivot = p; break; }
        uint32_t at = 0;
        for (int i = 0; i < got; ++i) {
            const int p = i == 0 ? pivot : (i <= pivot ? i - 1 : i);
            slot_of[p] = (uint32_t)i;
            offs[p] = at;
            at += (t.cand_key[p] + 63u) & ~63u;
        }
        roff[(size_t)q * (n_probes + 1) + got] = at;
    }
    __syncthreads();
    for (int p = tid; p < got; p += nth) {
        const uint32_t i = slot_of[p], l = s.rec_pos[p], at = offs[p];
        probes[(size_t)q * n_probes + i] = l;
        if (probe_dists) probe_dists[(size_t)q * n_probes + i] = __uint_as_float(s.rec_key[p]);
        roff[(size_t)q * (n_probes + 1) + i] = at;
        pairs[(size_t)q * n_probes + i] = make_uint4(l, t.cand_key[p], t.cand_pos[p], at);
    }
}

// One workgroup per query; the small record capacity (more workgroups per compute unit) when the selection works
// from strip summaries and n_probes allows.
template <class... Args>
void launch_select_probes(int nq, hipStream_t st, uint32_t* A, const StripSummary* S, int strip_w, const float* queries,
                          const float* centroids, float centroid_norm_max, int d, int n_lists, int n_probes, Args... rest) {
    if (S && n_probes <= SEL_CAP_SMALL)
        hipLaunchKernelGGL(select_probes_kernel<SEL_CAP_SMALL>, dim3(nq), dim3(SEL_THREADS), 0, st, A, S, strip_w, queries, centroids,
                           centroid_norm_max, d, n_lists, n_probes, rest...);
    else
        hipLaunchKernelGGL(select_probes_kernel<SEL_CAP>, dim3(nq), dim3(SEL_THREADS), 0, st, A, S, strip_w, queries, centroids,
                           centroid_norm_max, d, n_lists, n_probes, rest...);
}

// Same layout step for caller-given probes.
__global__ void __launch_bounds__(256)
layout_probes_kernel(const uint32_t* __restrict__ probes_in, int nq, int n_probes, int n_lists,
                     const uint32_t* __restrict__ list_sizes, const int64_t* __restrict__ group_offsets,
                     uint32_t* __restrict__ probes, uint32_t* __restrict__ roff, uint4* __restrict__ pairs) {
    int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= nq) return;
    uint32_t at = 0;
    for (int p = 0; p < n_probes; ++p) {
        uint32_t l = probes_in[(size_t)q * n_probes + p];
        const bool ok = l < (uint32_t)n_lists;                 // an out-of-range entry is skipped
        const uint32_t len = ok ? list_sizes[l] : 0u;
        probes[(size_t)q * n_probes + p] = l;
        roff[(size_t)q * (n_probes + 1) + p] = at;
        pairs[(size_t)q * n_probes + p] = make_uint4(l, len, ok ? (uint32_t)group_offsets[l] : 0u, at);
        at += (len + 63u) & ~63u;
    }
    roff[(size_t)q * (n_probes + 1) + n_probes] = at;
}

// ================================================================================================
// Steps 2-4: residual, lookup table in LDS, code scan.
// ================================================================================================
template <int LUT> struct LutTraits;     // bytes: size of one table entry
template <> struct LutTraits<IVFPQ_LUT_FP32> { static constexpr int bytes = 4; };
template <> struct LutTraits<IVFPQ_LUT_FP16> { static constexpr int bytes = 2; };
template <> struct LutTraits<IVFPQ_LUT_FP8_E5M3> { static constexpr int bytes = 1; };
template <> struct LutTraits<IVFPQ_LUT_FP8_E4M4> { static constexpr int bytes = 1; };
// The two 8-bit formats.  shift: how far a code is shifted to line up with the FP32 exponent/mantissa
// field (23 less the mantissa bits); top_exp: the largest exponent field; bias_min/bias_max: range of
// the exponent bias for which every code is a finite normal FP32 number.
template <int LUT> struct Fp8Format {     // e5m3
    static constexpr int shift = 20, top_exp = 31, bias_min = -96, bias_max = 110;
};
template <> struct Fp8Format<IVFPQ_LUT_FP8_E4M4> {
    static constexpr int shift = 19, top_exp = 15, bias_min = -100, bias_max = 110;
};
template <int LUT> constexpr bool kIsFp8 = LUT == IVFPQ_LUT_FP8_E5M3 || LUT == IVFPQ_LUT_FP8_E4M4;

// Constants of a sign-less 8-bit float (Sec. II) with M mantissa bits (shift = 23 - M) and exponent
// bias B: value(b) = (1 + mant/2^M) * 2^(exp - B).  Both conversions are a shift plus a bias
// adjustment on the FP32 bit pattern:
//   code = (clamp_s32(bits, lo, hi) - sub) >> shift        bits = (code << shift) + lo
// lo = (127 - B) << 23 is the smallest value, hi = lo + (255 << shift) the largest; sub = lo less half
// an 8-bit ulp, so that the shift rounds to nearest with ties up, or lo itself to truncate.  The clamp
// acts on the pattern as a signed integer: zero and negatives give code 0, +Inf code 255.
// e5m3 with B = 15: lo = 0x38000000, hi = 0x47F00000, sub = 0x37F80000.
struct Fp8Params { int lo, hi, sub; };

__host__ __device__ inline Fp8Params fp8_params(int shift, int bias, int truncate) {
    Fp8Params p;
    p.lo = (127 - bias) << 23;
    p.hi = p.lo + (255 << shift);
    p.sub = truncate ? p.lo : p.lo - (1 << (shift - 1));
    return p;
}
// The code of x, left in the TOP byte of the result (low bits undefined): the clamp is one
// three-operand median once the upper limit sits in a vector register (`hi_v`; an instruction takes
// one scalar operand only), the bias subtraction and the shift are one add-shift.
template <int SHIFT>
__device__ inline uint32_t fp8_code_top_byte(float x, const Fp8Params p, int hi_v) {
    int b;
    uint32_t t;
    const int nsub = -p.sub;
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(b) : "v"(__float_as_int(x)), "s"(p.lo), "v"(hi_v));     // clamp to [lo, hi]
    asm("v_add_lshl_u32 %0, %1, %2, %3" : "=v"(t) : "v"(b), "s"(nsub), "n"(24 - SHIFT));            // (b - sub) << (24 - SHIFT)
    return t;
}
// four codes (of f[0..3], lowest byte first) gathered from the top bytes with three byte permutes
template <int SHIFT>
__device__ inline uint32_t fp8_pack4(const float f[4], const Fp8Params p, int hi_v) {
    const uint32_t t0 = fp8_code_top_byte<SHIFT>(f[0], p, hi_v), t1 = fp8_code_top_byte<SHIFT>(f[1], p, hi_v);
    const uint32_t t2 = fp8_code_top_byte<SHIFT>(f[2], p, hi_v), t3 = fp8_code_top_byte<SHIFT>(f[3], p, hi_v);
    // selector bytes: 0-3 pick a byte of the second operand, 4-7 of the first, 0x0c gives zero
    const uint32_t p01 = __builtin_amdgcn_perm(t1, t0, 0x0c0c0703u);
    const uint32_t p23 = __builtin_amdgcn_perm(t3, t2, 0x07030c0cu);
    return p01 | p23;
}
template <int SHIFT>
__device__ inline float fp8_to_f32(uint32_t b, const Fp8Params p) { return __uint_as_float((b << SHIFT) + (uint32_t)p.lo); }

// IEEE half, round to nearest even, saturating at the largest finite half.
__device__ inline uint32_t half_bits_from_f32(float x) {
    float c = x > 65504.0f ? 65504.0f : x;
    return (uint32_t)__half_as_ushort(__float2half_rn(c));
}

// One table entry: sum over the sub-vector, left to right, of (cb - rq)^2 with one rounding per
// step (subtract, then fused multiply-add into the running sum).
template <int M>
__device__ inline float lut_entry(const float* cbv, const float* rq) {
    float acc = 0.f;
#pragma unroll
    for (int t = 0; t < M; ++t) {
        float diff = cbv[t] - rq[t];
        acc = __builtin_fmaf(diff, diff, acc);
    }
    return acc;
}

template <int LUT>
__device__ inline void store4(unsigned char* lut, int e, const float f[4], const Fp8Params fp8, int hi_v) {
    if constexpr (LUT == IVFPQ_LUT_FP32) {
        *reinterpret_cast<float4*>(lut + (size_t)e * 4) = make_float4(f[0], f[1], f[2], f[3]);
    } else if constexpr (LUT == IVFPQ_LUT_FP16) {
        uint2 v;
        v.x = half_bits_from_f32(f[0]) | (half_bits_from_f32(f[1]) << 16);
        v.y = half_bits_from_f32(f[2]) | (half_bits_from_f32(f[3]) << 16);
        *reinterpret_cast<uint2*>(lut + (size_t)e * 2) = v;
    } else {
        constexpr int SH = Fp8Format<LUT>::shift;
        *reinterpret_cast<uint32_t*>(lut + e) = fp8_pack4<SH>(f, fp8, hi_v);
    }
}

// Visits every entry of F[pq_dim][ksub], 4 consecutive entries of one sub-space per call of
// sink(first entry index, values) (ksub is 16 or 256, so 4 consecutive entries never straddle
// sub-spaces).  codebooks: global [pq_dim][ksub][M]; rq: LDS [pq_dim*M].
template <int M, class Sink>
__device__ __forceinline__ void visit_lut(const float* __restrict__ codebooks, const float* rq, int e_begin, int n_entries,
                                 int bits, int m_runtime, Sink sink) {
    for (int e = e_begin + threadIdx.x * 4; e < n_entries; e += blockDim.x * 4) {
        const int j = e >> bits;
        float f[4];
        if constexpr (M > 0) {
            float r[M];
#pragma unroll
            for (int t = 0; t < M; ++t) r[t] = rq[j * M + t];
            float cbv[4 * M];
            const float4* src = reinterpret_cast<const float4*>(codebooks + (size_t)e * M);
#pragma unroll
            for (int v = 0; v < M; ++v) {
                float4 x = src[v];
                cbv[4 * v] = x.x; cbv[4 * v + 1] = x.y; cbv[4 * v + 2] = x.z; cbv[4 * v + 3] = x.w;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) f[u] = lut_entry<M>(cbv + u * M, r);
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float* cbv = codebooks + (size_t)(e + u) * m_runtime;
                float acc = 0.f;
                for (int t = 0; t < m_runtime; ++t) {
                    float diff = cbv[t] - rq[j * m_runtime + t];
                    acc = __builtin_fmaf(diff, diff, acc);
                }
                f[u] = acc;
            }
        }
        sink(e, f);
    }
}

// 8-bit codes: a table row has 256 entries = 4 per lane of a wave, so every wave visits whole rows
// (row index wave-uniform: residual components are read once per row, addresses advance by a
// constant stride).
template <int M, class Sink>
__device__ __forceinline__ void visit_lut_rows256(const float* __restrict__ codebooks, const float* rq, int row0, int pq_dim, Sink sink) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_waves = blockDim.x >> 6;
    const size_t src_step = (size_t)n_waves * 256 * M;
    const int e_step = n_waves * 256;
    auto load_row = [&](const float* src, float (&cbv)[4 * M]) {
#pragma unroll
        for (int v = 0; v < M; ++v) {
            float4 x = reinterpret_cast<const float4*>(src)[v];
            cbv[4 * v] = x.x; cbv[4 * v + 1] = x.y; cbv[4 * v + 2] = x.z; cbv[4 * v + 3] = x.w;
        }
    };
    auto finish_row = [&](const float (&cbv)[4 * M], int j, int e) {
        float r[M];
#pragma unroll
        for (int t = 0; t < M; ++t) r[t] = rq[j * M + t];
        float f[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) f[u] = lut_entry<M>(cbv + u * M, r);
        sink(e, f);
    };
    const float* src = codebooks + ((size_t)(row0 + wave) * 256 + lane * 4) * M;
    int e = (row0 + wave) * 256 + lane * 4;
    int j = row0 + wave;
    // two rows per trip (written out: both rows' loads are in flight before either is used; deeper
    // prefetching costs registers, hence occupancy, and measured slower)
    for (; j + n_waves < pq_dim; j += 2 * n_waves) {
        float c0[4 * M], c1[4 * M];
        load_row(src, c0);
        load_row(src + src_step, c1);
        finish_row(c0, j, e);
        finish_row(c1, j + n_waves, e + e_step);
        src += 2 * src_step;
        e += 2 * e_step;
    }
    if (j < pq_dim) {
        float c0[4 * M];
        load_row(src, c0);
        finish_row(c0, j, e);
    }
}

// rows (sub-spaces) row0 .. row1 - 1 of the table
template <int BITS, class Sink>
__device__ __forceinline__ void visit_lut_any_m(const float* __restrict__ codebooks, const float* rq, int row0, int row1, int m, Sink sink) {
    const int e_begin = row0 << BITS, e_end = row1 << BITS;
    if constexpr (BITS == 8) {
        switch (m) {
            case 1: visit_lut_rows256<1>(codebooks, rq, row0, row1, sink); return;
            case 2: visit_lut_rows256<2>(codebooks, rq, row0, row1, sink); return;
            case 4: visit_lut_rows256<4>(codebooks, rq, row0, row1, sink); return;
            default: break;
        }
    }
    switch (m) {
        case 1: visit_lut<1>(codebooks, rq, e_begin, e_end, BITS, m, sink); break;
        case 2: visit_lut<2>(codebooks, rq, e_begin, e_end, BITS, m, sink); break;
        case 4: visit_lut<4>(codebooks, rq, e_begin, e_end, BITS, m, sink); break;
        default: visit_lut<0>(codebooks, rq, e_begin, e_end, BITS, m, sink); break;
    }
}

// Encoding of an 8-bit table as the caller configured it: fixed constants, or a bias chosen per table.
struct Fp8Mode {
    Fp8Params fixed;     // constants for the configured bias and rounding
    int truncate;        // rounding of the encode: 0 nearest (ties up), 1 truncate
    int per_table;       // 1: the bias follows the largest entry of each table
};

// Step 3: builds F[pq_dim][ksub] in LDS in the table's dtype; rq must be complete (barrier passed).
// Ends with a barrier.  Returns the constants the 8-bit lookups decode with (workgroup-uniform).
// Per-table bias (a power-of-two scale of the table, expressed as a shift of the format's exponent
// bias): a first pass over the entries finds the largest one; with e its FP32 exponent, the bias is
// top_exp - e, so that the entry's binade becomes the format's top binade; a second pass encodes.
// row0, row1: only these rows (sub-spaces) are built (the whole table for a per-table bias, which needs its
// largest entry).
template <int LUT, int BITS>
__device__ __forceinline__ Fp8Params stage_table(const float* __restrict__ codebooks, const float* rq, int pq_dim, int m,
                                        unsigned char* lut, uint32_t* max_slot, const Fp8Mode mode, int row0, int row1) {
    Fp8Params fp8 = mode.fixed;
    if constexpr (kIsFp8<LUT>) {
        if (mode.per_table) {
            if (threadIdx.x == 0) *max_slot = 0u;
            __syncthreads();
            float mx = 0.f;                       // entries are sums of squares: never negative
            row0 = 0; row1 = pq_dim;
            visit_lut_any_m<BITS>(codebooks, rq, 0, pq_dim, m, [&](int, const float (&f)[4]) {
                mx = fmaxf(fmaxf(mx, f[0]), fmaxf(f[1], fmaxf(f[2], f[3])));
            });
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, kWave));
            if ((threadIdx.x & (kWave - 1)) == 0) atomicMax(max_slot, __float_as_uint(mx));
            __syncthreads();
            const int e = (int)(*max_slot >> 23) - 127;
            int bias = Fp8Format<LUT>::top_exp - e;
            bias = min(max(bias, Fp8Format<LUT>::bias_min), Fp8Format<LUT>::bias_max);
            bias = __builtin_amdgcn_readfirstlane(bias);
            fp8 = fp8_params(Fp8Format<LUT>::shift, bias, mode.truncate);
        }
    }
    int hi_v = fp8.hi;
    asm volatile("" : "+v"(hi_v));       // the upper clamp limit, held in a vector register
    visit_lut_any_m<BITS>(codebooks, rq, row0, row1, m, [&](int e, const float (&f)[4]) { store4<LUT>(lut, e, f, fp8, hi_v); });
    __syncthreads();
    return fp8;
}

template <int LUT>
__device__ inline float lut_get(const unsigned char* lut, uint32_t idx, const Fp8Params fp8) {
    if constexpr (LUT == IVFPQ_LUT_FP32) return reinterpret_cast<const float*>(lut)[idx];
    else if constexpr (LUT == IVFPQ_LUT_FP16) return __half2float(reinterpret_cast<const __half*>(lut)[idx]);
    else return fp8_to_f32<Fp8Format<LUT>::shift>(lut[idx], fp8);
}

// Bit-packed codes: the codes of a vector are one bit string, sub-space j in bits [j*BITS, (j+1)*BITS).
// A "code group" is the shortest run of sub-spaces that ends on a 32-bit boundary: SPG sub-spaces in
// WPG words (8 in 1 for 4-bit codes, 4 in 1 for 8-bit, 32 in 5 / 16 in 3 / 32 in 7 for 5 / 6 / 7 bits).
template <int BITS> struct CodeGroup {
    static constexpr int g = (BITS % 8 == 0) ? 8 : (BITS % 4 == 0) ? 4 : (BITS % 2 == 0) ? 2 : 1;   // gcd(BITS, 32)
    static constexpr int SPG = 32 / g, WPG = BITS / g;
};

// adds the table entries selected by the SPG codes held in w[0 .. WPG) (sub-spaces row0.. ascending)
template <int LUT, int BITS>
__device__ inline float add_group(float acc, const unsigned char* lut, const uint32_t* w, int row0, const Fp8Params fp8) {
    constexpr int SPG = CodeGroup<BITS>::SPG, KSUB = 1 << BITS;
    if constexpr (BITS == 8 && (LUT == IVFPQ_LUT_FP16 || LUT == IVFPQ_LUT_FP32)) {
        // Whole-byte codes and entries of 2 or 4 bytes: the entry's byte offset in its row comes out of one
        // sub-dword shift, the row's offset goes into the LDS read's immediate, and a half entry is converted by
        // the instruction that adds it: 2 vector instructions per lookup.  (The table sits at LDS address 0: the
        // kernel has no static LDS, which the host verifies before the first launch.)
        constexpr int E = LutTraits<LUT>::bytes, LG = ilog2(E);
        const uint32_t off[4] = {byte_shl<0, LG>(w[0]), byte_shl<1, LG>(w[0]), byte_shl<2, LG>(w[0]), byte_shl<3, LG>(w[0])};
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const uint32_t x = LdsWord<E>::load(off[s] + (uint32_t)(row0 + s) * (uint32_t)(KSUB * E));
            if constexpr (LUT == IVFPQ_LUT_FP16) acc = add_half_lo(acc, x);
            else acc += __uint_as_float(x);
        }
        return acc;
    }
#pragma unroll
    for (int s = 0; s < SPG; ++s) {
        constexpr uint32_t mask = (uint32_t)KSUB - 1u;
        const int bit = s * BITS, wi = bit >> 5, sh = bit & 31;
        uint32_t code;
        if (sh + BITS <= 32) code = (w[wi] >> sh) & mask;
        else code = ((w[wi] >> sh) | (w[wi + 1] << (32 - sh))) & mask;     // the field straddles two words
        acc += lut_get<LUT>(lut, (uint32_t)(row0 + s) * (uint32_t)KSUB + code, fp8);
    }
    return acc;
}

constexpr int kAliveCap = 64;    // groups of a wave that the first pass of the split scan can note for the second
constexpr int kStageCap = 128;   // survivors a wave stages in LDS before it appends them (8 bytes each)

struct ScanArgs {
    const float* queries;         // [nq][d] (tile base)
    const float* centroids;
    const float* codebooks;
    const uint32_t* list_sizes;
    const int64_t* group_offsets;
    const uint8_t* codes;
    const uint4* pairs;           // [nq][n_probes] {cluster, length, first group, R offset}; unused in single-list mode
    const uint32_t* bounds;       // [nq] per-query upper bound of the k-th smallest R (filtered mode)
    uint32_t* counts;             // [nq] survivors appended so far (filtered mode)
    uint32_t* Rpos;               // [nq][stride] row position of each appended survivor (filtered mode)
    Fp8Mode fp8;                  // encoding of the 8-bit table dtypes (unused by the other two)
    int mode;                     // 1: nearest probe of every query, every R written in place;
                                  // 2: the other probes, only R <= bound appended behind the nearest probe's segment
    float* R;                     // [nq][stride]
    size_t stride;
    int n_probes;
    int n_lists;
    int d, pq_dim, m, bits;
    int n_chunks;                 // chunks per vector (code_bytes / CW)
    int single_list;              // >= 0: scan this cluster for query 0, R written from offset 0
    const uint32_t* order;        // mode 2: pairs (as q * (n_probes - 1) + probe - 1) grouped by cluster, or null
    uint32_t n_pairs;             // mode 2: number of such pairs
    uint32_t order_block;         // mode 2: consecutive pairs of the grouped order that stay on one XCD
    int early_exit;               // mode 2: stop adding for a 64-vector group once every partial sum is over the bound
};

// Code layout of one cluster (written by ivfpq_upload): vectors in groups of 64 (the last one
// zero-padded); inside a group, chunk c of all 64 vectors is contiguous:
//   byte address = ((group * n_chunks + c) * 64 + lane) * CW
// so one wave-wide load of chunk c reads 64*CW contiguous bytes.
template <int LUT, int BITS, int CW, int NCH>
__global__ void __launch_bounds__(1024)
scan_kernel(ScanArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int ksub = 1 << BITS;
    const int n_entries = a.pq_dim * ksub;
    // LDS: table | residual (d floats) | 16 bytes (largest entry, per-table bias) | survivor staging
    unsigned char* lut = smem;
    float* rq = reinterpret_cast<float*>(smem + (((size_t)n_entries * LutTraits<LUT>::bytes + 15) & ~(size_t)15));
    unsigned char* after_rq = reinterpret_cast<unsigned char*>(rq) + (((size_t)a.d * 4 + 15) & ~(size_t)15);
    uint32_t* max_slot = reinterpret_cast<uint32_t*>(after_rq);
    Fp8Params fp8 = a.fp8.fixed;

    int q, l;
    uint32_t len, first_group, row_pos0 = 0;
    float* Rout;
    if (a.single_list >= 0) {
        q = 0; l = a.single_list; Rout = a.R;
        len = a.list_sizes[l];
        first_group = (uint32_t)a.group_offsets[l];
    } else {
        size_t pair_idx;
        if (a.mode == 1) {
            q = blockIdx.x;
            pair_idx = (size_t)q * a.n_probes;
        } else if (a.order == nullptr) {
            q = blockIdx.x / (a.n_probes - 1);
            pair_idx = (size_t)q * a.n_probes + 1 + (blockIdx.x - q * (a.n_probes - 1));
        } else {
            // Pairs grouped by cluster, and workgroups go round-robin to the 8 XCDs: blocks of
            // `order_block` consecutive pairs of the grouped order are dealt to the XCDs in turn, so that
            // the workgroups scanning one cluster run on one XCD (a few, for a cluster with many pairs)
            // at about the same time and its codes come from that XCD's L2 after the first read.
            const uint32_t xcd = blockIdx.x & 7u, rank = blockIdx.x >> 3;
            const uint32_t slot = ((rank / a.order_block) * 8u + xcd) * a.order_block + rank % a.order_block;
            if (slot >= a.n_pairs) return;
            const uint32_t lin = a.order[slot];
            q = (int)(lin / (uint32_t)(a.n_probes - 1));
            pair_idx = (size_t)q * a.n_probes + 1 + (lin - (uint32_t)q * (uint32_t)(a.n_probes - 1));
        }
        const uint4 pair = a.pairs[pair_idx];
        l = (int)pair.x; len = pair.y; first_group = pair.z;
        Rout = a.R + (size_t)q * a.stride + pair.w;
        row_pos0 = pair.w;
    }
    if (len == 0) return;     // empty cluster (or a caller-given probe that was out of range)
    const bool filtered = a.single_list < 0 && a.mode == 2;
    const bool prune = filtered && a.early_exit != 0;
    uint32_t bound = 0, seg0 = 0;
    if (filtered) {
        bound = a.bounds[q];
        seg0 = a.pairs[(size_t)q * a.n_probes + 1].w;     // padded length of the nearest probe's segment
    }
    // filtered mode: every wave stages its survivors in a private LDS buffer and appends them to the
    // query's row with one global atomic per flush (the counter of a query is shared by all the
    // workgroups of that query: one atomic per 64-vector group would serialise on it)
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));    // the same for the whole wave: loop counters and group addresses stay scalar
    uint2* stage = reinterpret_cast<uint2*>(after_rq + 16) + (size_t)wave * kStageCap;
    uint32_t staged = 0;       // wave-uniform
    const int n_groups = (int)((len + 63u) >> 6);
    const int lane = threadIdx.x & (kWave - 1);
    const int n_waves = blockDim.x >> 6;
    const int nch = NCH > 0 ? NCH : a.n_chunks;
    const uint8_t* codes_l = a.codes + (size_t)first_group * 64 * ((size_t)nch * CW);

    using chunk_t = typename std::conditional<CW == 16, uint4, uint32_t>::type;
    const chunk_t* cbase = reinterpret_cast<const chunk_t*>(codes_l);

    constexpr int NBUF = NCH > 0 ? NCH : 1;
    constexpr int SPG = CodeGroup<BITS>::SPG, WPG = CodeGroup<BITS>::WPG;

    auto load_group = [&](chunk_t (&buf)[NBUF], int g) {
#pragma unroll
        for (int c = 0; c < NBUF; ++c) buf[c] = cbase[((size_t)g * NBUF + c) * 64 + lane];
    };
    // Eq. (1) for the vector this lane holds in buf: sub-spaces in ascending order
    // (blocks_tag: how many blocks of kBlockSub sub-spaces to add, the leading ones; NBLK = all)
    constexpr int NG = CW == 16 ? (4 * NBUF) / WPG : 0;                          // code groups per vector
    constexpr int EVERY = 16 / SPG > 0 ? 16 / SPG : 1;                           // code groups per block of 16 sub-spaces
    constexpr int NBLK = (NG + EVERY - 1) / EVERY;
    auto accumulate = [&](const chunk_t (&buf)[NBUF], auto blocks_tag) -> float {
        constexpr int BLOCKS = decltype(blocks_tag)::value;
        float acc = 0.f;
        if constexpr (CW == 16) {
            uint32_t w[4 * NBUF];
#pragma unroll
            for (int c = 0; c < NBUF; ++c) { w[4 * c] = buf[c].x; w[4 * c + 1] = buf[c].y; w[4 * c + 2] = buf[c].z; w[4 * c + 3] = buf[c].w; }
            static_assert((4 * NBUF) % WPG == 0 || NCH == 0, "16-byte chunks must hold whole code groups");
            // Table entries are never negative, so the partial sums only grow: once those of all 64
            // vectors are over the query's bound none of them can survive, and the rest of their
            // lookups is skipped (checked every 16 sub-spaces; the partial sum then fails the filter).
            bool over = false;                       // wave-uniform
#pragma unroll
            for (int blk = 0; blk < BLOCKS; ++blk) {
                if (over) continue;
#pragma unroll
                for (int e = 0; e < EVERY; ++e) {
                    const int cg = blk * EVERY + e;
                    if (cg < NG) acc = add_group<LUT, BITS>(acc, lut, w + cg * WPG, cg * SPG, fp8);
                }
                if (blk + 1 < BLOCKS && prune) over = ballot64(__float_as_uint(acc) <= bound) == 0;
            }
        }
        return acc;      // 4-byte chunks take the loop over code groups below instead
    };
    auto flush_stage = [&]() {
        if (staged == 0) return;
        uint32_t base = 0;
        if (lane == 0) base = atomicAdd(&a.counts[q], staged);
        base = (uint32_t)__builtin_amdgcn_readfirstlane((int)base);
        uint32_t* dst_key = reinterpret_cast<uint32_t*>(a.R) + (size_t)q * a.stride + seg0 + base;
        uint32_t* dst_pos = a.Rpos + (size_t)q * a.stride + seg0 + base;
        for (uint32_t j = lane; j < staged; j += kWave) {
            const uint2 e = stage[j];
            dst_key[j] = e.x;
            dst_pos[j] = e.y;
        }
        staged = 0;
    };
    auto store_R = [&](int g, float acc) {
        const uint32_t i = (uint32_t)g * 64u + lane;
        if (!filtered) {
            if (i < len) Rout[i] = acc;
            else if (a.single_list < 0) Rout[i] = __uint_as_float(kPadKey);   // padding slot of the R scratch
        } else {
            // keep only what can still be among the k best
            // (the mask is the AND of two compares' results; a ballot of their conjunction goes through a 0/1 value)
            const bool keep = i < len && __float_as_uint(acc) <= bound;
            const unsigned long long m = ballot64(i < len) & ballot64(__float_as_uint(acc) <= bound);
            if (m != 0) {
                if (staged + 64u > (uint32_t)kStageCap) flush_stage();
                if (keep) stage[staged + lanes_below(m)] = make_uint2(__float_as_uint(acc), row_pos0 + i);
                staged += (uint32_t)__popcll(m);
            }
        }
    };

    // issue the loads of this wave's first group before the table is built: HBM latency overlaps it
    chunk_t buf_a[NBUF], buf_b[NBUF];
    int g = wave;
    if constexpr (NCH > 0) {
        if (g < n_groups) load_group(buf_a, g);
    }

    // step 2: residual of the query against this cluster's centroid
    for (int t = threadIdx.x; t < a.d; t += blockDim.x)
        rq[t] = a.queries[(size_t)q * a.d + t] - a.centroids[(size_t)l * a.d + t];
    __syncthreads();
    // Filtered scan with early exit, tables of two or more chunks' worth of rows: most groups are over the
    // bound after the first half of the sub-spaces, so the second half of the table is built only if some
    // group of this pair is still in the race.  Pass 1 builds the leading rows and adds them up for every
    // group, noting the groups with a partial sum under the bound; if there are any, the remaining rows are
    // built and those groups are added up from the start (same order: same R).
    constexpr int HBLK = (NBLK + 1) / 2;                             // blocks of the first pass
    constexpr int HROWS = HBLK * EVERY * SPG;                        // table rows they use
    constexpr int HCH = (HBLK * EVERY * WPG + 3) / 4;                // 16-byte chunks that hold their codes
    // Worth it only if the first pass weeds out most groups and the rows it saves are expensive.  Measured
    // (scan stage, 10,000 queries): 64 sub-spaces of 8-bit codes, first pass 32: 2.13 -> 1.68 ms (e5m3), 3.06 ->
    // 2.74 ms (fp32); 48 sub-spaces, first pass 32: 2.20 -> 2.47 ms (fp32); 32 sub-spaces, first pass 16: 6.5 ->
    // 8.1 ms (most groups went through twice); 4-bit codes (16-entry rows cost nothing to build): 6.8 -> 9.7 ms.
    // Hence: 8-bit codes, four chunks, the first pass takes half of them.
    constexpr bool kCanSplit = BITS == 8 && NCH == 4 && HROWS >= 32 && 2 * HBLK == NBLK;
    bool lazy = false;
    if constexpr (kCanSplit) lazy = prune && !(kIsFp8<LUT> && a.fp8.per_table);
    if constexpr (kCanSplit) {
        if (lazy) {
            uint32_t* any_alive = max_slot + 1;
            uint16_t* alive = reinterpret_cast<uint16_t*>(after_rq + 16 + (size_t)n_waves * kStageCap * 8) + (size_t)wave * kAliveCap;
            if (threadIdx.x == 0) *any_alive = 0u;
            fp8 = stage_table<LUT, BITS>(a.codebooks, rq, a.pq_dim, a.m, lut, max_slot, a.fp8, 0, HROWS);
            uint32_t n_alive = 0;                // wave-uniform
            bool redo_all = false;               // more groups in the race than the list holds: take them all again
            auto load_head = [&](chunk_t (&buf)[NBUF], int grp) {
#pragma unroll
                for (int c = 0; c < HCH; ++c) buf[c] = cbase[((size_t)grp * NBUF + c) * 64 + lane];
            };
            auto first_pass = [&](int grp, const chunk_t (&buf)[NBUF]) {
                const float acc = accumulate(buf, std::integral_constant<int, HBLK>{});
                if ((ballot64((uint32_t)grp * 64u + lane < len) & ballot64(__float_as_uint(acc) <= bound)) != 0) {
                    if (n_alive < (uint32_t)kAliveCap && grp / n_waves < 65536) { if (lane == 0) alive[n_alive] = (uint16_t)(grp / n_waves); ++n_alive; }
                    else redo_all = true;
                }
            };
            // (the loads of the wave's first group were issued in full above; later groups load the head only)
            while (g < n_groups) {
                const int gn = g + n_waves;
                if (gn < n_groups) load_head(buf_b, gn);
                first_pass(g, buf_a);
                if (gn >= n_groups) break;
                g = gn + n_waves;
                if (g < n_groups) load_head(buf_a, g);
                first_pass(gn, buf_b);
            }
            if (lane == 0 && (n_alive != 0 || redo_all)) atomicOr(any_alive, 1u);
            __syncthreads();
            if (*any_alive == 0u) return;
            (void)stage_table<LUT, BITS>(a.codebooks, rq, a.pq_dim, a.m, lut, max_slot, a.fp8, HROWS, a.pq_dim);
            if (redo_all) {
                for (g = wave; g < n_groups; g += n_waves) {
                    load_group(buf_a, g);
                    store_R(g, accumulate(buf_a, std::integral_constant<int, NBLK>{}));
                }
            } else {
                for (uint32_t t = 0; t < n_alive; ++t) {
                    g = (int)alive[t] * n_waves + wave;
                    load_group(buf_a, g);
                    store_R(g, accumulate(buf_a, std::integral_constant<int, NBLK>{}));
                }
            }
            flush_stage();
            return;
        }
    }
    // step 3: the table
    fp8 = stage_table<LUT, BITS>(a.codebooks, rq, a.pq_dim, a.m, lut, max_slot, a.fp8, 0, a.pq_dim);

    // step 4: Eq. (1), one lane per coded vector; the next group is loaded into the other register
    // buffer while the current one is looked up
    if constexpr (NCH > 0) {
        while (g < n_groups) {
            int gn = g + n_waves;
            if (gn < n_groups) load_group(buf_b, gn);
            store_R(g, accumulate(buf_a, std::integral_constant<int, NBLK>{}));
            if (gn >= n_groups) break;
            g = gn + n_waves;
            if (g < n_groups) load_group(buf_a, g);
            store_R(gn, accumulate(buf_b, std::integral_constant<int, NBLK>{}));
        }
    } else {
        // 4-byte chunks: one code group (WPG words) at a time
        for (; g < n_groups; g += n_waves) {
            float acc = 0.f;
            const int ncg = nch / WPG;
            for (int cg = 0; cg < ncg; ++cg) {
                uint32_t w[WPG];
#pragma unroll
                for (int u = 0; u < WPG; ++u)
                    w[u] = reinterpret_cast<const uint32_t*>(codes_l)[((size_t)g * nch + cg * WPG + u) * 64 + lane];
                acc = add_group<LUT, BITS>(acc, lut, w, cg * SPG, fp8);
                if (prune && ((cg + 1) * SPG) % 16 == 0 && cg + 1 < ncg && ballot64(__float_as_uint(acc) <= bound) == 0) break;
            }
            store_R(g, acc);
        }
    }
    if (filtered) flush_stage();
}

#include "ivfpq_scan_group.hpp"

// Steps 2-3 only: the table of one pair, copied out of LDS byte for byte.
template <int LUT>
__global__ void __launch_bounds__(256)
dump_lut_kernel(const float* __restrict__ query, const float* __restrict__ centroid,
                const float* __restrict__ codebooks, int d, int pq_dim, int m, int bits, Fp8Mode fp8,
                unsigned char* __restrict__ out) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int n_entries = pq_dim << bits;
    const size_t lut_bytes = (size_t)n_entries * LutTraits<LUT>::bytes;
    unsigned char* lut = smem;
    float* rq = reinterpret_cast<float*>(smem + ((lut_bytes + 15) & ~(size_t)15));
    uint32_t* max_slot = reinterpret_cast<uint32_t*>(reinterpret_cast<unsigned char*>(rq) + (((size_t)d * 4 + 15) & ~(size_t)15));
    for (int t = threadIdx.x; t < d; t += blockDim.x) rq[t] = query[t] - centroid[t];
    __syncthreads();
    switch (bits) {
        case 8: (void)stage_table<LUT, 8>(codebooks, rq, pq_dim, m, lut, max_slot, fp8, 0, pq_dim); break;
        case 7: (void)stage_table<LUT, 7>(codebooks, rq, pq_dim, m, lut, max_slot, fp8, 0, pq_dim); break;
        case 6: (void)stage_table<LUT, 6>(codebooks, rq, pq_dim, m, lut, max_slot, fp8, 0, pq_dim); break;
        case 5: (void)stage_table<LUT, 5>(codebooks, rq, pq_dim, m, lut, max_slot, fp8, 0, pq_dim); break;
        default: (void)stage_table<LUT, 4>(codebooks, rq, pq_dim, m, lut, max_slot, fp8, 0, pq_dim); break;
    }
    for (size_t i = threadIdx.x; i < lut_bytes / 4; i += blockDim.x)
        reinterpret_cast<uint32_t*>(out)[i] = reinterpret_cast<const uint32_t*>(lut)[i];
}

// ================================================================================================
// The (query, probe) pairs of the filtered scan grouped by cluster (a counting sort: count, offsets,
// scatter; the order inside a cluster is whatever the atomics give and does not affect any result).
// ================================================================================================
// Plain streaming read: every thread loads 16-byte words grid-strided and folds them into one word
// per workgroup.  It measures the read rate this chip's HBM reaches for the simplest possible access
// pattern - the ceiling a code scan that streams every byte from HBM could attain.
__global__ void __launch_bounds__(256) stream_read_kernel(const uint4* __restrict__ p, size_t n16, uint32_t* __restrict__ out) {
    uint4 acc = make_uint4(0u, 0u, 0u, 0u);
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) {
        const uint4 v = p[i];
        acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
    }
    uint32_t x = acc.x ^ acc.y ^ acc.z ^ acc.w;
    for (int o = 32; o > 0; o >>= 1) x ^= __shfl_xor(x, o);
    __shared__ uint32_t part[4];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = x;
    __syncthreads();
    if (threadIdx.x == 0) out[blockIdx.x] = part[0] ^ part[1] ^ part[2] ^ part[3];
}

__global__ void fill_u32_kernel(uint32_t* p, size_t n, uint32_t v) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

__global__ void pair_count_kernel(const uint4* __restrict__ pairs, uint32_t n_pairs, int n_probes, int n_lists,
                                  uint32_t* __restrict__ counts) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_pairs) return;
    const uint32_t q = i / (uint32_t)(n_probes - 1), p = 1 + i - q * (uint32_t)(n_probes - 1);
    const uint32_t l = pairs[(size_t)q * n_probes + p].x;
    atomicAdd(&counts[l < (uint32_t)n_lists ? l : 0u], 1u);       // a caller-given probe may be out of range
}

// The same two steps for few clusters, where many pairs name the same cluster and one global atomic per
// pair would serialise: a workgroup of 1024 threads takes kPairChunk pairs, counts them per cluster in LDS
// and issues one global atomic per cluster it met.  Dynamic LDS: n_lists words (count) or 2 n_lists (scatter).
constexpr uint32_t kPairChunk = 8192;
constexpr int kPairLdsLists = 8192;       // up to this many clusters

__device__ inline uint32_t pair_cluster(const uint4* __restrict__ pairs, uint32_t i, int n_probes, int n_lists) {
    const uint32_t q = i / (uint32_t)(n_probes - 1), p = 1 + i - q * (uint32_t)(n_probes - 1);
    const uint32_t l = pairs[(size_t)q * n_probes + p].x;
    return l < (uint32_t)n_lists ? l : 0u;                        // a caller-given probe may be out of range
}

__global__ void __launch_bounds__(1024)
pair_count_lds_kernel(const uint4* __restrict__ pairs, uint32_t n_pairs, int n_probes, int n_lists,
                      uint32_t* __restrict__ counts) {
    extern __shared__ uint32_t s_cnt[];
    for (int l = threadIdx.x; l < n_lists; l += blockDim.x) s_cnt[l] = 0;
    __syncthreads();
    const uint32_t i0 = blockIdx.x * kPairChunk, i1 = i0 + kPairChunk < n_pairs ? i0 + kPairChunk : n_pairs;
    for (uint32_t i = i0 + threadIdx.x; i < i1; i += blockDim.x) atomicAdd(&s_cnt[pair_cluster(pairs, i, n_probes, n_lists)], 1u);
    __syncthreads();
    for (int l = threadIdx.x; l < n_lists; l += blockDim.x)
        if (s_cnt[l]) atomicAdd(&counts[l], s_cnt[l]);
}

__global__ void __launch_bounds__(1024)
pair_scatter_lds_kernel(const uint4* __restrict__ pairs, uint32_t n_pairs, int n_probes, int n_lists,
                        const uint32_t* __restrict__ offsets, uint32_t* __restrict__ cursor, uint32_t* __restrict__ order) {
    extern __shared__ uint32_t s_mem[];
    uint32_t* s_cnt = s_mem;                  // pairs of this chunk per cluster, then the running rank
    uint32_t* s_base = s_mem + n_lists;       // first slot of this chunk's pairs inside the cluster's range
    for (int l = threadIdx.x; l < n_lists; l += blockDim.x) s_cnt[l] = 0;
    __syncthreads();
    const uint32_t i0 = blockIdx.x * kPairChunk, i1 = i0 + kPairChunk < n_pairs ? i0 + kPairChunk : n_pairs;
    for (uint32_t i = i0 + threadIdx.x; i < i1; i += blockDim.x) atomicAdd(&s_cnt[pair_cluster(pairs, i, n_probes, n_lists)], 1u);
    __syncthreads();
    for (int l = threadIdx.x; l < n_lists; l += blockDim.x) {
        const uint32_t c = s_cnt[l];
        s_base[l] = c ? offsets[l] + atomicAdd(&cursor[l], c) : 0u;
        s_cnt[l] = 0;
    }
    __syncthreads();
    for (uint32_t i = i0 + threadIdx.x; i < i1; i += blockDim.x) {
        const uint32_t l = pair_cluster(pairs, i, n_probes, n_lists);
        order[s_base[l] + atomicAdd(&s_cnt[l], 1u)] = i;
    }
}

// offsets[l] = counts[0] + ... + counts[l-1]; one workgroup, 4096 counters per trip: four consecutive
// counters per thread (coalesced), a scan inside each wave, the 16 wave totals through LDS
__global__ void __launch_bounds__(1024)
pair_offsets_kernel(const uint32_t* __restrict__ counts, int n_lists, uint32_t* __restrict__ offsets) {
    __shared__ uint32_t wave_total[16];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    uint32_t carry = 0;
    for (int base = 0; base < n_lists; base += 4096) {
        const int i = base + tid * 4;
        uint32_t c[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) c[u] = i + u < n_lists ? counts[i + u] : 0u;
        const uint32_t own = c[0] + c[1] + c[2] + c[3];
        const uint32_t incl = wave_inclusive_scan(own);
        if (lane == kWave - 1) wave_total[wave] = incl;
        __syncthreads();
        uint32_t before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const uint32_t t = wave_total[w];
            before += w < wave ? t : 0u;
            total += t;
        }
        uint32_t at = carry + before + incl - own;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (i + u < n_lists) offsets[i + u] = at;
            at += c[u];
        }
        carry += total;
        __syncthreads();
    }
}

__global__ void pair_scatter_kernel(const uint4* __restrict__ pairs, uint32_t n_pairs, int n_probes, int n_lists,
                                    const uint32_t* __restrict__ offsets, uint32_t* __restrict__ cursor,
                                    uint32_t* __restrict__ order) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_pairs) return;
    const uint32_t q = i / (uint32_t)(n_probes - 1), p = 1 + i - q * (uint32_t)(n_probes - 1);
    uint32_t l = pairs[(size_t)q * n_probes + p].x;
    if (l >= (uint32_t)n_lists) l = 0u;
    order[offsets[l] + atomicAdd(&cursor[l], 1u)] = i;
}

// ================================================================================================
// Between the two scan launches: per query, an upper bound of the k-th smallest R, taken from the
// nearest probed cluster (whose R values are all in place): its k-th smallest R.  With fewer than
// k vectors there the bound admits everything.  The values of that cluster that are not above the
// bound become the first entries of the query's survivor list (behind the cluster's segment of the R
// row: value + position), which the filtered scan extends; the top-k step then reads that list only.
// ================================================================================================
constexpr uint32_t kAdmitAll = 0xFFFFFFFEu;   // every real R is below this, the padding key is above

__global__ void __launch_bounds__(SEL_THREADS)
bound_kernel(float* __restrict__ R, uint32_t* __restrict__ Rpos, size_t stride, const uint4* __restrict__ pairs,
             int n_probes, int k, uint32_t* __restrict__ bounds, uint32_t* __restrict__ counts) {
    constexpr uint32_t KEYS = 4096;         // segments up to this length are selected from LDS
    __shared__ KthShared s;
    __shared__ uint32_t keys[KEYS];
    const int q = blockIdx.x;
    const int tid = threadIdx.x, nth = blockDim.x;
    const uint32_t seg0 = n_probes > 1 ? pairs[(size_t)q * n_probes + 1].w : 0u;
    const uint32_t len0 = pairs[(size_t)q * n_probes].y;       // real values in the segment (the rest is padding)
    uint32_t* row = reinterpret_cast<uint32_t*>(R + (size_t)q * stride);
    uint32_t* row_pos = Rpos + (size_t)q * stride;
    const bool in_lds = seg0 <= KEYS;
    if (in_lds)
        for (uint32_t i = tid; i < seg0; i += nth) keys[i] = row[i];
    uint32_t bound = kAdmitAll;
    if (len0 >= (uint32_t)k && seg0 >= len0) {
        uint32_t r0, r1;
        if (in_lds) bound = block_kth_key(s, seg0, (uint32_t)k, [&](uint32_t i) { return keys[i]; }, &r0, &r1);
        else bound = block_kth_key(s, seg0, (uint32_t)k, [&](uint32_t i) { return row[i]; }, &r0, &r1);
    }
    __syncthreads();
    if (tid == 0) s.n_rec = 0;
    __syncthreads();
    const uint32_t real = len0 < seg0 ? len0 : seg0;
    for (uint32_t i = tid; i < real; i += nth) {
        const uint32_t key = in_lds ? keys[i] : row[i];
        if (key <= bound) {
            const uint32_t slot = seg0 + atomicAdd(&s.n_rec, 1u);
            row[slot] = key;
            row_pos[slot] = i;
        }
    }
    __syncthreads();
    if (tid == 0) { bounds[q] = bound; counts[q] = s.n_rec; }
}

// ================================================================================================
// Step 5: the k smallest (R, id) of a query.  With several probes the candidates are the survivor list
// (the nearest cluster's values under the bound, then what the filtered scan kept); with one probe, the
// cluster's segment itself.
// ================================================================================================
template <int CAP>          // record capacity, >= k
__global__ void __launch_bounds__(SEL_THREADS)
topk_kernel(const float* __restrict__ R, const uint32_t* __restrict__ Rpos, size_t stride,
            const uint32_t* __restrict__ roff, const uint32_t* __restrict__ probes,
            const uint32_t* __restrict__ bounds, const uint32_t* __restrict__ counts, int n_probes, int k,
            const int64_t* __restrict__ list_offsets, const int64_t* __restrict__ ids,
            int64_t* __restrict__ out_ids, float* __restrict__ out_dists) {
    __shared__ RowSelectSharedT<CAP> t;
    auto& s = t.sel;
    const int q = blockIdx.x;
    const int tid = threadIdx.x, nth = blockDim.x;
    const uint32_t* s_roff = roff + (size_t)q * (n_probes + 1);     // read through the vector cache:
    const uint32_t* s_probe = probes + (size_t)q * n_probes;        // only the few survivors look them up
    const uint32_t seg0 = s_roff[1];          // padded length of the nearest probe's segment (a multiple of 64)
    const bool listed = n_probes > 1;         // candidates = the survivor list behind that segment
    const uint32_t n = listed ? counts[q] : seg0;
    const uint32_t* row = reinterpret_cast<const uint32_t*>(R + (size_t)q * stride) + (listed ? seg0 : 0u);
    const uint32_t* row_pos = Rpos + (size_t)q * stride + (listed ? seg0 : 0u);

    // position of candidate i in the unfiltered layout (probe segments back to back)
    auto pos_of = [&](uint32_t i) { return listed ? row_pos[i] : i; };
    // tie key = the caller's id of the candidate at that position (padding slots sort last)
    auto id_of = [&](uint32_t pos, uint32_t key) -> long long {
        if (key == kPadKey) return 0x7FFFFFFFFFFFFFFFll;
        int lo = 0, hi = n_probes;            // largest probe slot with roff[slot] <= pos
        while (hi - lo > 1) {
            int mid = (lo + hi) >> 1;
            if (s_roff[mid] <= pos) lo = mid; else hi = mid;
        }
        return (long long)ids[list_offsets[s_probe[lo]] + (int64_t)(pos - s_roff[lo])];
    };
    // The survivor list was filtered by the query's bound already, so that bound weeds out nothing here: the
    // selection takes its own from a sample of the list (the k-th smallest of its first entries), and one pass over
    // the list with that bound leaves a few hundred candidates.
    const int got = block_select_row(t, row, n, (uint32_t)k, false, 0u, pos_of, id_of);
    for (int j = tid; j < k; j += nth) {
        int64_t id = -1;
        float dist = __uint_as_float(0x7F800000u);
        if (j < got && s.rec_key[j] != kPadKey) { id = (int64_t)s.rec_tie[j]; dist = __uint_as_float(s.rec_key[j]); }
        out_ids[(size_t)q * k + j] = id;
        out_dists[(size_t)q * k + j] = dist;
    }
}

// ================================================================================================
// Re-ranking with the stored vectors: per query the exact squared distances of its candidates (fp32,
// direct form) and the k smallest by (distance, id).  One workgroup per query; a group of 8 adjacent
// lanes per candidate (each lane sums every 8th component, then three exchange steps: a fixed order).
// Candidate ids outside [0, n_data) are skipped.
// ================================================================================================
__global__ void __launch_bounds__(SEL_THREADS)
refine_kernel(const float* __restrict__ data, long long n_data, int d, const float* __restrict__ queries,
              const int64_t* __restrict__ cand, int n_cand, int k, int64_t* __restrict__ out_ids,
              float* __restrict__ out_dists) {
    __shared__ SelectShared s;
    __shared__ uint32_t keys[SEL_CAP];
    const int q = blockIdx.x;
    const int tid = threadIdx.x, nth = blockDim.x;
    const float* qv = queries + (size_t)q * d;
    const int64_t* my = cand + (size_t)q * n_cand;
    for (int base = 0; base < n_cand; base += nth / 8) {
        const int c = base + (tid >> 3);
        const bool valid = c < n_cand;
        const long long id = valid ? (long long)my[c] : -1ll;
        const bool ok = id >= 0 && id < n_data;
        float acc = 0.f;
        if (ok) {
            const float* x = data + (size_t)id * d;
            for (int u = tid & 7; u < d; u += 8) { const float diff = qv[u] - x[u]; acc = __builtin_fmaf(diff, diff, acc); }
        }
        acc = sum_over_8_lanes(acc);
        if (valid && (tid & 7) == 0) keys[c] = ok ? __float_as_uint(acc) : kPadKey;
    }
    __syncthreads();
    const int got = block_select_smallest(s, (uint32_t)n_cand, (uint32_t)k,
        [&](uint32_t i) { return keys[i]; },
        [&](uint32_t i) { return keys[i] == kPadKey ? 0x7FFFFFFFFFFFFFFFll : (long long)my[i]; });
    for (int j = tid; j < k; j += nth) {
        int64_t id = -1;
        float dist = __uint_as_float(0x7F800000u);
        if (j < got && s.rec_key[j] != kPadKey) { id = (int64_t)s.rec_tie[j]; dist = __uint_as_float(s.rec_key[j]); }
        out_ids[(size_t)q * k + j] = id;
        out_dists[(size_t)q * k + j] = dist;
    }
}

// ================================================================================================
// Host side
// ================================================================================================
struct ImageLayout {
    size_t centroids, centroid_norms, codebooks, list_offsets, list_sizes, group_offsets, codes, ids, total;
};

int chunk_width(const ivfpq_index* idx) {
    const int cb = idx->code_bytes(), p = idx->pq_bits;
    const bool wide = cb % 16 == 0 && cb / 16 <= 4 && (p == 4 || p == 8 || (p == 6 && cb == 48));
    return wide ? 16 : 4;
}

ImageLayout image_layout(const ivfpq_index* idx) {
    ImageLayout L{};
    size_t at = 0;
    auto take = [&](size_t bytes) { size_t o = at; at = align_up(at + bytes); return o; };
    L.centroids = take(idx->centroids.size() * sizeof(float));
    L.centroid_norms = take((size_t)idx->n_lists * sizeof(float));
    L.codebooks = take(idx->codebooks.size() * sizeof(float));
    L.list_offsets = take(((size_t)idx->n_lists + 1) * sizeof(int64_t));
    L.list_sizes = take((size_t)idx->n_lists * sizeof(uint32_t));
    L.group_offsets = take(((size_t)idx->n_lists + 1) * sizeof(int64_t));
    L.codes = take((size_t)idx->total_groups * 64 * idx->code_bytes());
    L.ids = take((size_t)idx->n * sizeof(int64_t));
    L.total = at == 0 ? kAlign : at;
    return L;
}

struct Plan {
    int64_t tile;           // queries per tile
    size_t stride;          // R slots per query
    size_t probes, probe_d, roff, pairs, bounds, counts, D, S, split, R, Rpos, order, list_counts, list_cursor, list_offsets, total;
};


// given_probes: the caller chooses the clusters and may name one several times, so the bound on a
// query's candidates is n_probes times the largest cluster rather than the n_probes largest ones
// limit: the bytes the plan should stay within (0: the index's workspace limit); a tile holds at least one
// query, so the caller compares plan->total with what it has.
int make_plan(const ivfpq_index* idx, int64_t nq, int32_t n_probes, bool given_probes, Plan* plan, size_t limit = 0) {
    if (limit == 0) limit = idx->workspace_limit;
    const bool need_D = !given_probes;
    int64_t stride = given_probes
        ? (int64_t)n_probes * (idx->sorted_padded_sizes.empty() ? 0 : idx->sorted_padded_sizes[0])
        : idx->max_padded_candidates(n_probes);
    // the survivor list of a query also takes the nearest cluster's values under the bound
    stride += idx->sorted_padded_sizes.empty() ? 0 : idx->sorted_padded_sizes[0];
    if (stride >= ((int64_t)1 << 31))
        return fail(IVFPQ_EUNSUPPORTED, "a query may see %lld candidates (limit 2^31)", (long long)stride);
    if (stride < 64) stride = 64;
    const size_t strips = ((size_t)idx->n_lists + 31) / 32;      // strip summaries of the ranking keys, narrowest strips
    size_t per_query = (size_t)stride * 8 + (need_D ? ((size_t)idx->n_lists + 4 * strips + coarse_padded_dim(idx->d)) * 4 : 0);
    // what does not grow with the tile: three per-cluster counter arrays, the centroids' bf16 halves, alignment slack
    const size_t fixed = 3 * align_up((size_t)idx->n_lists * 4)
                         + (need_D ? coarse_split_bytes(128, (size_t)idx->n_lists, idx->d) : 0) + 24 * kAlign;      // 128: the query rows' padding
    per_query += (size_t)n_probes * 28 + 16;      // probe lists, distances, offsets, descriptors, order, bound, counter
    int64_t tile = limit > fixed ? (int64_t)((limit - fixed) / per_query) : 1;
    tile = std::max<int64_t>(1, std::min<int64_t>(tile, std::max<int64_t>(nq, 1)));
    plan->tile = tile;
    plan->stride = (size_t)stride;
    size_t at = 0;
    auto take = [&](size_t bytes) { size_t o = at; at = align_up(at + bytes); return o; };
    plan->probes = take((size_t)tile * n_probes * 4);
    plan->probe_d = take((size_t)tile * n_probes * 4);
    plan->roff = take((size_t)tile * (n_probes + 1) * 4);
    plan->pairs = take((size_t)tile * n_probes * 16);
    plan->bounds = take((size_t)tile * 4);
    plan->counts = take((size_t)tile * 4);
    plan->D = take(need_D ? (size_t)tile * idx->n_lists * 4 : 0);
    plan->S = take(need_D ? (size_t)tile * strips * sizeof(StripSummary) : 0);
    plan->split = take(need_D ? coarse_split_bytes((size_t)tile, (size_t)idx->n_lists, idx->d) : 0);
    plan->R = take((size_t)tile * stride * 4);
    plan->Rpos = take((size_t)tile * stride * 4);
    plan->order = take((size_t)tile * (n_probes > 1 ? n_probes - 1 : 0) * 4);
    plan->list_counts = take((size_t)idx->n_lists * 4);
    plan->list_cursor = take((size_t)idx->n_lists * 4);
    plan->list_offsets = take((size_t)idx->n_lists * 4);
    plan->total = at;
    return IVFPQ_OK;
}

int check_search_args(const ivfpq_index* idx, const void* q, int64_t nq, int32_t n_probes, int32_t k,
                      int32_t lut_dtype, bool need_k) {
    if (!idx) return fail(IVFPQ_EINVAL, "null index");
    if (nq < 0) return fail(IVFPQ_EINVAL, "nq=%lld", (long long)nq);
    if (nq > 0 && !q) return fail(IVFPQ_EINVAL, "null queries");
    if (n_probes < 1 || n_probes > idx->n_lists || n_probes > IVFPQ_MAX_PROBES)
        return fail(IVFPQ_EINVAL, "n_probes=%d outside [1, min(n_lists=%d, %d)]", n_probes, idx->n_lists, IVFPQ_MAX_PROBES);
    if (need_k && (k < 1 || k > IVFPQ_MAX_K)) return fail(IVFPQ_EINVAL, "k=%d outside [1, %d]", k, IVFPQ_MAX_K);
    if (lut_dtype < 0 || lut_dtype > 3) return fail(IVFPQ_EINVAL, "unknown lut_dtype %d", lut_dtype);
    return IVFPQ_OK;
}

size_t lut_elem_bytes(int lut_dtype) { return lut_dtype == IVFPQ_LUT_FP32 ? 4 : (lut_dtype == IVFPQ_LUT_FP16 ? 2 : 1); }

size_t scan_lds_bytes(const ivfpq_index* idx, int lut_dtype) {
    size_t lut = (size_t)idx->pq_dim * idx->ksub() * lut_elem_bytes(lut_dtype);
    return ((lut + 15) & ~(size_t)15) + (((size_t)idx->d * 4 + 15) & ~(size_t)15) + 16;
}
// plus the per-wave survivor staging of the filtered scan
size_t scan_lds_bytes_staged(const ivfpq_index* idx, int lut_dtype, int threads) {
    return scan_lds_bytes(idx, lut_dtype) + (size_t)(threads / 64) * (kStageCap * 8 + kAliveCap * 2)
           + (size_t)idx->tuning.lds_pad;      // the pad sits behind everything the kernel addresses
}

int check_device(const ivfpq_index* idx) {
    if (!idx->dev.valid) return fail(IVFPQ_ESTATE, "index has no device image: call ivfpq_upload first");
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev != idx->dev.device)
        return fail(IVFPQ_ESTATE, "index was uploaded to device %d, current device is %d", idx->dev.device, dev);
    return IVFPQ_OK;
}

int scan_threads(const ivfpq_index* idx, int lut_dtype) {
    if (idx->tuning.scan_threads) return idx->tuning.scan_threads;       // validated by ivfpq_set_tuning
    // measured on MI355X: small tables want many 4-wave workgroups per CU; large tables want the
    // largest workgroup of which two still fit the CU's LDS (table + residual + survivor staging);
    // long lists (24 or more 64-vector groups on average) want 2-wave workgroups: the table build of
    // one pair then overlaps the scan of more others
    size_t lds = scan_lds_bytes(idx, lut_dtype);
    if (idx->n_lists > 0 && idx->n / idx->n_lists >= 24 * 64 && lds <= 24 * 1024) return 128;
    if (lds <= 32 * 1024) return 256;       // (half table, 48 sub-spaces, 29 KB: 1.19 ms with 256 threads, 1.26 with 512)
    if (lds <= 40 * 1024) return 512;
    if (2 * (lds + (size_t)16 * kStageCap * 8) <= kLdsBytes) return 1024;
    return 512;
}

// The filtered scan runs its pairs grouped by cluster unless their number does not fit the 32-bit
// order array.  Measured on MI355X (10,000 queries): scan stage 10.4 -> 6.8 ms at 10^8 vectors,
// 1.91 -> 1.51 ms at 10^7, 3.92 -> 3.73 ms at 10^6 (sort kernels included).
constexpr uint32_t kOrderBlock = 64;     // consecutive pairs of the grouped order that stay on one XCD

bool group_pairs_by_cluster(size_t n_pairs) { return n_pairs < ((size_t)1 << 32) - 8 * (size_t)kOrderBlock; }

// The scan kernels address their tables by LDS offsets counted from 0: their dynamic LDS must be the first
// thing in the workgroup's LDS, which holds when the compiled kernel has no static LDS.  Checked once per
// kernel (hipFuncGetAttributes is not a stream operation; later launches make no call besides the launch).
int require_no_static_lds(const void* kernel) {
    static std::mutex mu;
    static std::vector<const void*> ok;
    std::lock_guard<std::mutex> lock(mu);
    for (const void* k : ok)
        if (k == kernel) return IVFPQ_OK;
    hipFuncAttributes attr;
    HIP_TRY(hipFuncGetAttributes(&attr, kernel));
    if (attr.sharedSizeBytes != 0)
        return fail(IVFPQ_EUNSUPPORTED, "internal: a scan kernel was built with %zu bytes of static LDS", (size_t)attr.sharedSizeBytes);
    ok.push_back(kernel);
    return IVFPQ_OK;
}

template <int LUT, int BITS>
int launch_scan_bits(const ScanArgs& a, int cw, int nch, dim3 grid, int threads, size_t lds, hipStream_t st) {
    auto go = [&](auto kernel) -> int {
        if (int s = allow_full_lds(kernel)) return s;
        if (int s = require_no_static_lds(reinterpret_cast<const void*>(kernel))) return s;
        hipLaunchKernelGGL(kernel, grid, dim3(threads), lds, st, a);
        HIP_TRY(hipGetLastError());
        return IVFPQ_OK;
    };
    if (cw == 16) {
        // 16-byte chunks need whole code groups per vector's chunk set: always true for 4- and 8-bit
        // codes; of the other widths only 6-bit codes with 48 bytes per vector qualify
        if constexpr (BITS == 4 || BITS == 8) {
            switch (nch) {
                case 1: return go(scan_kernel<LUT, BITS, 16, 1>);
                case 2: return go(scan_kernel<LUT, BITS, 16, 2>);
                case 3: return go(scan_kernel<LUT, BITS, 16, 3>);
                case 4: return go(scan_kernel<LUT, BITS, 16, 4>);
                default: break;
            }
        } else if constexpr (BITS == 6) {
            if (nch == 3) return go(scan_kernel<LUT, BITS, 16, 3>);
        }
        return fail(IVFPQ_EUNSUPPORTED, "internal: no scan kernel for %d chunks of 16 bytes of %d-bit codes", nch, BITS);
    }
    return go(scan_kernel<LUT, BITS, 4, 0>);
}

template <int LUT>
int launch_scan_lut(const ScanArgs& a, int bits, int cw, int nch, dim3 grid, int threads, size_t lds, hipStream_t st) {
    switch (bits) {
        case 8: return launch_scan_bits<LUT, 8>(a, cw, nch, grid, threads, lds, st);
        case 7: return launch_scan_bits<LUT, 7>(a, cw, nch, grid, threads, lds, st);
        case 6: return launch_scan_bits<LUT, 6>(a, cw, nch, grid, threads, lds, st);
        case 5: return launch_scan_bits<LUT, 5>(a, cw, nch, grid, threads, lds, st);
        default: return launch_scan_bits<LUT, 4>(a, cw, nch, grid, threads, lds, st);
    }
}

// ---- the group kernel: up to G pairs of one cluster per workgroup, tables interleaved entry by entry ----
size_t scan_group_lds_bytes(const ivfpq_index* idx, int lut_dtype, int G, int threads) {
    return kGroupHead + (size_t)idx->pq_dim * ((size_t)1 << idx->pq_bits) * G * lut_elem_bytes(lut_dtype) + (((size_t)G * idx->d * 4 + 15) & ~(size_t)15)
           + (size_t)(threads / 64) * (kGroupStageAll * 8 + kAliveCap * 2) + 16 + (size_t)idx->tuning.lds_pad;
}
// Workgroup size of the group kernel.  Measured on MI355X (filtered scan, 10,000 queries): with long lists (24 or
// more 64-vector groups on average) two-wave workgroups win when six or more of them share a compute unit's LDS
// (e5m3, two pairs, 10^8 vectors: 4.81 ms against 5.30 with four waves) and lose badly otherwise (half table, two
// pairs, 35 KB: 8.04 ms against 5.63).
int scan_group_threads(const ivfpq_index* idx, int lut_dtype, int G) {
    if (idx->tuning.scan_threads) return std::min(idx->tuning.scan_threads, 512);       // the kernel's launch bound
    const bool long_lists = idx->n_lists > 0 && idx->n / idx->n_lists >= 24 * 64;
    return long_lists && scan_group_lds_bytes(idx, lut_dtype, G, 128) <= 24 * 1024 ? 128 : 256;
}
// How many pairs of a cluster share a workgroup (0: the group kernel does not apply).  It serves 8-bit and 4-bit
// codes in 16-byte chunks, sub-vectors of 1, 2 or 4 components and fixed encoding constants.  The widest layout
// whose workgroup leaves room for four workgroups per compute unit (40 KB of LDS) is taken.  With 8-bit codes,
// four pairs only for the one-byte table dtypes: with wider entries the LDS read of four entries costs what it
// saves.  Measured (filtered scan, 10,000 queries; one / two / four pairs): e5m3 at 10^8 vectors, 32 sub-spaces:
// 6.02 / 4.81 / 4.58 ms; at 10^7, 48 sub-spaces: 1.08 / 0.96 / 1.05; half at 10^8: 6.58 / 5.63 / 7.19; float:
// 8.30 / 8.75 / -.  With 4-bit codes (16-entry rows, a few KB of tables) four pairs for every dtype: 10^8 vectors,
// 64 sub-spaces, e5m3 6.67 / 5.95 / 5.21 ms, half 7.56 / 6.48 / 4.62, float 6.31 / 4.71 / 4.02.
int scan_group_width(const ivfpq_index* idx, int lut_dtype, const Fp8Mode& fp8, uint32_t order_block) {
    if ((idx->pq_bits != 8 && idx->pq_bits != 4) || chunk_width(idx) != 16 || fp8.per_table) return 0;
    if (idx->pq_bits == 4 && idx->pq_dim % 16 != 0) return 0;      // the table is built in blocks of 256 entries
    const int m = idx->d / idx->pq_dim;
    if (m != 1 && m != 2 && m != 4) return 0;
    const int want = idx->tuning.scan_share;
    if (want == 1) return 0;
    const bool one_byte = lut_dtype == IVFPQ_LUT_FP8_E5M3 || lut_dtype == IVFPQ_LUT_FP8_E4M4;
    for (int G : {4, 2}) {
        if (want != 0 && want != G) continue;
        if (order_block < (uint32_t)G || order_block % (uint32_t)G) continue;
        const size_t lds = scan_group_lds_bytes(idx, lut_dtype, G, scan_group_threads(idx, lut_dtype, G));
        if (want == G) { if (lds <= kLdsBytes) return G; continue; }
        if (idx->pq_bits == 8) {
            if (G == 4 && !one_byte) continue;
            if (lut_dtype == IVFPQ_LUT_FP32) continue;
        }
        // (64 sub-spaces with the early exit on: both kernels build the second half of the tables only if some group
        // still needs it; 10^6 vectors, e5m3, one / two pairs: 1.43-1.51 / 1.32 ms; half and float tables of two queries
        // exceed the 40 KB and stay with one pair: 1.95 / 2.44 and 2.46 / 3.81 ms)
        if (lds <= 40 * 1024) return G;
    }
    return 0;
}
int launch_scan_group(const ivfpq_index* idx, const ScanArgs& a, int lut_dtype, int G, hipStream_t st) {
    const int threads = scan_group_threads(idx, lut_dtype, G);
    const size_t lds = scan_group_lds_bytes(idx, lut_dtype, G, threads);
    if (lds > kLdsBytes) return fail(IVFPQ_EUNSUPPORTED, "tables + staging + pad need %zu bytes of LDS (limit %zu)", lds, kLdsBytes);
    const uint32_t n_slots = (a.n_pairs + (uint32_t)G - 1u) / (uint32_t)G, per = 8u * (a.order_block / (uint32_t)G);
    const dim3 grid((n_slots + per - 1) / per * per);
    auto go = [&](auto kernel) -> int {
        if (int s = allow_full_lds(kernel)) return s;
        if (int s = require_no_static_lds(reinterpret_cast<const void*>(kernel))) return s;
        hipLaunchKernelGGL(kernel, grid, dim3(threads), lds, st, a);
        HIP_TRY(hipGetLastError());
        return IVFPQ_OK;
    };
    const int nch = idx->code_bytes() / 16;
    auto by_nch = [&](auto lut_tag, auto g_tag) -> int {
        constexpr int LUT = decltype(lut_tag)::value, GG = decltype(g_tag)::value;
        if (idx->pq_bits == 4)
            switch (nch) {
                case 1: return go(scan_group_kernel<LUT, 1, GG, 4, false>);
                case 2: return go(scan_group_kernel<LUT, 2, GG, 4, false>);
                case 3: return go(scan_group_kernel<LUT, 3, GG, 4, false>);
                default: return go(scan_group_kernel<LUT, 4, GG, 4, false>);
            }
        switch (nch) {
            case 1: return go(scan_group_kernel<LUT, 1, GG, 8, false>);
            case 2: return go(scan_group_kernel<LUT, 2, GG, 8, false>);
            case 3: return go(scan_group_kernel<LUT, 3, GG, 8, false>);
            default:
                // 64 sub-spaces with the early exit on: the second half of the tables is built only if needed
                return a.early_exit ? go(scan_group_kernel<LUT, 4, GG, 8, true>) : go(scan_group_kernel<LUT, 4, GG, 8, false>);
        }
    };
    auto by_g = [&](auto lut_tag) -> int {
        return G == 4 ? by_nch(lut_tag, std::integral_constant<int, 4>{}) : by_nch(lut_tag, std::integral_constant<int, 2>{});
    };
    switch (lut_dtype) {
        case IVFPQ_LUT_FP32: return by_g(std::integral_constant<int, IVFPQ_LUT_FP32>{});
        case IVFPQ_LUT_FP16: return by_g(std::integral_constant<int, IVFPQ_LUT_FP16>{});
        case IVFPQ_LUT_FP8_E5M3: return by_g(std::integral_constant<int, IVFPQ_LUT_FP8_E5M3>{});
        default: return by_g(std::integral_constant<int, IVFPQ_LUT_FP8_E4M4>{});
    }
}

int launch_scan(const ivfpq_index* idx, ScanArgs a, int lut_dtype, dim3 grid, hipStream_t st) {
    const int threads = scan_threads(idx, lut_dtype);
    const size_t lds = scan_lds_bytes_staged(idx, lut_dtype, threads);
    if (lds > kLdsBytes)
        return fail(IVFPQ_EUNSUPPORTED, "lookup table + residual + staging need %zu bytes of LDS (limit %zu)", lds, kLdsBytes);
    const int cw = chunk_width(idx);
    const int nch = idx->code_bytes() / cw;
    a.n_chunks = nch;
    const int bits = idx->pq_bits;
    switch (lut_dtype) {
        case IVFPQ_LUT_FP32: return launch_scan_lut<IVFPQ_LUT_FP32>(a, bits, cw, nch, grid, threads, lds, st);
        case IVFPQ_LUT_FP16: return launch_scan_lut<IVFPQ_LUT_FP16>(a, bits, cw, nch, grid, threads, lds, st);
        case IVFPQ_LUT_FP8_E5M3: return launch_scan_lut<IVFPQ_LUT_FP8_E5M3>(a, bits, cw, nch, grid, threads, lds, st);
        default: return launch_scan_lut<IVFPQ_LUT_FP8_E4M4>(a, bits, cw, nch, grid, threads, lds, st);
    }
}

Fp8Mode fp8_mode(const ivfpq_index* idx, int lut_dtype) {
    Fp8Mode m{};
    if (lut_dtype == IVFPQ_LUT_FP8_E5M3 || lut_dtype == IVFPQ_LUT_FP8_E4M4) {
        const ivfpq::Fp8Options& o = idx->fp8_opt[lut_dtype - IVFPQ_LUT_FP8_E5M3];
        m.fixed = fp8_params(lut_dtype == IVFPQ_LUT_FP8_E5M3 ? Fp8Format<IVFPQ_LUT_FP8_E5M3>::shift : Fp8Format<IVFPQ_LUT_FP8_E4M4>::shift,
                             o.bias, o.truncate);
        m.truncate = o.truncate;
        m.per_table = o.per_table;
    }
    return m;
}

ScanArgs base_scan_args(const ivfpq_index* idx, int lut_dtype) {
    ScanArgs a{};
    a.centroids = idx->dev.centroids;
    a.codebooks = idx->dev.codebooks;
    a.list_sizes = idx->dev.list_sizes;
    a.group_offsets = idx->dev.group_offsets;
    a.codes = idx->dev.codes;
    a.d = idx->d; a.pq_dim = idx->pq_dim; a.m = idx->m(); a.bits = idx->pq_bits;
    a.n_lists = idx->n_lists;
    a.fp8 = fp8_mode(idx, lut_dtype);
    a.single_list = -1;
    a.early_exit = idx->tuning.early_exit >= 0;
    return a;
}

// ---- stage timing ----
int timing_mark(const ivfpq_index* idx, hipStream_t st, void** out) {
    if (idx->events_used == idx->event_pool.size()) {
        hipEvent_t e;
        HIP_TRY(hipEventCreate(&e));
        idx->event_pool.push_back((void*)e);
    }
    hipEvent_t e = (hipEvent_t)idx->event_pool[idx->events_used++];
    HIP_TRY(hipEventRecord(e, st));
    *out = (void*)e;
    return IVFPQ_OK;
}

struct StageTimer {
    const ivfpq_index* idx; hipStream_t st; int stage; void* a = nullptr; bool on;
    StageTimer(const ivfpq_index* i, hipStream_t s, int stage_) : idx(i), st(s), stage(stage_), on(i->timing) {}
    int begin() { return on ? timing_mark(idx, st, &a) : IVFPQ_OK; }
    int end() {
        if (!on) return IVFPQ_OK;
        void* b = nullptr;
        if (int s = timing_mark(idx, st, &b)) return s;
        idx->spans.push_back({a, b, stage});
        return IVFPQ_OK;
    }
};

// static_scratch: the workspace is the library's own fixed device array (d_ws is resolved after the checks)
int search_impl(const ivfpq_index* idx, const float* d_queries, int64_t nq, const uint32_t* d_probes_in,
                int32_t n_probes, int32_t k, int32_t lut_dtype, int64_t* d_ids, float* d_dists,
                void* d_ws, size_t ws_bytes, void* hip_stream, bool static_scratch = false) {
    if (int s = check_search_args(idx, d_queries, nq, n_probes, k, lut_dtype, true)) return s;
    if (nq > 0 && (!d_ids || !d_dists)) return fail(IVFPQ_EINVAL, "null output pointer");
    Plan plan;
    if (static_scratch) {
        // sized before anything touches the device: a request beyond the fixed array is refused as such
        if (int s = make_plan(idx, nq, n_probes, d_probes_in != nullptr, &plan, kStaticScratchBytes)) return s;
        if (plan.total > kStaticScratchBytes)
            return fail(IVFPQ_ENOSPACE, "one query with %d probes on this index needs %zu bytes of scratch; the static "
                        "scratch holds %zu (use ivfpq_search with a caller workspace)", n_probes, plan.total, kStaticScratchBytes);
    }
    if (int s = check_device(idx)) return s;
    if (nq == 0) return IVFPQ_OK;
    if (static_scratch) {
        if (int s = static_scratch_ptr(&d_ws)) return s;
        ws_bytes = kStaticScratchBytes;
    } else if (int s = make_plan(idx, nq, n_probes, d_probes_in != nullptr, &plan)) {
        return s;
    }
    if (!d_ws || ws_bytes < plan.total)
        return fail(IVFPQ_ENOSPACE, "workspace of %zu bytes given, %zu needed", ws_bytes, plan.total);
    if (scan_lds_bytes_staged(idx, lut_dtype, scan_threads(idx, lut_dtype)) > kLdsBytes)
        return fail(IVFPQ_EUNSUPPORTED, "lookup table + residual + staging need %zu bytes of LDS (limit %zu)",
                    scan_lds_bytes_staged(idx, lut_dtype, scan_threads(idx, lut_dtype)), kLdsBytes);
    hipStream_t st = (hipStream_t)hip_stream;
    unsigned char* ws = (unsigned char*)d_ws;
    uint32_t* w_probes = (uint32_t*)(ws + plan.probes);
    float* w_probe_d = (float*)(ws + plan.probe_d);
    uint32_t* w_roff = (uint32_t*)(ws + plan.roff);
    uint4* w_pairs = (uint4*)(ws + plan.pairs);
    uint32_t* w_bounds = (uint32_t*)(ws + plan.bounds);
    uint32_t* w_counts = (uint32_t*)(ws + plan.counts);
    uint32_t* w_Rpos = (uint32_t*)(ws + plan.Rpos);
    float* w_D = (float*)(ws + plan.D);
    StripSummary* w_S = (StripSummary*)(ws + plan.S);
    float* w_R = (float*)(ws + plan.R);

    if (idx->timing) { idx->events_used = 0; idx->spans.clear(); idx->stage_valid = true; }
    StageTimer whole(idx, st, 3);
    if (int s = whole.begin()) return s;
    for (int64_t q0 = 0; q0 < nq; q0 += plan.tile) {
        const int tq = (int)std::min<int64_t>(plan.tile, nq - q0);
        const float* qt = d_queries + (size_t)q0 * idx->d;
        // step 1
        StageTimer t0(idx, st, 0);
        if (int s = t0.begin()) return s;
        if (!d_probes_in) {
            StripSummary* strips = coarse_use_strips(tq, idx->n_lists, n_probes) ? w_S : nullptr;
            StageTimer t4(idx, st, 4);
            if (int s = t4.begin()) return s;
            if (int s = launch_coarse(qt, idx->dev.centroids, idx->dev.centroid_norms, tq, idx->n_lists, idx->d, (uint32_t*)w_D, strips, ws + plan.split, st)) return s;
            if (int s = t4.end()) return s;
            launch_select_probes((int)tq, st, (uint32_t*)w_D, (const StripSummary*)strips,
                                 coarse_strip_width(tq, idx->n_lists), qt,
                                 idx->dev.centroids, idx->centroid_norm_max, idx->d, idx->n_lists,
                                 n_probes, idx->dev.list_sizes, idx->dev.group_offsets, w_probes, w_probe_d, w_roff, w_pairs, k);
            HIP_TRY(hipGetLastError());
        } else {
            hipLaunchKernelGGL(layout_probes_kernel, dim3((tq + 255) / 256), dim3(256), 0, st,
                               d_probes_in + (size_t)q0 * n_probes, tq, n_probes, idx->n_lists, idx->dev.list_sizes,
                               idx->dev.group_offsets, w_probes, w_roff, w_pairs);
            HIP_TRY(hipGetLastError());
        }
        if (int s = t0.end()) return s;
        // steps 2-4
        StageTimer t1(idx, st, 1);
        if (int s = t1.begin()) return s;
        // nearest probe of every query first: its R values give the bound that filters the rest
        ScanArgs a = base_scan_args(idx, lut_dtype);
        a.queries = qt; a.pairs = w_pairs; a.R = w_R; a.stride = plan.stride;
        a.n_probes = n_probes; a.bounds = w_bounds; a.counts = w_counts; a.Rpos = w_Rpos;
        a.mode = 1;
        StageTimer t5(idx, st, 5);
        if (int s = t5.begin()) return s;
        if (int s = launch_scan(idx, a, lut_dtype, dim3((unsigned)tq), st)) return s;
        if (int s = t5.end()) return s;
        StageTimer t6(idx, st, 6);
        if (n_probes > 1) {
            hipLaunchKernelGGL(bound_kernel, dim3(tq), dim3(SEL_THREADS), 0, st, w_R, w_Rpos, plan.stride, w_pairs, n_probes, k,
                               w_bounds, w_counts);
            HIP_TRY(hipGetLastError());
            a.mode = 2;
            const size_t n_pairs = (size_t)tq * (n_probes - 1);
            if (group_pairs_by_cluster(n_pairs)) {
                uint32_t* w_order = (uint32_t*)(ws + plan.order);
                uint32_t* w_lc = (uint32_t*)(ws + plan.list_counts);
                uint32_t* w_cur = (uint32_t*)(ws + plan.list_cursor);
                uint32_t* w_lo = (uint32_t*)(ws + plan.list_offsets);
                const unsigned pb = (unsigned)((n_pairs + 255) / 256);
                // counts and cursors are adjacent in the plan only up to alignment: two fills
                hipLaunchKernelGGL(fill_u32_kernel, dim3((idx->n_lists + 255) / 256), dim3(256), 0, st, w_lc, (size_t)idx->n_lists, 0u);
                hipLaunchKernelGGL(fill_u32_kernel, dim3((idx->n_lists + 255) / 256), dim3(256), 0, st, w_cur, (size_t)idx->n_lists, 0u);
                if (idx->n_lists <= kPairLdsLists) {
                    const unsigned cb = (unsigned)((n_pairs + kPairChunk - 1) / kPairChunk);
                    const size_t lds = (size_t)idx->n_lists * 4;
                    if (int s = allow_full_lds(pair_scatter_lds_kernel)) return s;
                    hipLaunchKernelGGL(pair_count_lds_kernel, dim3(cb), dim3(1024), lds, st, w_pairs, (uint32_t)n_pairs, n_probes, idx->n_lists, w_lc);
                    hipLaunchKernelGGL(pair_offsets_kernel, dim3(1), dim3(1024), 0, st, w_lc, idx->n_lists, w_lo);
                    hipLaunchKernelGGL(pair_scatter_lds_kernel, dim3(cb), dim3(1024), 2 * lds, st, w_pairs, (uint32_t)n_pairs, n_probes,
                                       idx->n_lists, w_lo, w_cur, w_order);
                } else {
                    hipLaunchKernelGGL(pair_count_kernel, dim3(pb), dim3(256), 0, st, w_pairs, (uint32_t)n_pairs, n_probes, idx->n_lists, w_lc);
                    hipLaunchKernelGGL(pair_offsets_kernel, dim3(1), dim3(1024), 0, st, w_lc, idx->n_lists, w_lo);
                    hipLaunchKernelGGL(pair_scatter_kernel, dim3(pb), dim3(256), 0, st, w_pairs, (uint32_t)n_pairs, n_probes, idx->n_lists,
                                       w_lo, w_cur, w_order);
                }
                HIP_TRY(hipGetLastError());
                a.order = w_order;
                a.n_pairs = (uint32_t)n_pairs;
                const uint32_t blk = idx->tuning.order_block > 0 ? (uint32_t)idx->tuning.order_block : kOrderBlock;
                a.order_block = blk;
                if (int s = t6.begin()) return s;
                if (const int G = scan_group_width(idx, lut_dtype, a.fp8, blk)) {
                    a.n_chunks = idx->code_bytes() / 16;
                    if (int s = launch_scan_group(idx, a, lut_dtype, G, st)) return s;
                } else {
                    const size_t grid = (n_pairs + 8 * (size_t)blk - 1) / (8 * (size_t)blk) * (8 * (size_t)blk);
                    if (int s = launch_scan(idx, a, lut_dtype, dim3((unsigned)grid), st)) return s;
                }
            } else {
                if (int s = t6.begin()) return s;
                if (int s = launch_scan(idx, a, lut_dtype, dim3((unsigned)n_pairs), st)) return s;
            }
            if (int s = t6.end()) return s;
        }
        if (int s = t1.end()) return s;
        // step 5
        StageTimer t2(idx, st, 2);
        if (int s = t2.begin()) return s;
        if (k <= SEL_CAP_SMALL)
            hipLaunchKernelGGL(topk_kernel<SEL_CAP_SMALL>, dim3(tq), dim3(SEL_THREADS), 0, st, w_R, w_Rpos, plan.stride, w_roff, w_probes,
                               w_bounds, w_counts, n_probes, k, idx->dev.list_offsets, idx->dev.ids, d_ids + (size_t)q0 * k,
                               d_dists + (size_t)q0 * k);
        else
            hipLaunchKernelGGL(topk_kernel<SEL_CAP>, dim3(tq), dim3(SEL_THREADS), 0, st, w_R, w_Rpos, plan.stride, w_roff, w_probes,
                               w_bounds, w_counts, n_probes, k, idx->dev.list_offsets, idx->dev.ids, d_ids + (size_t)q0 * k,
                               d_dists + (size_t)q0 * k);
        HIP_TRY(hipGetLastError());
        if (int s = t2.end()) return s;
    }
    if (int s = whole.end()) return s;
    return IVFPQ_OK;
}

}  // namespace

namespace ivfpq {
void release_device_state(ivfpq_index* idx) {
    for (void* e : idx->event_pool) (void)hipEventDestroy((hipEvent_t)e);
    idx->event_pool.clear();
}
}  // namespace ivfpq

extern "C" {

size_t ivfpq_device_bytes(const ivfpq_index_t* index) {
    if (!index) { set_error("ivfpq_device_bytes: null index"); return 0; }
    return image_layout(index).total;
}

}  // extern "C"

namespace {
int upload_impl(ivfpq_index_t* idx, void* d_buf, size_t bytes, void* hip_stream) {
    if (!idx || !d_buf) return fail(IVFPQ_EINVAL, "ivfpq_upload: null pointer");
    const ImageLayout L = image_layout(idx);
    if (bytes < L.total) return fail(IVFPQ_ENOSPACE, "device buffer of %zu bytes given, %zu needed", bytes, L.total);
    if (((uintptr_t)d_buf % kAlign) != 0) return fail(IVFPQ_EINVAL, "device buffer must be %zu-byte aligned", kAlign);
    if (idx->total_groups >= ((int64_t)1 << 32))
        return fail(IVFPQ_EUNSUPPORTED, "%lld 64-vector groups (limit 2^32)", (long long)idx->total_groups);
    hipStream_t st = (hipStream_t)hip_stream;
    unsigned char* base = (unsigned char*)d_buf;
    const int cb = idx->code_bytes(), cw = chunk_width(idx), nch = cb / cw;

    std::vector<uint32_t> sizes((size_t)idx->n_lists);
    std::vector<int64_t> goff((size_t)idx->n_lists + 1, 0);
    for (int l = 0; l < idx->n_lists; ++l) {
        int64_t len = idx->list_offsets[l + 1] - idx->list_offsets[l];
        sizes[l] = (uint32_t)len;
        goff[l + 1] = goff[l] + (len + 63) / 64;
    }
    std::vector<float> cnorm((size_t)idx->n_lists);
    float cn_max = 0.f;
    for (int l = 0; l < idx->n_lists; ++l) {
        double acc = 0.0;
        for (int t = 0; t < idx->d; ++t) { double v = idx->centroids[(size_t)l * idx->d + t]; acc += v * v; }
        cnorm[l] = (float)acc;
        if (cnorm[l] > cn_max) cn_max = cnorm[l];
    }
    idx->centroid_norm_max = cn_max;
    HIP_TRY(hipMemcpyAsync(base + L.centroid_norms, cnorm.data(), cnorm.size() * 4, hipMemcpyHostToDevice, st));
    // interleave the codes, one cluster at a time, through a bounded staging buffer
    HIP_TRY(hipMemcpyAsync(base + L.centroids, idx->centroids.data(), idx->centroids.size() * 4, hipMemcpyHostToDevice, st));
    HIP_TRY(hipMemcpyAsync(base + L.codebooks, idx->codebooks.data(), idx->codebooks.size() * 4, hipMemcpyHostToDevice, st));
    HIP_TRY(hipMemcpyAsync(base + L.list_offsets, idx->list_offsets.data(), idx->list_offsets.size() * 8, hipMemcpyHostToDevice, st));
    HIP_TRY(hipMemcpyAsync(base + L.list_sizes, sizes.data(), sizes.size() * 4, hipMemcpyHostToDevice, st));
    HIP_TRY(hipMemcpyAsync(base + L.group_offsets, goff.data(), goff.size() * 8, hipMemcpyHostToDevice, st));
    if (idx->n > 0)
        HIP_TRY(hipMemcpyAsync(base + L.ids, idx->ids.data(), idx->ids.size() * 8, hipMemcpyHostToDevice, st));
    HIP_TRY(hipStreamSynchronize(st));

    const size_t group_bytes = (size_t)64 * cb;
    const size_t stage_groups = std::max<size_t>(1, ((size_t)256 << 20) / group_bytes);
    std::vector<uint8_t> stage;
    int64_t g_done = 0;
    while (g_done < idx->total_groups) {
        const int64_t g_end = std::min<int64_t>(idx->total_groups, g_done + (int64_t)stage_groups);
        stage.assign((size_t)(g_end - g_done) * group_bytes, 0);
        // clusters overlapping [g_done, g_end), dealt to a few host threads (each writes its own groups)
        const int l_first = (int)(std::upper_bound(goff.begin(), goff.end(), g_done) - goff.begin()) - 1;
        const int l_last = (int)(std::lower_bound(goff.begin(), goff.end(), g_end) - goff.begin());   // exclusive
        auto interleave = [&](int t, int n_threads) {
            for (int l = l_first + t; l < l_last && l < idx->n_lists; l += n_threads) {
                const int64_t lo = idx->list_offsets[l], len = idx->list_offsets[l + 1] - lo;
                for (int64_t g = std::max(goff[l], g_done); g < std::min(goff[l + 1], g_end); ++g) {
                    uint8_t* dst = stage.data() + (size_t)(g - g_done) * group_bytes;
                    const int64_t first = (g - goff[l]) * 64;
                    for (int v = 0; v < 64 && first + v < len; ++v) {
                        const uint8_t* src = &idx->codes[(size_t)(lo + first + v) * cb];
                        for (int c = 0; c < nch; ++c)
                            std::memcpy(dst + ((size_t)c * 64 + v) * cw, src + (size_t)c * cw, (size_t)cw);
                    }
                }
            }
        };
        const int n_threads = (int)std::max(1u, std::min(16u, std::thread::hardware_concurrency()));
        if (n_threads == 1 || l_last - l_first < 64) {
            interleave(0, 1);
        } else {
            std::vector<std::thread> pool;
            for (int t = 0; t < n_threads; ++t) pool.emplace_back(interleave, t, n_threads);
            for (auto& th : pool) th.join();
        }
        HIP_TRY(hipMemcpy(base + L.codes + (size_t)g_done * group_bytes, stage.data(), stage.size(), hipMemcpyHostToDevice));
        g_done = g_end;
    }
    // set-up of the static scratch for this device (ivfpq_search_static looks it up here, not in the hot loop)
    void* scratch_dev = nullptr;
    if (int s = static_scratch_ptr(&scratch_dev)) return s;
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    idx->dev.valid = true;
    idx->dev.device = dev;
    idx->dev.centroids = (const float*)(base + L.centroids);
    idx->dev.centroid_norms = (const float*)(base + L.centroid_norms);
    idx->dev.codebooks = (const float*)(base + L.codebooks);
    idx->dev.list_offsets = (const int64_t*)(base + L.list_offsets);
    idx->dev.list_sizes = (const uint32_t*)(base + L.list_sizes);
    idx->dev.group_offsets = (const int64_t*)(base + L.group_offsets);
    idx->dev.codes = (const uint8_t*)(base + L.codes);
    idx->dev.ids = (const int64_t*)(base + L.ids);
    return IVFPQ_OK;
}
}  // namespace

extern "C" {

int ivfpq_upload(ivfpq_index_t* idx, void* d_buf, size_t bytes, void* hip_stream) {
    return guarded("ivfpq_upload", [&] { return upload_impl(idx, d_buf, bytes, hip_stream); });
}

size_t ivfpq_search_workspace_bytes(const ivfpq_index_t* index, int64_t nq, int32_t n_probes, int32_t k,
                                    int32_t lut_dtype) {
    (void)k; (void)lut_dtype;
    if (!index || n_probes < 1 || nq < 0) { set_error("ivfpq_search_workspace_bytes: bad arguments"); return 0; }
    Plan own, given;   // large enough for ivfpq_search and for ivfpq_search_with_probes
    if (make_plan(index, nq, n_probes, false, &own) != IVFPQ_OK) return 0;
    if (make_plan(index, nq, n_probes, true, &given) != IVFPQ_OK) return 0;
    return std::max(own.total, given.total);
}

int ivfpq_search(const ivfpq_index_t* index, const float* d_queries, int64_t nq, int32_t n_probes, int32_t k,
                 int32_t lut_dtype, int64_t* d_ids, float* d_dists, void* d_workspace, size_t workspace_bytes,
                 void* hip_stream) {
    return guarded("ivfpq_search", [&] {
        return search_impl(index, d_queries, nq, nullptr, n_probes, k, lut_dtype, d_ids, d_dists, d_workspace,
                           workspace_bytes, hip_stream);
    });
}

int ivfpq_search_static(const ivfpq_index_t* index, const float* d_queries, int64_t nq, int32_t n_probes, int32_t k,
                        int32_t lut_dtype, int64_t* d_ids, float* d_dists, void* hip_stream) {
    return guarded("ivfpq_search_static", [&] {
        return search_impl(index, d_queries, nq, nullptr, n_probes, k, lut_dtype, d_ids, d_dists, nullptr, 0,
                           hip_stream, true);
    });
}

int ivfpq_search_with_probes(const ivfpq_index_t* index, const float* d_queries, int64_t nq,
                             const uint32_t* d_probes, int32_t n_probes, int32_t k, int32_t lut_dtype,
                             int64_t* d_ids, float* d_dists, void* d_workspace, size_t workspace_bytes,
                             void* hip_stream) {
    if (nq > 0 && !d_probes) return fail(IVFPQ_EINVAL, "ivfpq_search_with_probes: null probes");
    return guarded("ivfpq_search_with_probes", [&] {
        return search_impl(index, d_queries, nq, d_probes, n_probes, k, lut_dtype, d_ids, d_dists, d_workspace,
                           workspace_bytes, hip_stream);
    });
}

int ivfpq_select_probes(const ivfpq_index_t* idx, const float* d_queries, int64_t nq, int32_t n_probes,
                        uint32_t* d_probes, float* d_probe_dists, void* d_workspace, size_t workspace_bytes,
                        void* hip_stream) {
    if (int s = check_search_args(idx, d_queries, nq, n_probes, 1, 0, false)) return s;
    if (nq > 0 && !d_probes) return fail(IVFPQ_EINVAL, "ivfpq_select_probes: null output");
    if (int s = check_device(idx)) return s;
    if (nq == 0) return IVFPQ_OK;
    Plan plan;
    if (int s = make_plan(idx, nq, n_probes, false, &plan)) return s;
    if (!d_workspace || workspace_bytes < plan.total)
        return fail(IVFPQ_ENOSPACE, "workspace of %zu bytes given, %zu needed", workspace_bytes, plan.total);
    hipStream_t st = (hipStream_t)hip_stream;
    float* w_D = (float*)((unsigned char*)d_workspace + plan.D);
    StripSummary* w_S = (StripSummary*)((unsigned char*)d_workspace + plan.S);
    for (int64_t q0 = 0; q0 < nq; q0 += plan.tile) {
        const int tq = (int)std::min<int64_t>(plan.tile, nq - q0);
        StripSummary* strips = coarse_use_strips(tq, idx->n_lists, n_probes) ? w_S : nullptr;
        if (int s = launch_coarse(d_queries + (size_t)q0 * idx->d, idx->dev.centroids, idx->dev.centroid_norms, tq,
                                  idx->n_lists, idx->d, (uint32_t*)w_D, strips, (unsigned char*)d_workspace + plan.split, st))
            return s;
        launch_select_probes((int)tq, st, (uint32_t*)w_D, (const StripSummary*)strips,
                             coarse_strip_width(tq, idx->n_lists), d_queries + (size_t)q0 * idx->d, idx->dev.centroids, idx->centroid_norm_max, idx->d,
                             idx->n_lists, n_probes, idx->dev.list_sizes, idx->dev.group_offsets, d_probes + (size_t)q0 * n_probes,
                             d_probe_dists ? d_probe_dists + (size_t)q0 * n_probes : nullptr, (uint32_t*)nullptr,
                             (uint4*)nullptr, 0);
        HIP_TRY(hipGetLastError());
    }
    return IVFPQ_OK;
}

int ivfpq_dump_lut(const ivfpq_index_t* idx, const float* d_query, uint32_t list_id, int32_t lut_dtype,
                   void* d_lut_out, void* hip_stream) {
    if (!idx || !d_query || !d_lut_out) return fail(IVFPQ_EINVAL, "ivfpq_dump_lut: null pointer");
    if (lut_dtype < 0 || lut_dtype > 3) return fail(IVFPQ_EINVAL, "unknown lut_dtype %d", lut_dtype);
    if (list_id >= (uint32_t)idx->n_lists) return fail(IVFPQ_EINVAL, "list_id %u >= n_lists %d", list_id, idx->n_lists);
    if (int s = check_device(idx)) return s;
    const size_t lds = scan_lds_bytes(idx, lut_dtype);
    if (lds > kLdsBytes) return fail(IVFPQ_EUNSUPPORTED, "lookup table needs %zu bytes of LDS (limit %zu)", lds, kLdsBytes);
    hipStream_t st = (hipStream_t)hip_stream;
    const float* centroid = idx->dev.centroids + (size_t)list_id * idx->d;
    auto go = [&](auto kernel) -> int {
        if (int s = allow_full_lds(kernel)) return s;
        hipLaunchKernelGGL(kernel, dim3(1), dim3(256), lds, st, d_query, centroid, idx->dev.codebooks, idx->d,
                           idx->pq_dim, idx->m(), idx->pq_bits, fp8_mode(idx, lut_dtype), (unsigned char*)d_lut_out);
        HIP_TRY(hipGetLastError());
        return IVFPQ_OK;
    };
    switch (lut_dtype) {
        case IVFPQ_LUT_FP32: return go(dump_lut_kernel<IVFPQ_LUT_FP32>);
        case IVFPQ_LUT_FP16: return go(dump_lut_kernel<IVFPQ_LUT_FP16>);
        case IVFPQ_LUT_FP8_E5M3: return go(dump_lut_kernel<IVFPQ_LUT_FP8_E5M3>);
        default: return go(dump_lut_kernel<IVFPQ_LUT_FP8_E4M4>);
    }
}

int ivfpq_scan_list(const ivfpq_index_t* idx, const float* d_query, uint32_t list_id, int32_t lut_dtype,
                    float* d_R_out, void* hip_stream) {
    if (!idx || !d_query) return fail(IVFPQ_EINVAL, "ivfpq_scan_list: null pointer");
    if (lut_dtype < 0 || lut_dtype > 3) return fail(IVFPQ_EINVAL, "unknown lut_dtype %d", lut_dtype);
    if (list_id >= (uint32_t)idx->n_lists) return fail(IVFPQ_EINVAL, "list_id %u >= n_lists %d", list_id, idx->n_lists);
    if (int s = check_device(idx)) return s;
    if (idx->list_offsets[list_id + 1] == idx->list_offsets[list_id]) return IVFPQ_OK;
    if (!d_R_out) return fail(IVFPQ_EINVAL, "ivfpq_scan_list: null output");
    ScanArgs a = base_scan_args(idx, lut_dtype);
    a.queries = d_query; a.R = d_R_out; a.single_list = (int)list_id; a.n_probes = 1;
    return launch_scan(idx, a, lut_dtype, dim3(1), (hipStream_t)hip_stream);
}

int ivfpq_refine(const float* d_data, int64_t n_data, int32_t d, const float* d_queries, int64_t nq,
                 const int64_t* d_cand_ids, int32_t n_cand, int32_t k, int64_t* d_ids, float* d_dists, void* hip_stream) {
    if (nq < 0 || n_data < 0 || d < 1) return fail(IVFPQ_EINVAL, "ivfpq_refine: bad shape");
    if (n_cand < 1 || n_cand > IVFPQ_MAX_K) return fail(IVFPQ_EINVAL, "n_cand=%d outside [1, %d]", n_cand, IVFPQ_MAX_K);
    if (k < 1 || k > IVFPQ_MAX_K) return fail(IVFPQ_EINVAL, "k=%d outside [1, %d]", k, IVFPQ_MAX_K);
    if (nq == 0) return IVFPQ_OK;
    if (!d_queries || !d_cand_ids || !d_ids || !d_dists || (n_data > 0 && !d_data))
        return fail(IVFPQ_EINVAL, "ivfpq_refine: null pointer");
    if (nq > 0x7FFFFFFF) return fail(IVFPQ_EUNSUPPORTED, "ivfpq_refine: nq=%lld (limit 2^31 - 1 per call)", (long long)nq);
    hipLaunchKernelGGL(refine_kernel, dim3((unsigned)nq), dim3(SEL_THREADS), 0, (hipStream_t)hip_stream, d_data,
                       (long long)n_data, d, d_queries, d_cand_ids, n_cand, k, d_ids, d_dists);
    HIP_TRY(hipGetLastError());
    return IVFPQ_OK;
}

int ivfpq_stream_read(const void* d_buf, size_t bytes, uint32_t* d_out, int32_t n_out, void* hip_stream) {
    if (!d_buf || !d_out) return fail(IVFPQ_EINVAL, "null pointer");
    if (n_out < 1 || n_out > 65536) return fail(IVFPQ_EINVAL, "n_out=%d outside 1..65536", n_out);
    if (((uintptr_t)d_buf & 15) != 0 || (bytes & 15) != 0) return fail(IVFPQ_EINVAL, "buffer and size must be multiples of 16 bytes");
    hipLaunchKernelGGL(stream_read_kernel, dim3(n_out), dim3(256), 0, (hipStream_t)hip_stream,
                       (const uint4*)d_buf, bytes / 16, d_out);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(IVFPQ_EHIP, "stream_read_kernel launch failed: %s", hipGetErrorString(e));
    return IVFPQ_OK;
}

int ivfpq_scan_kernel_info(const ivfpq_index_t* idx, int32_t lut_dtype, char* buf, size_t buf_bytes) {
    if (!idx || !buf || buf_bytes == 0) return fail(IVFPQ_EINVAL, "ivfpq_scan_kernel_info: null pointer");
    if (lut_dtype < 0 || lut_dtype > 3) return fail(IVFPQ_EINVAL, "unknown lut_dtype %d", lut_dtype);
    static const char* const names[4] = {"fp32", "fp16", "e5m3", "e4m4"};
    const int threads = scan_threads(idx, lut_dtype), cw = chunk_width(idx), nch = idx->code_bytes() / cw;
    const uint32_t blk = idx->tuning.order_block > 0 ? (uint32_t)idx->tuning.order_block : kOrderBlock;
    if (const int G = scan_group_width(idx, lut_dtype, fp8_mode(idx, lut_dtype), blk))
        snprintf(buf, buf_bytes, "scan_group_kernel<%s, %d-bit codes, %d chunks, %d pairs> %d threads, %zu bytes of LDS", names[lut_dtype], idx->pq_bits, nch, G,
                 scan_group_threads(idx, lut_dtype, G), scan_group_lds_bytes(idx, lut_dtype, G, scan_group_threads(idx, lut_dtype, G)));
    else
        snprintf(buf, buf_bytes, "scan_kernel<%s, %d-bit codes, %d-byte chunks x %d> %d threads, %zu bytes of LDS", names[lut_dtype],
                 idx->pq_bits, cw, cw == 16 ? nch : 0, threads, scan_lds_bytes_staged(idx, lut_dtype, threads));
    return IVFPQ_OK;
}

int ivfpq_set_stage_timing(ivfpq_index_t* index, int32_t enabled) {
    if (!index) return fail(IVFPQ_EINVAL, "null index");
    index->timing = enabled != 0;
    index->stage_valid = false;
    return IVFPQ_OK;
}

int ivfpq_stage_times_ms(ivfpq_index_t* index, float ms[8]) {
    if (!index || !ms) return fail(IVFPQ_EINVAL, "null pointer");
    if (!index->timing || !index->stage_valid) return fail(IVFPQ_ESTATE, "no timed search call recorded");
    for (int i = 0; i < 8; ++i) ms[i] = 0.f;
    for (const auto& sp : index->spans) {
        float t = 0.f;
        HIP_TRY(hipEventElapsedTime(&t, (hipEvent_t)sp.a, (hipEvent_t)sp.b));
        ms[sp.stage] += t;
    }
    return IVFPQ_OK;
}

}  // extern "C"
