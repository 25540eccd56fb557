// Internal definitions shared by the host-side and device-side halves of libivfpq.
#pragma once

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <exception>
#include <new>
#include <string>
#include <vector>

#include "../../include/ivfpq.h"

namespace ivfpq {

// Encoding options of one 8-bit table dtype (ivfpq_set_fp8_encoding).
struct Fp8Options {
    int32_t bias;        // exponent bias of the format
    int32_t truncate;    // 0: round to nearest, ties up; 1: truncate
    int32_t per_table;   // 1: the bias is chosen per (query, cluster) table from its largest entry
};

// Launch heuristics a caller may override per index (ivfpq_set_tuning); 0 = the library's own choice.
struct Tuning {
    int32_t scan_threads = 0;   // workgroup size of the scan kernels (64 ... 1024)
    int32_t order_block = 0;    // consecutive pairs of the cluster-grouped order that stay on one XCD
    int32_t scan_share = 0;     // 0: heuristic; 1: one (query, probe) pair per workgroup; 2 or 4: up to that many pairs of a cluster
    int32_t early_exit = 0;     // 0: on (default); 1: on; -1: off (every lookup of Eq. (1) is made)
    int32_t lds_pad = 0;        // extra bytes of LDS requested per scan workgroup (occupancy experiments)
};

// Device image of an index.  All pointers point into the single buffer the caller handed to
// ivfpq_upload; the library owns none of them.
struct DeviceImage {
    bool valid = false;
    int device = -1;
    const float* centroids = nullptr;      // [n_lists][d]
    const float* centroid_norms = nullptr; // [n_lists] squared L2 norms
    const float* codebooks = nullptr;      // [pq_dim][ksub][m]
    const int64_t* list_offsets = nullptr; // [n_lists+1], unpadded vector offsets (into ids)
    const uint32_t* list_sizes = nullptr;  // [n_lists]
    const int64_t* group_offsets = nullptr;// [n_lists+1], offsets in 64-vector groups (into codes)
    const uint8_t* codes = nullptr;        // interleaved, see ivfpq_upload
    const int64_t* ids = nullptr;          // [n] list order
};

}  // namespace ivfpq

struct ivfpq_index {
    int64_t n = 0;
    int32_t d = 0, n_lists = 0, pq_dim = 0, pq_bits = 0;
    std::vector<float> centroids;       // [n_lists][d]
    std::vector<float> codebooks;       // [pq_dim][2^pq_bits][d/pq_dim]
    std::vector<int64_t> list_offsets;  // [n_lists+1]
    std::vector<uint8_t> codes;         // [n][code_bytes], list order
    std::vector<int64_t> ids;           // [n], list order

    // derived at import
    int64_t total_groups = 0;           // sum over lists of ceil(len/64)
    std::vector<uint32_t> sorted_padded_sizes;  // padded list lengths, descending

    ivfpq::DeviceImage dev;
    ivfpq::Fp8Options fp8_opt[2] = {{15, 0, 0}, {7, 0, 0}};   // e5m3, e4m4 (ivfpq_set_fp8_encoding)
    float centroid_norm_max = 0.f;      // largest squared centroid norm (set by ivfpq_upload)
    size_t workspace_limit = (size_t)32 << 30;   // search scratch (R, positions, ranking values) per query tile

    ivfpq::Tuning tuning;               // ivfpq_set_tuning

    // stage timing (hipEvent_t kept as void* so this header stays free of HIP types).  Search calls take the
    // handle as const and record into these: with timing enabled, calls on one index must not overlap.
    bool timing = false;
    mutable bool stage_valid = false;
    struct Span { void* a; void* b; int stage; };
    mutable std::vector<void*> event_pool;
    mutable std::vector<Span> spans;
    mutable size_t events_used = 0;

    int32_t ksub() const { return 1 << pq_bits; }
    int32_t m() const { return d / pq_dim; }
    int32_t code_bytes() const { return pq_dim * pq_bits / 8; }
    // upper bound of (padded) candidates one query can see with n_probes probes
    int64_t max_padded_candidates(int32_t n_probes) const {
        int64_t s = 0;
        for (int32_t i = 0; i < n_probes && i < (int32_t)sorted_padded_sizes.size(); ++i)
            s += sorted_padded_sizes[i];
        return s;
    }
};

namespace ivfpq {

void set_error(const char* fmt, ...);
int fail(int status, const char* fmt, ...);

// Runs `body` (-> int status) and turns a C++ exception into a status: nothing throws across the C ABI.
template <class Body>
int guarded(const char* what, Body&& body) {
    try {
        return body();
    } catch (const std::bad_alloc&) {
        return fail(IVFPQ_ENOSPACE, "%s: out of host memory", what);
    } catch (const std::exception& e) {
        return fail(IVFPQ_EINVAL, "%s: %s", what, e.what());
    } catch (...) {
        return fail(IVFPQ_EINVAL, "%s: unknown exception", what);
    }
}

// validates shape parameters common to build and import; returns IVFPQ_OK or sets the error
int check_shape(int64_t n, int32_t d, int32_t n_lists, int32_t pq_dim, int32_t pq_bits);

// fills the derived fields after the logical arrays are in place
void finish_import(ivfpq_index* idx);

// SplitMix64: the generator behind every seeded draw of the builders
struct SplitMix64 {
    uint64_t s;
    explicit SplitMix64(uint64_t seed) : s(seed) {}
    uint64_t next() {
        uint64_t z = (s += 0x9E3779B97F4A7C15ull);
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
    uint64_t below(uint64_t bound) { return next() % bound; }
};

// `k` start rows out of `n` (ascending): distinct when n >= k, cycling otherwise
std::vector<int64_t> draw_rows(SplitMix64& rng, int64_t n, int k);
// at most `limit` rows of [0, n) at a fixed stride (all rows when n <= limit)
std::vector<int64_t> stride_rows(int64_t n, int64_t limit);

// called by ivfpq_free before the handle goes away (destroys HIP events); defined in the device half
void release_device_state(ivfpq_index* idx);

}  // namespace ivfpq
