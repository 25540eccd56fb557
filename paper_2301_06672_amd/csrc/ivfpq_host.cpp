// Host half of libivfpq: handle management, import/export of the logical index, and the CPU index
// builder (arXiv 2301.06672, Sec. I-C, first enumeration: clustering, residuals, product
// quantisation, saved lists).  Index construction is not part of the timed search path.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <limits>
#include <memory>
#include <numeric>
#include <unordered_set>

#include <omp.h>

#include "ivfpq_internal.hpp"

namespace ivfpq {

static thread_local std::string g_error;

void set_error(const char* fmt, ...) {
    char buf[1024];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_error = buf;
}

int fail(int status, const char* fmt, ...) {
    char buf[1024];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_error = buf;
    return status;
}

int check_shape(int64_t n, int32_t d, int32_t n_lists, int32_t pq_dim, int32_t pq_bits) {
    if (n < 0 || d < 1 || n_lists < 1 || pq_dim < 1)
        return fail(IVFPQ_EINVAL, "bad shape: n=%lld d=%d n_lists=%d pq_dim=%d", (long long)n, d, n_lists, pq_dim);
    if (d % pq_dim != 0) return fail(IVFPQ_EINVAL, "d=%d is not a multiple of pq_dim=%d", d, pq_dim);
    if (pq_bits < 4 || pq_bits > 8) return fail(IVFPQ_EINVAL, "pq_bits=%d, must be 4 ... 8", pq_bits);
    if ((pq_dim * pq_bits) % 32 != 0)
        return fail(IVFPQ_EINVAL, "pq_dim*pq_bits/8 = %g bytes per vector, must be a multiple of 4",
                    pq_dim * pq_bits / 8.0);
    return IVFPQ_OK;
}

void finish_import(ivfpq_index* idx) {
    idx->total_groups = 0;
    idx->sorted_padded_sizes.resize(idx->n_lists);
    for (int32_t l = 0; l < idx->n_lists; ++l) {
        int64_t len = idx->list_offsets[l + 1] - idx->list_offsets[l];
        int64_t groups = (len + 63) / 64;
        idx->total_groups += groups;
        idx->sorted_padded_sizes[l] = (uint32_t)(groups * 64);
    }
    std::sort(idx->sorted_padded_sizes.begin(), idx->sorted_padded_sizes.end(), std::greater<uint32_t>());
}

// Seeded row draws shared by the host and the device builder.
// `k` start rows out of `n`: distinct when n >= k, cycling otherwise
std::vector<int64_t> draw_rows(SplitMix64& rng, int64_t n, int k) {
    std::vector<int64_t> rows;
    rows.reserve(k);
    if (n >= k) {
        std::unordered_set<int64_t> seen;
        while ((int)rows.size() < k) {
            int64_t r = (int64_t)rng.below((uint64_t)n);
            if (seen.insert(r).second) rows.push_back(r);
        }
        std::sort(rows.begin(), rows.end());
    } else {
        for (int c = 0; c < k; ++c) rows.push_back(n > 0 ? c % n : 0);
    }
    return rows;
}

std::vector<int64_t> stride_rows(int64_t n, int64_t limit) {
    std::vector<int64_t> rows;
    if (n <= limit) {
        rows.resize(n);
        std::iota(rows.begin(), rows.end(), (int64_t)0);
    } else {
        rows.resize(limit);
        for (int64_t i = 0; i < limit; ++i) rows[i] = (int64_t)(((__int128)i * n) / limit);
    }
    return rows;
}

// ------------------------------------------------------------------------------------------------
// k-means used by the builder.  fp32, distance ranking by |c|^2 - 2 x.c (the |x|^2 term does not
// change the arg-min); ties go to the lower centre index.
// ------------------------------------------------------------------------------------------------
namespace {

// labels[i] = nearest centre of row i.  x: [n][dim], centres: [k][dim].
void assign_rows(const float* x, int64_t n, int dim, const float* centres, int k, int32_t* labels) {
    std::vector<float> ct((size_t)dim * k);   // transposed centres [dim][k], scaled by -2
    std::vector<float> cnorm(k);
    for (int c = 0; c < k; ++c) {
        float s = 0.f;
        for (int t = 0; t < dim; ++t) {
            float v = centres[(size_t)c * dim + t];
            s += v * v;
            ct[(size_t)t * k + c] = -2.f * v;
        }
        cnorm[c] = s;
    }
    constexpr int RB = 4;
#pragma omp parallel
    {
        std::vector<float> acc((size_t)RB * k);
#pragma omp for schedule(static)
        for (int64_t i0 = 0; i0 < n; i0 += RB) {
            int rows = (int)std::min<int64_t>(RB, n - i0);
            for (int r = 0; r < RB; ++r) std::memcpy(&acc[(size_t)r * k], cnorm.data(), sizeof(float) * k);
            float* a0 = &acc[0];
            float* a1 = &acc[(size_t)k];
            float* a2 = &acc[(size_t)2 * k];
            float* a3 = &acc[(size_t)3 * k];
            const float* x0 = x + (size_t)i0 * dim;
            const float* x1 = x + (size_t)std::min<int64_t>(i0 + 1, n - 1) * dim;
            const float* x2 = x + (size_t)std::min<int64_t>(i0 + 2, n - 1) * dim;
            const float* x3 = x + (size_t)std::min<int64_t>(i0 + 3, n - 1) * dim;
            for (int t = 0; t < dim; ++t) {
                const float* row = &ct[(size_t)t * k];
                float v0 = x0[t], v1 = x1[t], v2 = x2[t], v3 = x3[t];
#pragma omp simd
                for (int c = 0; c < k; ++c) {
                    float w = row[c];
                    a0[c] += v0 * w;
                    a1[c] += v1 * w;
                    a2[c] += v2 * w;
                    a3[c] += v3 * w;
                }
            }
            for (int r = 0; r < rows; ++r) {
                const float* a = &acc[(size_t)r * k];
                float best = a[0];
                int32_t arg = 0;
                for (int c = 1; c < k; ++c)
                    if (a[c] < best) { best = a[c]; arg = c; }
                labels[i0 + r] = arg;
            }
        }
    }
}

// Lloyd iterations; centres must hold the start on entry.  Empty clusters keep their centre.
void lloyd(const float* x, int64_t n, int dim, int k, int iters, float* centres) {
    std::vector<int32_t> labels((size_t)std::max<int64_t>(n, 1));
    int nt = omp_get_max_threads();
    for (int it = 0; it < iters; ++it) {
        assign_rows(x, n, dim, centres, k, labels.data());
        std::vector<double> sums((size_t)nt * k * dim, 0.0);
        std::vector<int64_t> counts((size_t)nt * k, 0);
#pragma omp parallel
        {
            int t = omp_get_thread_num();
            double* s = &sums[(size_t)t * k * dim];
            int64_t* cnt = &counts[(size_t)t * k];
#pragma omp for schedule(static)
            for (int64_t i = 0; i < n; ++i) {
                int32_t c = labels[i];
                cnt[c] += 1;
                const float* row = x + (size_t)i * dim;
                double* dst = s + (size_t)c * dim;
                for (int u = 0; u < dim; ++u) dst[u] += row[u];
            }
        }
#pragma omp parallel for schedule(static)
        for (int c = 0; c < k; ++c) {
            int64_t total = 0;
            for (int t = 0; t < nt; ++t) total += counts[(size_t)t * k + c];
            if (total == 0) continue;
            for (int u = 0; u < dim; ++u) {
                double s = 0.0;
                for (int t = 0; t < nt; ++t) s += sums[((size_t)t * k + c) * dim + u];
                centres[(size_t)c * dim + u] = (float)(s / (double)total);
            }
        }
    }
}

}  // namespace
}  // namespace ivfpq

using namespace ivfpq;

extern "C" {

const char* ivfpq_last_error(void) { return g_error.c_str(); }

static int build_host_impl(const float* data, int64_t n, int32_t d, int32_t n_lists, int32_t pq_dim,
                           int32_t pq_bits, int32_t kmeans_iters, uint64_t seed, ivfpq_index_t** out) {
    if (!data || !out) return fail(IVFPQ_EINVAL, "ivfpq_build_host: null pointer");
    *out = nullptr;
    if (int st = check_shape(n, d, n_lists, pq_dim, pq_bits)) return st;
    if (n < 1 || n_lists > n) return fail(IVFPQ_EINVAL, "need 1 <= n_lists <= n (n=%lld, n_lists=%d)", (long long)n, n_lists);
    if (kmeans_iters < 0) return fail(IVFPQ_EINVAL, "kmeans_iters=%d", kmeans_iters);

    std::unique_ptr<ivfpq_index> owner(new ivfpq_index);
    ivfpq_index* idx = owner.get();
    idx->n = n; idx->d = d; idx->n_lists = n_lists; idx->pq_dim = pq_dim; idx->pq_bits = pq_bits;
    const int m = d / pq_dim, ksub = 1 << pq_bits, cb = idx->code_bytes();
    SplitMix64 rng(seed ^ 0x2301066720230117ull);

    // (1) clusters: k-means on at most 256 rows per list, taken at a fixed stride
    {
        std::vector<int64_t> rows = stride_rows(n, (int64_t)256 * n_lists);
        std::vector<float> train((size_t)rows.size() * d);
        for (size_t i = 0; i < rows.size(); ++i)
            std::memcpy(&train[i * d], data + (size_t)rows[i] * d, sizeof(float) * d);
        std::vector<int64_t> start = draw_rows(rng, (int64_t)rows.size(), n_lists);
        idx->centroids.resize((size_t)n_lists * d);
        for (int c = 0; c < n_lists; ++c)
            std::memcpy(&idx->centroids[(size_t)c * d], &train[(size_t)start[c] * d], sizeof(float) * d);
        lloyd(train.data(), (int64_t)rows.size(), d, n_lists, kmeans_iters, idx->centroids.data());
    }
    // membership of every row; list order = ascending original id inside each list
    std::vector<int32_t> labels((size_t)n);
    assign_rows(data, n, d, idx->centroids.data(), n_lists, labels.data());
    idx->list_offsets.assign((size_t)n_lists + 1, 0);
    for (int64_t i = 0; i < n; ++i) idx->list_offsets[labels[i] + 1] += 1;
    for (int l = 0; l < n_lists; ++l) idx->list_offsets[l + 1] += idx->list_offsets[l];
    idx->ids.resize((size_t)n);
    {
        std::vector<int64_t> cursor(idx->list_offsets.begin(), idx->list_offsets.end() - 1);
        for (int64_t i = 0; i < n; ++i) idx->ids[cursor[labels[i]]++] = i;
    }
    // (2) residuals, kept in list order
    std::vector<float> residual((size_t)n * d);
#pragma omp parallel for schedule(static)
    for (int64_t pos = 0; pos < n; ++pos) {
        int64_t row = idx->ids[pos];
        const float* c = &idx->centroids[(size_t)labels[row] * d];
        const float* x = data + (size_t)row * d;
        float* r = &residual[(size_t)pos * d];
        for (int t = 0; t < d; ++t) r[t] = x[t] - c[t];
    }
    // (3) one codebook per sub-space, trained on at most 262144 residual rows; then encode all rows
    idx->codebooks.resize((size_t)pq_dim * ksub * m);
    std::vector<uint8_t> sub_codes((size_t)n * pq_dim);
    {
        std::vector<int64_t> rows = stride_rows(n, 262144);
        std::vector<float> train((size_t)rows.size() * m);
        std::vector<float> all((size_t)n * m);
        std::vector<int32_t> lab((size_t)n);
        for (int j = 0; j < pq_dim; ++j) {
#pragma omp parallel for schedule(static)
            for (int64_t i = 0; i < n; ++i)
                std::memcpy(&all[(size_t)i * m], &residual[(size_t)i * d + (size_t)j * m], sizeof(float) * m);
            for (size_t i = 0; i < rows.size(); ++i)
                std::memcpy(&train[i * m], &all[(size_t)rows[i] * m], sizeof(float) * m);
            float* book = &idx->codebooks[(size_t)j * ksub * m];
            std::vector<int64_t> start = draw_rows(rng, (int64_t)rows.size(), ksub);
            for (int c = 0; c < ksub; ++c)
                std::memcpy(book + (size_t)c * m, &train[(size_t)start[c] * m], sizeof(float) * m);
            lloyd(train.data(), (int64_t)rows.size(), m, ksub, kmeans_iters, book);
            assign_rows(all.data(), n, m, book, ksub, lab.data());
#pragma omp parallel for schedule(static)
            for (int64_t i = 0; i < n; ++i) sub_codes[(size_t)i * pq_dim + j] = (uint8_t)lab[i];
        }
    }
    // (4) packed codes in list order
    idx->codes.resize((size_t)n * cb);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        const uint8_t* s = &sub_codes[(size_t)i * pq_dim];
        uint8_t* o = &idx->codes[(size_t)i * cb];
        // one bit string per vector: sub-space j in bits [j*p, (j+1)*p), least significant bit first
        uint32_t acc = 0;
        int have = 0, at = 0;
        for (int j = 0; j < pq_dim; ++j) {
            acc |= (uint32_t)s[j] << have;
            have += pq_bits;
            while (have >= 8) { o[at++] = (uint8_t)acc; acc >>= 8; have -= 8; }
        }
    }
    finish_import(idx);
    *out = owner.release();
    return IVFPQ_OK;
}

int ivfpq_build_host(const float* data, int64_t n, int32_t d, int32_t n_lists, int32_t pq_dim,
                     int32_t pq_bits, int32_t kmeans_iters, uint64_t seed, ivfpq_index_t** out) {
    return guarded("ivfpq_build_host", [&] { return build_host_impl(data, n, d, n_lists, pq_dim, pq_bits, kmeans_iters, seed, out); });
}

static int from_arrays_impl(int64_t n, int32_t d, int32_t n_lists, int32_t pq_dim, int32_t pq_bits,
                            const float* centroids, const float* codebooks, const int64_t* list_offsets,
                            const uint8_t* codes, const int64_t* ids, ivfpq_index_t** out) {
    if (!out) return fail(IVFPQ_EINVAL, "ivfpq_index_from_arrays: null out pointer");
    *out = nullptr;
    if (!centroids || !codebooks || !list_offsets || (n > 0 && (!codes || !ids)))
        return fail(IVFPQ_EINVAL, "ivfpq_index_from_arrays: null pointer");
    if (int st = check_shape(n, d, n_lists, pq_dim, pq_bits)) return st;
    if (list_offsets[0] != 0 || list_offsets[n_lists] != n)
        return fail(IVFPQ_EINVAL, "list_offsets must start at 0 and end at n=%lld (got %lld..%lld)",
                    (long long)n, (long long)list_offsets[0], (long long)list_offsets[n_lists]);
    for (int32_t l = 0; l < n_lists; ++l) {
        int64_t len = list_offsets[l + 1] - list_offsets[l];
        if (len < 0) return fail(IVFPQ_EINVAL, "list_offsets decreases at list %d", l);
        if (len > (int64_t)1 << 30) return fail(IVFPQ_EUNSUPPORTED, "list %d has %lld vectors (limit 2^30)", l, (long long)len);
    }
    std::unique_ptr<ivfpq_index> owner(new ivfpq_index);
    ivfpq_index* idx = owner.get();
    idx->n = n; idx->d = d; idx->n_lists = n_lists; idx->pq_dim = pq_dim; idx->pq_bits = pq_bits;
    const size_t m = (size_t)d / pq_dim, ksub = (size_t)1 << pq_bits, cb = (size_t)idx->code_bytes();
    idx->centroids.assign(centroids, centroids + (size_t)n_lists * d);
    idx->codebooks.assign(codebooks, codebooks + (size_t)pq_dim * ksub * m);
    idx->list_offsets.assign(list_offsets, list_offsets + n_lists + 1);
    if (n > 0) {
        idx->codes.assign(codes, codes + (size_t)n * cb);
        idx->ids.assign(ids, ids + n);
    }
    finish_import(idx);
    *out = owner.release();
    return IVFPQ_OK;
}

int ivfpq_index_from_arrays(int64_t n, int32_t d, int32_t n_lists, int32_t pq_dim, int32_t pq_bits,
                            const float* centroids, const float* codebooks, const int64_t* list_offsets,
                            const uint8_t* codes, const int64_t* ids, ivfpq_index_t** out) {
    return guarded("ivfpq_index_from_arrays", [&] {
        return from_arrays_impl(n, d, n_lists, pq_dim, pq_bits, centroids, codebooks, list_offsets, codes, ids, out);
    });
}

int ivfpq_index_info(const ivfpq_index_t* index, int64_t* n, int32_t* d, int32_t* n_lists,
                     int32_t* pq_dim, int32_t* pq_bits) {
    if (!index) return fail(IVFPQ_EINVAL, "ivfpq_index_info: null index");
    if (n) *n = index->n;
    if (d) *d = index->d;
    if (n_lists) *n_lists = index->n_lists;
    if (pq_dim) *pq_dim = index->pq_dim;
    if (pq_bits) *pq_bits = index->pq_bits;
    return IVFPQ_OK;
}

int ivfpq_index_export(const ivfpq_index_t* index, float* centroids, float* codebooks,
                       int64_t* list_offsets, uint8_t* codes, int64_t* ids) {
    if (!index) return fail(IVFPQ_EINVAL, "ivfpq_index_export: null index");
    if (centroids) std::memcpy(centroids, index->centroids.data(), index->centroids.size() * sizeof(float));
    if (codebooks) std::memcpy(codebooks, index->codebooks.data(), index->codebooks.size() * sizeof(float));
    if (list_offsets) std::memcpy(list_offsets, index->list_offsets.data(), index->list_offsets.size() * sizeof(int64_t));
    if (codes && !index->codes.empty()) std::memcpy(codes, index->codes.data(), index->codes.size());
    if (ids && !index->ids.empty()) std::memcpy(ids, index->ids.data(), index->ids.size() * sizeof(int64_t));
    return IVFPQ_OK;
}

int ivfpq_set_fp8_encoding(ivfpq_index_t* index, int32_t lut_dtype, int32_t bias, int32_t rounding,
                           int32_t per_table_bias) {
    if (!index) return fail(IVFPQ_EINVAL, "ivfpq_set_fp8_encoding: null index");
    if (lut_dtype != IVFPQ_LUT_FP8_E5M3 && lut_dtype != IVFPQ_LUT_FP8_E4M4)
        return fail(IVFPQ_EINVAL, "lut_dtype %d is not an 8-bit table dtype", lut_dtype);
    // every code must stay a finite, normal FP32 number: 1 <= 127 - bias and 127 - bias + (top exponent) <= 254
    const int lo = lut_dtype == IVFPQ_LUT_FP8_E5M3 ? -96 : -100, hi = 110;
    if (bias < lo || bias > hi)
        return fail(IVFPQ_EINVAL, "%s bias %d outside [%d, %d]", lut_dtype == IVFPQ_LUT_FP8_E5M3 ? "e5m3" : "e4m4", bias, lo, hi);
    if (rounding != IVFPQ_ROUND_NEAREST && rounding != IVFPQ_ROUND_TRUNCATE)
        return fail(IVFPQ_EINVAL, "unknown rounding %d", rounding);
    if (per_table_bias != 0 && per_table_bias != 1) return fail(IVFPQ_EINVAL, "per_table_bias=%d (0 or 1)", per_table_bias);
    index->fp8_opt[lut_dtype - IVFPQ_LUT_FP8_E5M3] = {bias, rounding, per_table_bias};
    return IVFPQ_OK;
}

int ivfpq_set_workspace_limit(ivfpq_index_t* index, size_t bytes) {
    if (!index) return fail(IVFPQ_EINVAL, "ivfpq_set_workspace_limit: null index");
    if (bytes < ((size_t)1 << 20)) return fail(IVFPQ_EINVAL, "workspace limit of %zu bytes is below 1 MiB", bytes);
    index->workspace_limit = bytes;
    return IVFPQ_OK;
}

int ivfpq_set_tuning(ivfpq_index_t* index, int32_t knob, int32_t value) {
    if (!index) return fail(IVFPQ_EINVAL, "ivfpq_set_tuning: null index");
    switch (knob) {
        case IVFPQ_TUNE_SCAN_THREADS:
            if (value != 0 && value != 64 && value != 128 && value != 256 && value != 512 && value != 1024)
                return fail(IVFPQ_EINVAL, "scan threads %d (0, 64, 128, 256, 512 or 1024)", value);
            index->tuning.scan_threads = value;
            return IVFPQ_OK;
        case IVFPQ_TUNE_ORDER_BLOCK:
            if (value < 0 || value > (1 << 20)) return fail(IVFPQ_EINVAL, "order block %d outside [0, 2^20]", value);
            index->tuning.order_block = value;
            return IVFPQ_OK;
        case IVFPQ_TUNE_SCAN_SHARE:
            if (value != 0 && value != 1 && value != 2 && value != 4)
                return fail(IVFPQ_EINVAL, "scan share %d (0, 1, 2 or 4)", value);
            index->tuning.scan_share = value;
            return IVFPQ_OK;
        case IVFPQ_TUNE_EARLY_EXIT:
            if (value < -1 || value > 1) return fail(IVFPQ_EINVAL, "early exit %d (-1, 0 or 1)", value);
            index->tuning.early_exit = value;
            return IVFPQ_OK;
        case IVFPQ_TUNE_LDS_PAD:
            if (value < 0 || value > 160 * 1024 || (value & 15)) return fail(IVFPQ_EINVAL, "LDS pad %d (a multiple of 16 in [0, 163840])", value);
            index->tuning.lds_pad = value;
            return IVFPQ_OK;
        default:
            return fail(IVFPQ_EINVAL, "unknown tuning knob %d", knob);
    }
}

int ivfpq_set_e4m4_bias(ivfpq_index_t* index, int32_t bias) {
    if (!index) return fail(IVFPQ_EINVAL, "ivfpq_set_e4m4_bias: null index");
    const ivfpq::Fp8Options& o = index->fp8_opt[1];
    return ivfpq_set_fp8_encoding(index, IVFPQ_LUT_FP8_E4M4, bias, o.truncate, o.per_table);
}

void ivfpq_free(ivfpq_index_t* index) {
    if (!index) return;
    release_device_state(index);
    delete index;
}

}  // extern "C"
