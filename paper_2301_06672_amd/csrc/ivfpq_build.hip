// ivfpq_build.hip -- index construction on the GPU (gfx950): the steps before the search path
// (Sec. I-C, first enumeration): (1) k-means clusters, (2) residuals to the own centroid, (3) one
// codebook per sub-space trained on the residuals and the PQ code of every vector, (4) the saved
// lists.
//
// Every decision is an arg-min of float64 squared distances (components in ascending order, one
// multiply and one add per component, ties to the lower index), and every centre is the float64 sum
// of its members in ascending row order, divided by the count and rounded to fp32 once.  A CPU
// implementation with the same definitions therefore produces the same bits.
//
// Kernels:
//   coarse_rank_*_kernel   MFMA ranking values |c|^2 - 2 x.c of a tile of rows x all centres (all of them for
//                          few centres, else the two smallest of every strip of 32 / 64 centres)
//   nearest_kernel, nearest_strips_kernel   per row the smallest ranking value; a second value within the
//                          rigorous error bound of the first sends the row to exact float64 distances
//   count/offsets/scatter/sort_groups   rows grouped by label, ascending inside a group
//   update_centres_kernel  ordered float64 mean of every group
//   residual_rows_kernel   x - centroid of the own cluster (fp32), for the PQ training rows
//   pq_codes_kernel        nearest codeword per sub-space by float64 distances: training labels, or
//                          the packed PQ codes of all rows in list order
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <memory>
#include <vector>

#include "ivfpq_internal.hpp"
#include "ivfpq_rank.hpp"

using namespace ivfpq;

namespace {

constexpr size_t kRankTileBytes = (size_t)2 << 30;   // ranking values of one tile of rows
constexpr int SORT_CAP = 4096;                       // elements one workgroup sorts in LDS

__global__ void fill_u32_kernel(uint32_t* p, size_t n, uint32_t v) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// dst[i][:] = src[rows[i]][:]
__global__ void gather_rows_kernel(const float* __restrict__ src, const int64_t* __restrict__ rows, int64_t n_rows,
                                   int d, float* __restrict__ dst) {
    size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (size_t)n_rows * d) return;
    size_t i = e / d;
    int t = (int)(e - i * d);
    dst[e] = src[(size_t)rows[i] * d + t];
}

// codebooks[j][c][:] = Rt[init_rows[j][c]][j*m : (j+1)*m]
__global__ void init_codebooks_kernel(const float* __restrict__ Rt, const int64_t* __restrict__ init_rows, int pq_dim,
                                      int ksub, int m, int d, float* __restrict__ codebooks) {
    size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (size_t)pq_dim * ksub * m) return;
    int t = (int)(e % m);
    size_t jc = e / m;
    int j = (int)(jc / ksub);
    codebooks[e] = Rt[(size_t)init_rows[jc] * d + (size_t)j * m + t];
}

// squared norms of the centres (float64 sum rounded once) and the bit pattern of the largest
__global__ void __launch_bounds__(256)
centre_norms_kernel(const float* __restrict__ C, int k, int d, float* __restrict__ norms, uint32_t* __restrict__ max_bits) {
    const int lane = threadIdx.x & 63, c = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (c >= k) return;
    double acc = 0.0;
    for (int t = lane; t < d; t += 64) { double v = (double)C[(size_t)c * d + t]; acc += v * v; }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, kWave);
    if (lane == 0) {
        const float f = (float)acc;
        norms[c] = f;
        atomicMax(max_bits, __float_as_uint(f));
    }
}

// One wave per row.  A: ranking keys of a(x, c) = |c|^2 - 2 x.c for this tile.  The centre with the
// smallest a() is the nearest one unless another a() lies within twice the error bound of a(); then
// the float64 distances of all centres inside that band decide (ties to the lower index).
__global__ void __launch_bounds__(256)
nearest_kernel(const uint32_t* __restrict__ A, const float* __restrict__ X, const float* __restrict__ C,
               const uint32_t* __restrict__ norm_max_bits, int n_rows, int k, int d, int32_t* __restrict__ labels) {
    const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= n_rows) return;
    const uint32_t* keys = A + (size_t)row * k;
    const float* x = X + (size_t)row * d;
    float qn = 0.f;
    for (int t = lane; t < d; t += 64) qn = __builtin_fmaf(x[t], x[t], qn);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) qn += __shfl_xor(qn, off, kWave);
    // the two smallest keys this lane sees (four consecutive keys per 16-byte load when the row is
    // aligned for it, two loads in flight; a lane meets its keys in ascending index order either way)
    uint32_t m1 = 0xFFFFFFFFu, m2 = 0xFFFFFFFFu;
    int i1 = 0x7FFFFFFF;
    auto see = [&](uint32_t v, int c) {
        if (v < m1) { m2 = m1; m1 = v; i1 = c; }
        else if (v < m2) m2 = v;
    };
    if ((k & 3) == 0) {
        const uint4* keys4 = reinterpret_cast<const uint4*>(keys);
        const int k4 = k >> 2;
        int c4 = lane;
        for (; c4 + 64 < k4; c4 += 128) {
            const uint4 x = keys4[c4], y = keys4[c4 + 64];
            see(x.x, 4 * c4); see(x.y, 4 * c4 + 1); see(x.z, 4 * c4 + 2); see(x.w, 4 * c4 + 3);
            see(y.x, 4 * c4 + 256); see(y.y, 4 * c4 + 257); see(y.z, 4 * c4 + 258); see(y.w, 4 * c4 + 259);
        }
        if (c4 < k4) {
            const uint4 x = keys4[c4];
            see(x.x, 4 * c4); see(x.y, 4 * c4 + 1); see(x.z, 4 * c4 + 2); see(x.w, 4 * c4 + 3);
        }
    } else {
        for (int c = lane; c < k; c += 64) see(keys[c], c);
    }
    // wave: smallest key (lowest index among equals) and the second smallest overall
    uint32_t g1 = m1, g2 = m2;
    int gi = i1;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const uint32_t o1 = __shfl_xor(g1, off, kWave), o2 = __shfl_xor(g2, off, kWave);
        const int oi = __shfl_xor(gi, off, kWave);
        if (o1 < g1 || (o1 == g1 && oi < gi)) { g2 = min(g1, o2); g1 = o1; gi = oi; }
        else g2 = min(g2, o1);
    }
    // |a_computed - a_exact| <= delta
    const float delta = rank_error_bound(d, qn, __uint_as_float(*norm_max_bits));
    float lim = ordered_key_value(g1) + 2.f * delta;
    lim += __builtin_fabsf(lim) * 2.3841858e-07f;
    const uint32_t limit = (lim == lim) ? ordered_key(lim) : 0xFFFFFFFFu;
    if (gi >= k) gi = 0;                       // only if every key is the all-ones NaN pattern
    if (g2 > limit) {
        if (lane == 0) labels[row] = gi;
        return;
    }
    double best = __longlong_as_double(0x7FF0000000000000ll);
    int arg = 0x7FFFFFFF;
    for (int c = lane; c < k; c += 64) {
        if (keys[c] > limit) continue;
        const float* cc = C + (size_t)c * d;
        double dist = 0.0;
        for (int t = 0; t < d; ++t) { const double diff = (double)x[t] - (double)cc[t]; dist += diff * diff; }
        if (dist < best) { best = dist; arg = c; }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const double ob = __shfl_xor(best, off, kWave);
        const int oa = __shfl_xor(arg, off, kWave);
        if (ob < best || (ob == best && oa < arg)) { best = ob; arg = oa; }
    }
    if (lane == 0) labels[row] = arg < k ? arg : gi;      // no finite distance (NaN inputs): stay in range
}

// ---- rows grouped by label ----------------------------------------------------------------------
// The same decision from the ranking kernel's strip summaries S[n_strips][n_rows] (the two smallest
// tagged keys of every strip of strip_w centres): 64 rows per workgroup, four threads per row that each
// scan a quarter of the strips.  The smallest key and the second smallest of everything else decide: if
// the second lies beyond the first by more than the error bound, the strip's best centre is the answer;
// otherwise the strips that can hold the nearest centre are compared by float64 distances (their best
// centre, or all their centres if the strip's second key is within the bound as well).
__global__ void __launch_bounds__(256)
nearest_strips_kernel(const StripSummary* __restrict__ S, int strip_w, const float* __restrict__ X, const float* __restrict__ C,
                      const uint32_t* __restrict__ norm_max_bits, int n_rows, int k, int d, int32_t* __restrict__ labels) {
    __shared__ uint32_t s_b1[4][64], s_b2[4][64], s_i1[4][64];
    const int r = threadIdx.x & 63, sl = threadIdx.x >> 6;
    const int row = blockIdx.x * 64 + r;
    const int n_strips = (k + strip_w - 1) / strip_w;
    const size_t stride = (size_t)n_rows;
    uint32_t b1 = 0xFFFFFFFFu, b2 = 0xFFFFFFFFu, i1 = 0u;
    if (row < n_rows)
        for (int i = sl; i < n_strips; i += 4) {
            const StripSummary v = S[(size_t)i * stride + row];
            if (v.x < b1) { b2 = b1 < v.y ? b1 : v.y; b1 = v.x; i1 = (uint32_t)i; }
            else if (v.x < b2) b2 = v.x;
        }
    s_b1[sl][r] = b1; s_b2[sl][r] = b2; s_i1[sl][r] = i1;
    __syncthreads();
    // rows whose second key is within the error bound of the first wait here for the float64 comparison,
    // which the whole workgroup makes row by row
    __shared__ uint32_t s_slow[64], s_limit[64];
    __shared__ int s_first[64];
    __shared__ uint32_t s_n_slow, s_n_cand;
    __shared__ int s_cand[1024];
    __shared__ double s_best[256];
    __shared__ int s_arg[256];
    if (threadIdx.x == 0) s_n_slow = 0u;
    __syncthreads();
    if (sl == 0 && row < n_rows) {
        for (int o = 1; o < 4; ++o) {
            const uint32_t c1 = s_b1[o][r], c2 = s_b2[o][r], ci = s_i1[o][r];
            if (c1 < b1 || (c1 == b1 && ci < i1)) { b2 = b1 < c2 ? b1 : c2; b1 = c1; i1 = ci; }
            else if (c1 < b2) b2 = c1;
        }
        const float* x = X + (size_t)row * d;
        float qn = 0.f;
        for (int t = 0; t < d; ++t) qn = __builtin_fmaf(x[t], x[t], qn);
        const float delta = rank_error_bound(d, qn, __uint_as_float(*norm_max_bits));
        float lim = ordered_key_value(b1 | 63u) + 2.f * delta;
        lim += __builtin_fabsf(lim) * 2.3841858e-07f;
        const uint32_t limit = (lim == lim) ? ordered_key(lim) : 0xFFFFFFFFu;
        int first = (int)(i1 * (uint32_t)strip_w + (b1 & 63u));
        if (first >= k) first = 0;             // only if every key is the all-ones pattern
        if ((b2 & ~63u) > limit) {
            labels[row] = first;
        } else {
            const uint32_t slot = atomicAdd(&s_n_slow, 1u);
            s_slow[slot] = (uint32_t)r; s_limit[slot] = limit; s_first[slot] = first;
        }
    }
    __syncthreads();
    const uint32_t n_slow = s_n_slow;
    const int tid = threadIdx.x;
    for (uint32_t w = 0; w < n_slow; ++w) {
        const int srow = blockIdx.x * 64 + (int)s_slow[w];
        const uint32_t limit = s_limit[w];
        const float* x = X + (size_t)srow * d;
        if (tid == 0) s_n_cand = 0u;
        __syncthreads();
        // the centres that can be the nearest: per strip inside the bound its best one, its best two, or all
        for (int i = tid; i < n_strips; i += 256) {
            const StripSummary v = S[(size_t)i * stride + srow];
            if ((v.x & ~63u) > limit) continue;
            const int c0 = i * strip_w;
            int take[2], n_take = 0;
            bool all = false;
            if ((v.y & ~63u) > limit) { take[n_take++] = c0 + (int)(v.x & 63u); }
            else if ((v.z & ~63u) > limit) { take[n_take++] = c0 + (int)(v.x & 63u); take[n_take++] = c0 + (int)(v.y & 63u); }
            else all = true;
            if (all) {
                const int c1 = c0 + strip_w < k ? c0 + strip_w : k;
                const uint32_t slot = atomicAdd(&s_n_cand, (uint32_t)(c1 - c0));
                for (int c = c0; c < c1; ++c)
                    if (slot + (uint32_t)(c - c0) < 1024u) s_cand[slot + (uint32_t)(c - c0)] = c;
            } else {
                for (int u = 0; u < n_take; ++u)
                    if (take[u] < k) {
                        const uint32_t slot = atomicAdd(&s_n_cand, 1u);
                        if (slot < 1024u) s_cand[slot] = take[u];
                    }
            }
        }
        __syncthreads();
        const uint32_t n_cand = s_n_cand;
        double best = __longlong_as_double(0x7FF0000000000000ll);
        int arg = 0x7FFFFFFF;
        auto try_centre = [&](int c) {
            const float* cc = C + (size_t)c * d;
            double dist = 0.0;
            for (int t = 0; t < d; ++t) { const double diff = (double)x[t] - (double)cc[t]; dist += diff * diff; }
            if (dist < best || (dist == best && c < arg)) { best = dist; arg = c; }
        };
        if (n_cand <= 1024u) {
            for (uint32_t j = tid; j < n_cand; j += 256) try_centre(s_cand[j]);
        } else {
            // more than the list holds (a plateau of equal ranking values): every thread takes whole strips
            for (int i = tid; i < n_strips; i += 256) {
                const StripSummary v = S[(size_t)i * stride + srow];
                if ((v.x & ~63u) > limit) continue;
                const int c0 = i * strip_w, c1 = c0 + strip_w < k ? c0 + strip_w : k;
                for (int c = c0; c < c1; ++c) try_centre(c);
            }
        }
        s_best[tid] = best; s_arg[tid] = arg;
        __syncthreads();
        for (int off = 128; off > 0; off >>= 1) {
            if (tid < off) {
                const double ob = s_best[tid + off];
                const int oa = s_arg[tid + off];
                if (ob < s_best[tid] || (ob == s_best[tid] && oa < s_arg[tid])) { s_best[tid] = ob; s_arg[tid] = oa; }
            }
            __syncthreads();
        }
        if (tid == 0) labels[srow] = s_arg[0] < k ? s_arg[0] : s_first[w];      // no finite distance (NaN inputs): stay in range
        __syncthreads();
    }
}

__global__ void count_labels_kernel(const int32_t* __restrict__ labels, size_t n, uint32_t* __restrict__ counts) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) atomicAdd(&counts[labels[i]], 1u);
}

// offsets[0] = 0, offsets[g+1] = counts[0] + ... + counts[g]; one workgroup
__global__ void __launch_bounds__(1024)
offsets_kernel(const uint32_t* __restrict__ counts, int k, int64_t* __restrict__ offsets) {
    __shared__ unsigned long long part[1024];
    __shared__ unsigned long long carry;
    const int tid = threadIdx.x;
    if (tid == 0) { carry = 0; offsets[0] = 0; }
    __syncthreads();
    for (int base = 0; base < k; base += 1024) {
        const int g = base + tid;
        part[tid] = g < k ? counts[g] : 0u;
        __syncthreads();
        for (int off = 1; off < 1024; off <<= 1) {
            unsigned long long v = tid >= off ? part[tid - off] : 0ull;
            __syncthreads();
            part[tid] += v;
            __syncthreads();
        }
        if (g < k) offsets[g + 1] = (int64_t)(carry + part[tid]);
        __syncthreads();
        if (tid == 1023) carry += part[1023];
        __syncthreads();
    }
}

__global__ void scatter_rows_kernel(const int32_t* __restrict__ labels, size_t n, const int64_t* __restrict__ offsets,
                                    uint32_t* __restrict__ cursor, uint32_t* __restrict__ order) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t g = labels[i];
    order[(size_t)offsets[g] + atomicAdd(&cursor[g], 1u)] = (uint32_t)i;
}

// sorts s[0, np2) ascending, np2 a power of two (bitonic network, one workgroup)
__device__ void bitonic_lds(uint32_t* s, int np2) {
    for (int size = 2; size <= np2; size <<= 1)
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int i = threadIdx.x; i < (np2 >> 1); i += blockDim.x) {
                const int lo = 2 * i - (i & (stride - 1)), hi = lo + stride;
                const uint32_t a = s[lo], b = s[hi];
                const bool up = (lo & size) == 0;
                if ((a > b) == up) { s[lo] = b; s[hi] = a; }
            }
            __syncthreads();
        }
}

// The scatter above leaves every group in arbitrary order: one workgroup per group sorts it ascending
// (distinct values).  Groups longer than SORT_CAP: sorted runs of SORT_CAP, then pairwise merges by
// rank between `order` and `tmp`.
__global__ void __launch_bounds__(256)
sort_groups_kernel(uint32_t* __restrict__ order, uint32_t* __restrict__ tmp, const int64_t* __restrict__ offsets) {
    __shared__ uint32_t s[SORT_CAP];
    const size_t lo = (size_t)offsets[blockIdx.x], len = (size_t)offsets[blockIdx.x + 1] - lo;
    if (len < 2) return;
    uint32_t* seg = order + lo;
    for (size_t c0 = 0; c0 < len; c0 += SORT_CAP) {
        const int n = (int)min((size_t)SORT_CAP, len - c0);
        int np2 = 2;
        while (np2 < n) np2 <<= 1;
        for (int i = threadIdx.x; i < np2; i += blockDim.x) s[i] = i < n ? seg[c0 + i] : 0xFFFFFFFFu;
        __syncthreads();
        bitonic_lds(s, np2);
        for (int i = threadIdx.x; i < n; i += blockDim.x) seg[c0 + i] = s[i];
        __syncthreads();
    }
    if (len <= SORT_CAP) return;
    uint32_t* src = seg;
    uint32_t* dst = tmp + lo;
    for (size_t width = SORT_CAP; width < len; width <<= 1) {
        for (size_t i = threadIdx.x; i < len; i += blockDim.x) {
            const size_t run = i / width, a0 = (run >> 1) * 2 * width, b0 = a0 + width;
            const bool right = (run & 1) != 0;
            // the sibling run this element is ranked in
            const size_t o0 = right ? a0 : b0;
            const size_t o_len = o0 >= len ? 0 : min(width, len - o0);
            const uint32_t v = src[i];
            size_t l = 0, h = o_len;           // number of sibling elements below v
            while (l < h) {
                const size_t mid = (l + h) >> 1;
                if (src[o0 + mid] < v) l = mid + 1; else h = mid;
            }
            dst[a0 + (i - (right ? b0 : a0)) + l] = v;
        }
        __syncthreads();
        uint32_t* t = src; src = dst; dst = t;
    }
    if (src != seg) {
        for (size_t i = threadIdx.x; i < len; i += blockDim.x) seg[i] = src[i];
    }
}

// One wave per group: centre = float64 sum of the members in ascending order / count, rounded to
// fp32; an empty group keeps its centre.  Item i of `order` is (row, sub) = (i / items_per_row,
// i % items_per_row); its components are X[row * row_stride + sub * dim + t].
__global__ void __launch_bounds__(256)
update_centres_kernel(const float* __restrict__ X, size_t row_stride, int items_per_row, int dim,
                      const uint32_t* __restrict__ order, const int64_t* __restrict__ offsets, int k,
                      float* __restrict__ centres) {
    const int lane = threadIdx.x & 63, g = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (g >= k) return;
    const size_t lo = (size_t)offsets[g], hi = (size_t)offsets[g + 1];
    if (lo == hi) return;
    for (int t = lane; t < dim; t += 64) {
        double acc = 0.0;
        for (size_t i = lo; i < hi; ++i) {
            const uint32_t item = order[i];
            const size_t row = item / (uint32_t)items_per_row, sub = item % (uint32_t)items_per_row;
            acc += (double)X[row * row_stride + sub * dim + t];
        }
        centres[(size_t)g * dim + t] = (float)(acc / (double)(hi - lo));
    }
}

// Rt[i][:] = data[rows[i]][:] - C[labels[rows[i]]][:]   (fp32)
__global__ void residual_rows_kernel(const float* __restrict__ data, const int64_t* __restrict__ rows, int64_t n_rows,
                                     const int32_t* __restrict__ labels, const float* __restrict__ C, int d,
                                     float* __restrict__ Rt) {
    size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (size_t)n_rows * d) return;
    size_t i = e / d;
    int t = (int)(e - i * d);
    const int64_t row = rows[i];
    Rt[e] = data[(size_t)row * d + t] - C[(size_t)labels[row] * d + t];
}

// Nearest codeword per sub-space.  The codes of a vector are one bit string, sub-space j in bits
// [j*BITS, (j+1)*BITS); a code group is the shortest run of sub-spaces that ends on a 32-bit boundary
// (SPG sub-spaces in WPG words: 8 in 1 for 4-bit codes, 4 in 1 for 8-bit, 32 in 5 / 16 in 3 / 32 in 7
// for 5 / 6 / 7 bits).  A thread handles position p (blockIdx.x * 256 + threadIdx.x) and the code
// group blockIdx.y; the group's codebooks sit in LDS.  Row of position p: order[p] (or p); residual = X[row] - C[labels[row]] in
// fp32 (or X[row] itself when C is null).  Outputs (either may be null): train_labels[p][j] =
// j * ksub + code; codes32[p][...] = the group's words of the packed code.
template <int BITS>
__global__ void __launch_bounds__(256)
pq_codes_kernel(const float* __restrict__ X, const uint32_t* __restrict__ order, const int32_t* __restrict__ labels,
                const float* __restrict__ C, const float* __restrict__ codebooks, size_t n_pos, int d, int pq_dim, int m,
                int32_t* __restrict__ train_labels, uint32_t* __restrict__ codes32) {
    extern __shared__ float cb[];              // [SPG][ksub][m]
    constexpr int G = (BITS % 8 == 0) ? 8 : (BITS % 4 == 0) ? 4 : (BITS % 2 == 0) ? 2 : 1;   // gcd(BITS, 32)
    constexpr int SPW = 32 / G, WPG = BITS / G, KSUB = 1 << BITS;                             // SPW: sub-spaces per group
    const int group = blockIdx.y, j0 = group * SPW;
    const int per_word = SPW * KSUB * m;
    for (int e = threadIdx.x; e < per_word; e += blockDim.x) cb[e] = codebooks[(size_t)j0 * KSUB * m + e];
    __syncthreads();
    const size_t p = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= n_pos) return;
    const size_t row = order ? order[p] : p;
    const float* x = X + row * d;
    const float* c = C ? C + (size_t)labels[row] * d : nullptr;
    unsigned long long acc_bits = 0;           // codes waiting to fill a word, lowest sub-space in the low bits
    int have = 0, word = 0;
    const size_t words_per_code = (size_t)(pq_dim / SPW) * WPG;
    for (int s = 0; s < SPW; ++s) {
        const int j = j0 + s;
        const float* xs = x + (size_t)j * m;
        const float* book = cb + (size_t)s * KSUB * m;
        double best = __longlong_as_double(0x7FF0000000000000ll);
        int arg = 0;
        if (m <= 4) {
            float r[4] = {0.f, 0.f, 0.f, 0.f};
            for (int t = 0; t < m; ++t) r[t] = c ? xs[t] - c[(size_t)j * m + t] : xs[t];
            for (int code = 0; code < KSUB; ++code) {
                double dist = 0.0;
                for (int t = 0; t < m; ++t) { const double diff = (double)r[t] - (double)book[code * m + t]; dist += diff * diff; }
                if (dist < best) { best = dist; arg = code; }
            }
        } else {
            for (int code = 0; code < KSUB; ++code) {
                double dist = 0.0;
                for (int t = 0; t < m; ++t) {
                    const float r = c ? xs[t] - c[(size_t)j * m + t] : xs[t];
                    const double diff = (double)r - (double)book[code * m + t];
                    dist += diff * diff;
                }
                if (dist < best) { best = dist; arg = code; }
            }
        }
        if (train_labels) train_labels[p * pq_dim + j] = j * KSUB + arg;
        acc_bits |= (unsigned long long)arg << have;
        have += BITS;
        if (have >= 32) {
            if (codes32) codes32[p * words_per_code + (size_t)group * WPG + word] = (uint32_t)acc_bits;
            acc_bits >>= 32;
            have -= 32;
            ++word;
        }
    }
}

// ---- host side ----------------------------------------------------------------------------------
inline int sub_spaces_per_group(int bits) { return bits % 8 == 0 ? 4 : bits % 4 == 0 ? 8 : bits % 2 == 0 ? 16 : 32; }

inline unsigned blocks_for(size_t n, unsigned threads) { return (unsigned)((n + threads - 1) / threads); }

struct BuildPlan {
    int64_t n, n_ct, n_pt;          // rows, coarse training rows, PQ training rows
    int d, n_lists, pq_dim, pq_bits, m, ksub;
    size_t tile_rows;               // rows per ranking tile
    size_t n_group;                 // largest number of items grouped at once
    size_t k_group;                 // largest number of groups
    // offsets into the workspace
    bool use_strips;                // nearest centres from strip summaries instead of all ranking values
    size_t Xt, A, S, split, C, cnorm, cmax, labels_t, labels_all, order, tmp, counts, cursor, offsets, ct_rows, pt_rows,
           init_rows, Rt, pq_labels, codebooks, codes, total;
};

// Scratch of the nearest-centre step for up to n_rows_max rows against k centres: the tile height and
// the offsets of A (all ranking values; few centres) or S (strip summaries), of the bf16 operands, of the
// centre norms and their maximum.
template <class Take>
void plan_nearest(BuildPlan& P, size_t n_rows_max, int k, int d, Take&& take) {
    const size_t strips = ((size_t)k + 31) / 32;
    P.use_strips = k >= 256;
    const size_t per_row = (P.use_strips ? strips * sizeof(StripSummary) : (size_t)k * 4) + (size_t)coarse_padded_dim(d) * 4;
    P.tile_rows = std::max<size_t>(1, std::min<size_t>(kRankTileBytes / per_row, (size_t)2 << 20));
    P.tile_rows = std::min<size_t>(P.tile_rows, std::max<size_t>(n_rows_max, 1));
    P.A = take(P.use_strips ? 0 : P.tile_rows * (size_t)k * 4);
    P.S = take(P.use_strips ? P.tile_rows * strips * sizeof(StripSummary) : 0);
    P.split = take(coarse_split_bytes(P.tile_rows, (size_t)k, d));
    P.cnorm = take((size_t)k * 4);
    P.cmax = take(4);
}

BuildPlan make_build_plan(int64_t n, int d, int n_lists, int pq_dim, int pq_bits, int64_t n_ct, int64_t n_pt) {
    BuildPlan P{};
    P.n = n; P.n_ct = n_ct; P.n_pt = n_pt; P.d = d; P.n_lists = n_lists; P.pq_dim = pq_dim; P.pq_bits = pq_bits;
    P.m = d / pq_dim; P.ksub = 1 << pq_bits;
    P.n_group = std::max<size_t>((size_t)n, (size_t)n_pt * pq_dim);
    P.k_group = std::max<size_t>((size_t)n_lists, (size_t)pq_dim * P.ksub);
    size_t at = 0;
    auto take = [&](size_t bytes) { size_t o = at; at = align_up(at + bytes); return o; };
    P.Xt = take((size_t)n_ct * d * 4);
    plan_nearest(P, (size_t)std::max<int64_t>(n, n_ct), n_lists, d, take);
    P.C = take((size_t)n_lists * d * 4);
    P.labels_t = take((size_t)n_ct * 4);
    P.labels_all = take((size_t)n * 4);
    P.order = take(P.n_group * 4);
    P.tmp = take(P.n_group * 4);
    P.counts = take(P.k_group * 4);
    P.cursor = take(P.k_group * 4);
    P.offsets = take((P.k_group + 1) * 8);
    P.ct_rows = take((size_t)n_ct * 8);
    P.pt_rows = take((size_t)n_pt * 8);
    P.init_rows = take(P.k_group * 8);
    P.Rt = take((size_t)n_pt * d * 4);
    P.pq_labels = take((size_t)n_pt * pq_dim * 4);
    P.codebooks = take((size_t)pq_dim * P.ksub * P.m * 4);
    P.codes = take((size_t)n * (pq_dim * pq_bits / 8));
    P.total = at;
    return P;
}

// Everything the launches of a build assume, checked on the host before the first of them: workgroup counts
// that fit a grid dimension (2^31 - 1 along x, 65,535 along y), a ranking tile whose row count and strip
// summaries fit their 32-bit indices, and workspace sections that are aligned, ascending and inside the total.
int check_build_plan(const BuildPlan& P) {
    constexpr size_t kGridX = 0x7FFFFFFFull, kGridY = 65535;
    auto grid_ok = [&](size_t items, size_t per_block, const char* what) -> int {
        const size_t blocks = (items + per_block - 1) / per_block;
        if (blocks > kGridX) return fail(IVFPQ_EUNSUPPORTED, "%s would need %zu workgroups (limit %zu)", what, blocks, kGridX);
        return IVFPQ_OK;
    };
    const size_t d = (size_t)P.d, n = (size_t)P.n, n_ct = (size_t)P.n_ct, n_pt = (size_t)P.n_pt;
    if (int s = grid_ok(n_ct * d, 256, "gathering the cluster training rows")) return s;
    if (int s = grid_ok(n_pt * d, 256, "the residuals of the PQ training rows")) return s;
    if (int s = grid_ok(P.n_group, 256, "grouping rows by label")) return s;
    if (int s = grid_ok(n, 256, "encoding the rows")) return s;
    if (int s = grid_ok(P.k_group, 1, "sorting the groups")) return s;
    if (P.tile_rows < 1 || P.tile_rows > ((size_t)2 << 20))
        return fail(IVFPQ_EUNSUPPORTED, "internal: ranking tile of %zu rows (1 ... 2^21)", P.tile_rows);
    for (int k : {P.n_lists, P.ksub}) {
        // ranking GEMM: tiles of 128 x 128 (or 64 x 64): centres along x, rows along y
        const size_t gy = (P.tile_rows + 63) / 64, gx = ((size_t)k + 63) / 64;
        if (gy > kGridY) return fail(IVFPQ_EUNSUPPORTED, "internal: ranking tile of %zu rows needs %zu grid rows (limit %zu)", P.tile_rows, gy, kGridY);
        if (gx > kGridX) return fail(IVFPQ_EUNSUPPORTED, "%d centres need %zu grid columns", k, gx);
        if (int s = grid_ok(split_rows_padded(P.tile_rows) * (size_t)(coarse_padded_dim(P.d) / 8), 256, "splitting a tile of rows into bf16 halves")) return s;
    }
    const size_t strips = ((size_t)P.n_lists + 31) / 32;
    if (P.use_strips && P.tile_rows * strips >= ((size_t)1 << 32))
        return fail(IVFPQ_EUNSUPPORTED, "internal: %zu strip summaries per tile (limit 2^32)", P.tile_rows * strips);
    const size_t sections[] = {P.Xt, P.A, P.S, P.split, P.cnorm, P.cmax, P.C, P.labels_t, P.labels_all, P.order, P.tmp, P.counts,
                               P.cursor, P.offsets, P.ct_rows, P.pt_rows, P.init_rows, P.Rt, P.pq_labels, P.codebooks, P.codes};
    size_t prev = 0;
    for (size_t off : sections) {
        if (off % kAlign != 0 || off < prev || off > P.total)
            return fail(IVFPQ_EUNSUPPORTED, "internal: workspace section at %zu (previous %zu, total %zu)", off, prev, P.total);
        prev = off;
    }
    return IVFPQ_OK;
}

int fill_u32(uint32_t* p, size_t n, uint32_t v, hipStream_t st) {
    if (n == 0) return IVFPQ_OK;
    hipLaunchKernelGGL(fill_u32_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, st, p, n, v);
    HIP_TRY(hipGetLastError());
    return IVFPQ_OK;
}

// labels[i] = nearest centre of X[i], for n_rows rows
int assign_rows_device(const BuildPlan& P, unsigned char* ws, const float* X, size_t n_rows, const float* C, int k,
                       int32_t* labels, hipStream_t st) {
    float* cnorm = (float*)(ws + P.cnorm);
    uint32_t* cmax = (uint32_t*)(ws + P.cmax);
    uint32_t* A = (uint32_t*)(ws + P.A);
    StripSummary* S = (StripSummary*)(ws + P.S);
    if (int s = fill_u32(cmax, 1, 0u, st)) return s;
    hipLaunchKernelGGL(centre_norms_kernel, dim3(blocks_for((size_t)k, 4)), dim3(256), 0, st, C, k, P.d, cnorm, cmax);
    HIP_TRY(hipGetLastError());
    for (size_t r0 = 0; r0 < n_rows; r0 += P.tile_rows) {
        const int tr = (int)std::min(P.tile_rows, n_rows - r0);
        if (int s = launch_coarse(X + r0 * P.d, C, cnorm, tr, k, P.d, A, P.use_strips ? S : nullptr, ws + P.split, st)) return s;
        if (P.use_strips)
            hipLaunchKernelGGL(nearest_strips_kernel, dim3(blocks_for((size_t)tr, 64)), dim3(256), 0, st, (const StripSummary*)S,
                               coarse_strip_width(tr, k), X + r0 * P.d, C, cmax, tr, k, P.d, labels + r0);
        else
            hipLaunchKernelGGL(nearest_kernel, dim3(blocks_for((size_t)tr, 4)), dim3(256), 0, st, A, X + r0 * P.d, C, cmax, tr,
                               k, P.d, labels + r0);
        HIP_TRY(hipGetLastError());
    }
    return IVFPQ_OK;
}

// order = items grouped by label (ascending inside a group), offsets = group boundaries
int group_by_label(const BuildPlan& P, unsigned char* ws, const int32_t* labels, size_t n_items, int k, hipStream_t st) {
    uint32_t* counts = (uint32_t*)(ws + P.counts);
    uint32_t* cursor = (uint32_t*)(ws + P.cursor);
    int64_t* offsets = (int64_t*)(ws + P.offsets);
    uint32_t* order = (uint32_t*)(ws + P.order);
    uint32_t* tmp = (uint32_t*)(ws + P.tmp);
    if (int s = fill_u32(counts, (size_t)k, 0u, st)) return s;
    if (int s = fill_u32(cursor, (size_t)k, 0u, st)) return s;
    if (n_items > 0) {
        hipLaunchKernelGGL(count_labels_kernel, dim3(blocks_for(n_items, 256)), dim3(256), 0, st, labels, n_items, counts);
        HIP_TRY(hipGetLastError());
    }
    hipLaunchKernelGGL(offsets_kernel, dim3(1), dim3(1024), 0, st, counts, k, offsets);
    HIP_TRY(hipGetLastError());
    if (n_items > 0) {
        hipLaunchKernelGGL(scatter_rows_kernel, dim3(blocks_for(n_items, 256)), dim3(256), 0, st, labels, n_items, offsets,
                           cursor, order);
        HIP_TRY(hipGetLastError());
        hipLaunchKernelGGL(sort_groups_kernel, dim3((unsigned)k), dim3(256), 0, st, order, tmp, offsets);
        HIP_TRY(hipGetLastError());
    }
    return IVFPQ_OK;
}

int launch_pq_codes(const BuildPlan& P, const float* X, const uint32_t* order, const int32_t* labels, const float* C,
                    const float* codebooks, size_t n_pos, int32_t* train_labels, uint32_t* codes32, hipStream_t st) {
    if (n_pos == 0) return IVFPQ_OK;
    const int spw = sub_spaces_per_group(P.pq_bits);
    const size_t lds = (size_t)spw * P.ksub * P.m * 4;
    dim3 grid(blocks_for(n_pos, 256), (unsigned)(P.pq_dim / spw));
    auto go = [&](auto kernel) -> int {
        if (int s = allow_full_lds(kernel)) return s;
        hipLaunchKernelGGL(kernel, grid, dim3(256), lds, st, X, order, labels, C, codebooks, n_pos, P.d, P.pq_dim, P.m,
                           train_labels, codes32);
        HIP_TRY(hipGetLastError());
        return IVFPQ_OK;
    };
    switch (P.pq_bits) {
        case 8: return go(pq_codes_kernel<8>);
        case 7: return go(pq_codes_kernel<7>);
        case 6: return go(pq_codes_kernel<6>);
        case 5: return go(pq_codes_kernel<5>);
        default: return go(pq_codes_kernel<4>);
    }
}

int check_rows(const int64_t* rows, int64_t count, int64_t bound, const char* what) {
    for (int64_t i = 0; i < count; ++i)
        if (rows[i] < 0 || rows[i] >= bound)
            return fail(IVFPQ_EINVAL, "%s[%lld] = %lld outside [0, %lld)", what, (long long)i, (long long)rows[i], (long long)bound);
    return IVFPQ_OK;
}

int check_build_args(int64_t n, int32_t d, int32_t n_lists, int32_t pq_dim, int32_t pq_bits, int32_t kmeans_iters) {
    if (int st = check_shape(n, d, n_lists, pq_dim, pq_bits)) return st;
    if (n < 1 || n_lists > n) return fail(IVFPQ_EINVAL, "need 1 <= n_lists <= n (n=%lld, n_lists=%d)", (long long)n, n_lists);
    if (kmeans_iters < 0) return fail(IVFPQ_EINVAL, "kmeans_iters=%d", kmeans_iters);
    if (n >= ((int64_t)1 << 31)) return fail(IVFPQ_EUNSUPPORTED, "the device builder handles n < 2^31 rows (n=%lld)", (long long)n);
    const size_t lds = (size_t)sub_spaces_per_group(pq_bits) * ((size_t)1 << pq_bits) * (size_t)(d / pq_dim) * 4;
    if (lds > kLdsBytes)
        return fail(IVFPQ_EUNSUPPORTED, "codebooks of one code group need %zu bytes of LDS (limit %zu)", lds, kLdsBytes);
    return IVFPQ_OK;
}

}  // namespace

extern "C" {

size_t ivfpq_build_device_workspace_bytes(int64_t n, int32_t d, int32_t n_lists, int32_t pq_dim, int32_t pq_bits,
                                          int64_t n_coarse_train, int64_t n_pq_train) {
    if (check_build_args(n, d, n_lists, pq_dim, pq_bits, 0) != IVFPQ_OK) return 0;
    if (n_coarse_train <= 0) n_coarse_train = std::min<int64_t>(n, (int64_t)256 * n_lists);
    if (n_pq_train <= 0) n_pq_train = std::min<int64_t>(n, 262144);
    if ((__int128)n_pq_train * pq_dim >= ((__int128)1 << 32)) { set_error("n_pq_train * pq_dim must stay below 2^32"); return 0; }
    const BuildPlan P = make_build_plan(n, d, n_lists, pq_dim, pq_bits, n_coarse_train, n_pq_train);
    if (check_build_plan(P) != IVFPQ_OK) return 0;
    return P.total;
}

int ivfpq_assign_device(const float* d_rows, int64_t n_rows, int32_t d, const float* d_centres, int32_t n_centres,
                        int32_t* d_labels, void* d_workspace, size_t workspace_bytes, void* hip_stream) {
    if (!d_rows || !d_centres || !d_labels) return fail(IVFPQ_EINVAL, "ivfpq_assign_device: null pointer");
    if (n_rows < 0 || d < 1 || n_centres < 1) return fail(IVFPQ_EINVAL, "ivfpq_assign_device: bad shape");
    if (n_rows == 0) return IVFPQ_OK;
    BuildPlan P{};
    P.d = d;
    size_t at = 0;
    plan_nearest(P, (size_t)n_rows, n_centres, d, [&](size_t bytes) { size_t o = at; at = align_up(at + bytes); return o; });
    if (!d_workspace || workspace_bytes < at)
        return fail(IVFPQ_ENOSPACE, "workspace of %zu bytes given, %zu needed", workspace_bytes, at);
    return assign_rows_device(P, (unsigned char*)d_workspace, d_rows, (size_t)n_rows, d_centres, n_centres, d_labels,
                              (hipStream_t)hip_stream);
}

size_t ivfpq_assign_device_workspace_bytes(int64_t n_rows, int32_t d, int32_t n_centres) {
    if (n_rows < 0 || d < 1 || n_centres < 1) { set_error("ivfpq_assign_device_workspace_bytes: bad shape"); return 0; }
    BuildPlan P{};
    size_t at = 0;
    plan_nearest(P, (size_t)n_rows, n_centres, d, [&](size_t bytes) { size_t o = at; at = align_up(at + bytes); return o; });
    return at;
}

}  // extern "C"

namespace {
int build_device_impl(const float* d_data, int64_t n, int32_t d, int32_t n_lists, int32_t pq_dim, int32_t pq_bits,
                       int32_t kmeans_iters, const int64_t* coarse_train_rows, int64_t n_coarse_train,
                       const int64_t* coarse_init_rows, const int64_t* pq_train_rows, int64_t n_pq_train,
                       const int64_t* pq_init_rows, uint64_t seed, void* d_workspace, size_t workspace_bytes,
                       void* hip_stream, ivfpq_index_t** out) {
    if (!d_data || !out) return fail(IVFPQ_EINVAL, "ivfpq_build_device: null pointer");
    *out = nullptr;
    if (int s = check_build_args(n, d, n_lists, pq_dim, pq_bits, kmeans_iters)) return s;
    const int m = d / pq_dim, ksub = 1 << pq_bits, cb = pq_dim * pq_bits / 8;
    hipStream_t st = (hipStream_t)hip_stream;

    // the rows of the two training sets and of the k-means starts: the caller's, or drawn from the seed
    SplitMix64 rng(seed ^ 0x2301066720230117ull);
    std::vector<int64_t> ct_rows, ct_init, pt_rows, pt_init;
    if (coarse_train_rows) {
        if (n_coarse_train < 1) return fail(IVFPQ_EINVAL, "n_coarse_train=%lld", (long long)n_coarse_train);
        ct_rows.assign(coarse_train_rows, coarse_train_rows + n_coarse_train);
        if (int s = check_rows(ct_rows.data(), n_coarse_train, n, "coarse_train_rows")) return s;
    } else {
        ct_rows = stride_rows(n, (int64_t)256 * n_lists);
    }
    const int64_t n_ct = (int64_t)ct_rows.size();
    if (coarse_init_rows) {
        ct_init.assign(coarse_init_rows, coarse_init_rows + n_lists);
        if (int s = check_rows(ct_init.data(), n_lists, n_ct, "coarse_init_rows")) return s;
    } else {
        ct_init = draw_rows(rng, n_ct, n_lists);
    }
    if (pq_train_rows) {
        if (n_pq_train < 1) return fail(IVFPQ_EINVAL, "n_pq_train=%lld", (long long)n_pq_train);
        pt_rows.assign(pq_train_rows, pq_train_rows + n_pq_train);
        if (int s = check_rows(pt_rows.data(), n_pq_train, n, "pq_train_rows")) return s;
    } else {
        pt_rows = stride_rows(n, 262144);
    }
    const int64_t n_pt = (int64_t)pt_rows.size();
    if ((__int128)n_pt * pq_dim >= ((__int128)1 << 32))
        return fail(IVFPQ_EUNSUPPORTED, "n_pq_train * pq_dim must stay below 2^32");
    if (pq_init_rows) {
        pt_init.assign(pq_init_rows, pq_init_rows + (size_t)pq_dim * ksub);
        if (int s = check_rows(pt_init.data(), (int64_t)pq_dim * ksub, n_pt, "pq_init_rows")) return s;
    } else {
        for (int j = 0; j < pq_dim; ++j) {
            std::vector<int64_t> r = draw_rows(rng, n_pt, ksub);
            pt_init.insert(pt_init.end(), r.begin(), r.end());
        }
    }

    const BuildPlan P = make_build_plan(n, d, n_lists, pq_dim, pq_bits, n_ct, n_pt);
    if (int s = check_build_plan(P)) return s;
    if (!d_workspace || workspace_bytes < P.total)
        return fail(IVFPQ_ENOSPACE, "workspace of %zu bytes given, %zu needed", workspace_bytes, P.total);
    if (((uintptr_t)d_workspace % kAlign) != 0) return fail(IVFPQ_EINVAL, "workspace must be %zu-byte aligned", kAlign);
    unsigned char* ws = (unsigned char*)d_workspace;
    float* Xt = (float*)(ws + P.Xt);
    float* C = (float*)(ws + P.C);
    int32_t* labels_t = (int32_t*)(ws + P.labels_t);
    int32_t* labels_all = (int32_t*)(ws + P.labels_all);
    uint32_t* order = (uint32_t*)(ws + P.order);
    int64_t* offsets = (int64_t*)(ws + P.offsets);
    int64_t* d_ct_rows = (int64_t*)(ws + P.ct_rows);
    int64_t* d_pt_rows = (int64_t*)(ws + P.pt_rows);
    int64_t* d_init = (int64_t*)(ws + P.init_rows);
    float* Rt = (float*)(ws + P.Rt);
    int32_t* pq_labels = (int32_t*)(ws + P.pq_labels);
    float* codebooks = (float*)(ws + P.codebooks);
    uint32_t* codes32 = (uint32_t*)(ws + P.codes);

    // (1) clusters: Lloyd iterations on the training rows
    HIP_TRY(hipMemcpyAsync(d_ct_rows, ct_rows.data(), (size_t)n_ct * 8, hipMemcpyHostToDevice, st));
    HIP_TRY(hipMemcpyAsync(d_init, ct_init.data(), (size_t)n_lists * 8, hipMemcpyHostToDevice, st));
    hipLaunchKernelGGL(gather_rows_kernel, dim3(blocks_for((size_t)n_ct * d, 256)), dim3(256), 0, st, d_data, d_ct_rows, n_ct, d, Xt);
    HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(gather_rows_kernel, dim3(blocks_for((size_t)n_lists * d, 256)), dim3(256), 0, st, Xt, d_init,
                       (int64_t)n_lists, d, C);
    HIP_TRY(hipGetLastError());
    for (int it = 0; it < kmeans_iters; ++it) {
        if (int s = assign_rows_device(P, ws, Xt, (size_t)n_ct, C, n_lists, labels_t, st)) return s;
        if (int s = group_by_label(P, ws, labels_t, (size_t)n_ct, n_lists, st)) return s;
        hipLaunchKernelGGL(update_centres_kernel, dim3(blocks_for((size_t)n_lists, 4)), dim3(256), 0, st, Xt, (size_t)d, 1, d,
                           order, offsets, n_lists, C);
        HIP_TRY(hipGetLastError());
    }
    // membership of every row
    if (int s = assign_rows_device(P, ws, d_data, (size_t)n, C, n_lists, labels_all, st)) return s;

    // (2) + (3) residuals of the PQ training rows, one Lloyd k-means per sub-space (all sub-spaces at once)
    HIP_TRY(hipMemcpyAsync(d_pt_rows, pt_rows.data(), (size_t)n_pt * 8, hipMemcpyHostToDevice, st));
    HIP_TRY(hipMemcpyAsync(d_init, pt_init.data(), (size_t)pq_dim * ksub * 8, hipMemcpyHostToDevice, st));
    hipLaunchKernelGGL(residual_rows_kernel, dim3(blocks_for((size_t)n_pt * d, 256)), dim3(256), 0, st, d_data, d_pt_rows, n_pt,
                       labels_all, C, d, Rt);
    HIP_TRY(hipGetLastError());
    hipLaunchKernelGGL(init_codebooks_kernel, dim3(blocks_for((size_t)pq_dim * ksub * m, 256)), dim3(256), 0, st, Rt, d_init,
                       pq_dim, ksub, m, d, codebooks);
    HIP_TRY(hipGetLastError());
    for (int it = 0; it < kmeans_iters; ++it) {
        if (int s = launch_pq_codes(P, Rt, nullptr, nullptr, nullptr, codebooks, (size_t)n_pt, pq_labels, nullptr, st)) return s;
        if (int s = group_by_label(P, ws, pq_labels, (size_t)n_pt * pq_dim, pq_dim * ksub, st)) return s;
        hipLaunchKernelGGL(update_centres_kernel, dim3(blocks_for((size_t)pq_dim * ksub, 4)), dim3(256), 0, st, Rt, (size_t)d,
                           pq_dim, m, order, offsets, pq_dim * ksub, codebooks);
        HIP_TRY(hipGetLastError());
    }

    // (4) the lists (rows grouped by cluster, ascending id inside a list) and the packed codes in list order
    if (int s = group_by_label(P, ws, labels_all, (size_t)n, n_lists, st)) return s;
    if (int s = launch_pq_codes(P, d_data, order, labels_all, C, codebooks, (size_t)n, nullptr, codes32, st)) return s;

    std::unique_ptr<ivfpq_index> owner(new ivfpq_index);
    ivfpq_index* idx = owner.get();
    idx->n = n; idx->d = d; idx->n_lists = n_lists; idx->pq_dim = pq_dim; idx->pq_bits = pq_bits;
    idx->centroids.resize((size_t)n_lists * d);
    idx->codebooks.resize((size_t)pq_dim * ksub * m);
    idx->list_offsets.resize((size_t)n_lists + 1);
    idx->codes.resize((size_t)n * cb);
    idx->ids.resize((size_t)n);
    std::vector<uint32_t> order_h((size_t)n);
    auto copy_out = [&]() -> int {
        HIP_TRY(hipMemcpyAsync(idx->centroids.data(), C, idx->centroids.size() * 4, hipMemcpyDeviceToHost, st));
        HIP_TRY(hipMemcpyAsync(idx->codebooks.data(), codebooks, idx->codebooks.size() * 4, hipMemcpyDeviceToHost, st));
        HIP_TRY(hipMemcpyAsync(idx->list_offsets.data(), offsets, idx->list_offsets.size() * 8, hipMemcpyDeviceToHost, st));
        HIP_TRY(hipMemcpyAsync(idx->codes.data(), codes32, idx->codes.size(), hipMemcpyDeviceToHost, st));
        HIP_TRY(hipMemcpyAsync(order_h.data(), order, order_h.size() * 4, hipMemcpyDeviceToHost, st));
        HIP_TRY(hipStreamSynchronize(st));
        return IVFPQ_OK;
    };
    if (int s = copy_out()) return s;
    for (int64_t i = 0; i < n; ++i) idx->ids[(size_t)i] = (int64_t)order_h[(size_t)i];
    finish_import(idx);
    *out = owner.release();
    return IVFPQ_OK;
}
}  // namespace

extern "C" {

int ivfpq_build_device(const float* d_data, int64_t n, int32_t d, int32_t n_lists, int32_t pq_dim, int32_t pq_bits,
                       int32_t kmeans_iters, const int64_t* coarse_train_rows, int64_t n_coarse_train,
                       const int64_t* coarse_init_rows, const int64_t* pq_train_rows, int64_t n_pq_train,
                       const int64_t* pq_init_rows, uint64_t seed, void* d_workspace, size_t workspace_bytes,
                       void* hip_stream, ivfpq_index_t** out) {
    return guarded("ivfpq_build_device", [&] {
        return build_device_impl(d_data, n, d, n_lists, pq_dim, pq_bits, kmeans_iters, coarse_train_rows, n_coarse_train,
                                 coarse_init_rows, pq_train_rows, n_pq_train, pq_init_rows, seed, d_workspace,
                                 workspace_bytes, hip_stream, out);
    });
}

}  // extern "C"
