// Device code shared by the search kernels and the index builder: HIP error macro, small constants,
// order-preserving float keys and the MFMA ranking GEMMs |c|^2 - 2 x.c (fp32, and bf16 on split operands)
// with their epilogue (all keys, or per-strip summaries) and the bound of their error.
// Included by .hip translation units only; everything has internal linkage.
#pragma once

#include <hip/hip_runtime.h>

#include <mutex>
#include <type_traits>
#include <utility>
#include <vector>

#include "ivfpq_internal.hpp"

#define HIP_TRY(expr)                                                                               \
    do {                                                                                            \
        hipError_t e_ = (expr);                                                                     \
        if (e_ != hipSuccess)                                                                       \
            return ivfpq::fail(IVFPQ_EHIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
    } while (0)

namespace {

using ivfpq::fail;

constexpr int kWave = 64;
constexpr size_t kLdsBytes = 160 * 1024;       // LDS of one gfx950 compute unit
constexpr size_t kAlign = 256;

inline size_t align_up(size_t x, size_t a = kAlign) { return (x + a - 1) / a * a; }

// Lets `kernel` use dynamic LDS up to the whole compute unit's; done once per kernel and device, so
// that later launches make no call besides the launch itself (a caller may be capturing a HIP graph).
inline int allow_full_lds_ptr(const void* kernel) {
    static std::mutex mu;
    static std::vector<std::pair<const void*, int>> done;
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lock(mu);
    for (const auto& e : done)
        if (e.first == kernel && e.second == dev) return IVFPQ_OK;
    HIP_TRY(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes));
    done.emplace_back(kernel, dev);
    return IVFPQ_OK;
}
template <class Kernel>
int allow_full_lds(Kernel kernel) { return allow_full_lds_ptr(reinterpret_cast<const void*>(kernel)); }

// ================================================================================================
// Ranking values on the matrix cores (search step 1a; the assignment step of the index build).
// For ranking the clusters of one query |q - c|^2 can be replaced by a(q, c) = |c|^2 - 2 q.c (the
// |q|^2 term is common).  The dot products are one GEMM: a tile of 64 queries x 64 clusters per
// 256-thread workgroup on v_mfma_f32_32x32x2_f32 for small problems, 128 x 128 on the bf16 instruction
// with split operands for large ones, operands staged through LDS in slices of 16 components.  The
// expanded form cancels, so these values only SHORT-LIST clusters: the kernels that consume them bound the
// error of a() rigorously (rank_error_bound) and recompute the distances of everything inside that bound
// in direct form, so their decisions are exact.
// Values are stored as order-preserving unsigned keys (a() can be negative).
// ================================================================================================
constexpr int CK = 16;   // components per LDS slice
typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ inline uint32_t ordered_key(float f) {          // monotone map float -> uint32
    const uint32_t b = __float_as_uint(f);
    return b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}
__device__ inline float ordered_key_value(uint32_t key) {
    return __uint_as_float(key ^ ((key >> 31) ? 0x80000000u : 0xFFFFFFFFu));
}

// The three smallest, over the 32 lanes of a half-wave, of 16 values per lane (each lane brings its own
// three smallest, lo1 <= lo2 <= lo3), folded so that every exchange carries only what the receiver keeps: the lane
// whose index bit is set keeps the upper half of the remaining values and hands the lower half to its
// partner (8, 4, 2, 1 exchanges, then one more between neighbours).  Lane l of the half-wave ends with
// the result for value l / 2.  The partners are the lane 16 further (LDS swizzle) and the lanes the
// data-parallel permutes reach inside a row of 16: mirrored row (bit 3 differs), mirrored half-row
// (bit 2), quad neighbours (bits 1 and 0).
template <int CTRL>
__device__ inline uint32_t dpp_take(uint32_t x) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, CTRL, 0xF, 0xF, false);
}
__device__ inline uint32_t swizzle_take16(uint32_t x) { return (uint32_t)__builtin_amdgcn_ds_swizzle((int)x, 0x401F); }
__device__ inline uint32_t umin32(uint32_t a, uint32_t b) { return a < b ? a : b; }
__device__ inline uint32_t umax32(uint32_t a, uint32_t b) { return a < b ? b : a; }
struct Low3 { uint32_t m1, m2, m3; };             // the three smallest, ascending
__device__ inline uint32_t umin3(uint32_t a, uint32_t b, uint32_t c) { return umin32(umin32(a, b), c); }
// two sorted triples -> the three smallest of the six
__device__ inline Low3 merge_low3(Low3 a, Low3 b) {
    const uint32_t x = umax32(a.m1, b.m1), y = umin32(a.m2, b.m2);
    return Low3{umin32(a.m1, b.m1), umin32(x, y), umin3(umax32(x, y), a.m3, b.m3)};
}
template <int CTRL>
__device__ inline Low3 dpp_take3(Low3 v) { return Low3{dpp_take<CTRL>(v.m1), dpp_take<CTRL>(v.m2), dpp_take<CTRL>(v.m3)}; }
__device__ inline Low3 half_wave_low3x16(const uint32_t (&lo1)[16], const uint32_t (&lo2)[16], const uint32_t (&lo3)[16], int l32) {
    const bool b4 = (l32 & 16) != 0, b3 = (l32 & 8) != 0, b2 = (l32 & 4) != 0, b1 = (l32 & 2) != 0;
    Low3 a[8], b[4], c[2];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const Low3 keep{b4 ? lo1[t + 8] : lo1[t], b4 ? lo2[t + 8] : lo2[t], b4 ? lo3[t + 8] : lo3[t]};
        const Low3 give{b4 ? lo1[t] : lo1[t + 8], b4 ? lo2[t] : lo2[t + 8], b4 ? lo3[t] : lo3[t + 8]};
        a[t] = merge_low3(keep, Low3{swizzle_take16(give.m1), swizzle_take16(give.m2), swizzle_take16(give.m3)});   // from lane ^ 16
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const Low3 keep = b3 ? a[t + 4] : a[t], give = b3 ? a[t] : a[t + 4];
        b[t] = merge_low3(keep, dpp_take3<0x140>(give));       // row_mirror
    }
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const Low3 keep = b2 ? b[t + 2] : b[t], give = b2 ? b[t] : b[t + 2];
        c[t] = merge_low3(keep, dpp_take3<0x141>(give));       // row_half_mirror
    }
    const Low3 keep = b1 ? c[1] : c[0], give = b1 ? c[0] : c[1];
    const Low3 x = merge_low3(keep, dpp_take3<0x4E>(give));    // quad_perm [2,3,0,1]
    return merge_low3(x, dpp_take3<0xB1>(x));                  // quad_perm [1,0,3,2]
}

// What the ranking kernels store per (row, strip) when they do not store every key: the three smallest
// tagged keys of the strip, ascending (.w unused).
typedef uint4 StripSummary;

// Epilogue of the ranking kernels: turns the accumulated dot products of one workgroup tile (4 waves
// 2 x 2, each WB x WB blocks of 32 x 32) into order-preserving keys of a = |c|^2 - 2 q.c.
// Either all keys are stored, A[nq][n_lists] (S null), or only a summary of every strip of 32*WB
// consecutive clusters (the ones a wave covers), S[n_strips][nq] (strip-major, so that a wave stores the
// summaries of its 64 queries contiguously): the three smallest keys of the strip, each with its low six
// bits replaced by the cluster's position in the strip.  Clearing those bits lowers a key by at most 63
// units in the last place; a consumer takes (x & ~63) as a lower and (x | 63) as an upper bound of the key.  All-ones
// means "no such cluster".  stage: 1024 words of LDS that no wave still reads.
// Accumulator layout of a 32x32 block: register v of lane L holds row 8*(v/4) + 4*(L/32) + v%4, column L%32.
template <int WB>
__device__ __forceinline__ void rank_store(const floatx16 (&acc)[WB][WB], int q0, int l0, int nq, int n_lists,
                                           const float* __restrict__ centroid_norms, uint32_t* __restrict__ A,
                                           StripSummary* __restrict__ S, StripSummary* stage) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1, half = lane >> 5, l32 = lane & 31;
    if (!S) {
#pragma unroll
        for (int i = 0; i < WB; ++i)
#pragma unroll
            for (int j = 0; j < WB; ++j) {
                const int li = l0 + (wc * WB + j) * 32 + l32;
                if (li >= n_lists) continue;
                const float cn = centroid_norms[li];
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int qi = q0 + (wr * WB + i) * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                    if (qi < nq) A[(size_t)qi * n_lists + li] = ordered_key(__builtin_fmaf(-2.f, acc[i][j][v], cn));
                }
            }
        return;
    }
    const int n_strips = (n_lists + 32 * WB - 1) / (32 * WB);
    const int strip = blockIdx.x * 2 + wc;
#pragma unroll
    for (int i = 0; i < WB; ++i) {
        uint32_t lo1[16], lo2[16], lo3[16];       // per row: the smallest tagged keys among this lane's clusters
#pragma unroll
        for (int v = 0; v < 16; ++v) { lo1[v] = 0xFFFFFFFFu; lo2[v] = 0xFFFFFFFFu; lo3[v] = 0xFFFFFFFFu; }
#pragma unroll
        for (int j = 0; j < WB; ++j) {
            const int li = l0 + (wc * WB + j) * 32 + l32;
            const bool col_ok = li < n_lists;
            const float cn = col_ok ? centroid_norms[li] : 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const uint32_t key = ordered_key(__builtin_fmaf(-2.f, acc[i][j][v], cn));
                const uint32_t tagged = col_ok ? ((key & ~63u) | (uint32_t)(j * 32 + l32)) : 0xFFFFFFFFu;
                lo3[v] = umin32(lo3[v], umax32(lo2[v], tagged));
                lo2[v] = umin32(lo2[v], umax32(lo1[v], tagged));
                lo1[v] = umin32(lo1[v], tagged);
            }
        }
        const Low3 mine = half_wave_low3x16(lo1, lo2, lo3, l32);
        const int v = l32 >> 1;
        stage[wave * 64 + i * 32 + 8 * (v / 4) + 4 * half + (v % 4)] = make_uint4(mine.m1, mine.m2, mine.m3, 0xFFFFFFFFu);
    }
    __builtin_amdgcn_wave_barrier();              // the wave's own LDS writes above are read back below
    const int qi = q0 + wr * WB * 32 + lane;
    if (lane < WB * 32 && qi < nq && strip < n_strips) S[(size_t)strip * nq + qi] = stage[wave * 64 + lane];
}

// WB = 32x32 output blocks per wave and axis; the 4 waves sit 2 x 2, so the tile edge is 64 * WB.
// Four waves per SIMD (128 registers each, accumulators included) keep the MFMA pipe fed while other
// waves wait at the slice barriers: measured 9-12 % faster than the three the compiler picks unasked.
template <int WB>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4)))
coarse_rank_kernel(const float* __restrict__ queries, const float* __restrict__ centroids,
                   const float* __restrict__ centroid_norms, int nq, int n_lists, int d,
                   uint32_t* __restrict__ A, StripSummary* __restrict__ S) {
    constexpr int CT = 64 * WB;          // tile edge
    constexpr int RT = 4 * WB;           // components a thread loads per tile row and slice
    __shared__ __attribute__((aligned(16))) float qs[CK][CT + 4];      // also the epilogue's staging area (16-byte stores)
    __shared__ float cs[CK][CT + 4];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int q0 = blockIdx.y * CT, l0 = blockIdx.x * CT;
    floatx16 acc[WB][WB];
#pragma unroll
    for (int i = 0; i < WB; ++i)
#pragma unroll
        for (int j = 0; j < WB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    constexpr int TPR = CK / RT;              // threads per tile row when loading
    const int lr = tid / TPR;                 // row of the tile this thread loads
    const int lk = (tid % TPR) * RT;          // first of its RT components
    const bool vec_ok = (d & 3) == 0;
    const int half = lane >> 5, l32 = lane & 31;
    const int qi = q0 + lr, li = l0 + lr;
    float qv[RT], cv[RT];
    // global -> registers for the slice starting at component k0 (zero beyond the matrix edges)
    auto fetch = [&](int k0) {
        if (vec_ok && k0 + lk + RT <= d) {
#pragma unroll
            for (int v = 0; v < WB; ++v) {
                float4 x = make_float4(0.f, 0.f, 0.f, 0.f), y = x;
                if (qi < nq) x = reinterpret_cast<const float4*>(queries + (size_t)qi * d + k0 + lk)[v];
                if (li < n_lists) y = reinterpret_cast<const float4*>(centroids + (size_t)li * d + k0 + lk)[v];
                qv[4 * v] = x.x; qv[4 * v + 1] = x.y; qv[4 * v + 2] = x.z; qv[4 * v + 3] = x.w;
                cv[4 * v] = y.x; cv[4 * v + 1] = y.y; cv[4 * v + 2] = y.z; cv[4 * v + 3] = y.w;
            }
        } else {
#pragma unroll
            for (int u = 0; u < RT; ++u) {
                const int t = k0 + lk + u;
                qv[u] = (qi < nq && t < d) ? queries[(size_t)qi * d + t] : 0.f;
                cv[u] = (li < n_lists && t < d) ? centroids[(size_t)li * d + t] : 0.f;
            }
        }
    };
    fetch(0);
    for (int k0 = 0; k0 < d; k0 += CK) {
#pragma unroll
        for (int u = 0; u < RT; ++u) { qs[lk + u][lr] = qv[u]; cs[lk + u][lr] = cv[u]; }
        __syncthreads();
        if (k0 + CK < d) fetch(k0 + CK);       // the next slice travels while this one is multiplied
        // one MFMA consumes two components: lanes 0-31 feed component kk, lanes 32-63 component kk+1
#pragma unroll
        for (int kk = 0; kk < CK; kk += 2) {
            float av[WB], bv[WB];
#pragma unroll
            for (int i = 0; i < WB; ++i) av[i] = qs[kk + half][(wr * WB + i) * 32 + l32];
#pragma unroll
            for (int j = 0; j < WB; ++j) bv[j] = cs[kk + half][(wc * WB + j) * 32 + l32];
#pragma unroll
            for (int i = 0; i < WB; ++i)
#pragma unroll
                for (int j = 0; j < WB; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }
    rank_store<WB>(acc, q0, l0, nq, n_lists, centroid_norms, A, S, reinterpret_cast<StripSummary*>(&qs[0][0]));
}

// ------------------------------------------------------------------------------------------------
// Large problems: the same dot products from bf16 matrix instructions, 16 times the fp32 rate.
// Every fp32 operand x is split once into hi = bf16(x) and lo = bf16(x - hi) (x - hi is exact in fp32,
// |x - hi - lo| <= 2^-16 |x|) and q.c is taken as qh.ch + qh.cl + ql.ch with v_mfma_f32_32x32x16_bf16
// (bf16 products are exact in fp32; the sums are fp32).  What is dropped - ql.cl and the two split
// remainders - is at most 3.02 * 2^-16 |q||c|, which rank_error_bound() carries, so the exactness
// argument of the consumers is unchanged.
// ------------------------------------------------------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
constexpr int BK = 16;        // components per LDS slice = one matrix instruction deep

__device__ inline uint32_t bf16_round(float f) {          // round to nearest even; Inf stays Inf, NaN stays NaN
    const uint32_t b = __float_as_uint(f);
    if ((b & 0x7F800000u) == 0x7F800000u) return (b >> 16) | ((b & 0xFFFFu) ? 0x40u : 0u);
    return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
}

// X[rows][d] fp32 -> hi, lo in bf16, laid out slice by slice: [dp / 16][rows_pad][16], rows_pad = rows rounded
// up to the tile edge of 128, so that the 128 rows x 16 components which a workgroup of the GEMM stages per
// step are 4 KiB of consecutive memory (row-major operands give it 32 bytes out of every row: a quarter of
// each cache line fetched, four times over).  Components d..dp-1 and rows beyond the matrix are zero.  One
// thread per 8 components.
__host__ __device__ inline size_t split_rows_padded(size_t rows) { return (rows + 127) / 128 * 128; }
__global__ void __launch_bounds__(256)
split_bf16_kernel(const float* __restrict__ X, size_t rows, size_t rows_pad, int d, int dp, uint16_t* __restrict__ hi, uint16_t* __restrict__ lo) {
    const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int per_row = dp / 8;
    const size_t row = t / per_row;
    const int k0 = (int)(t % per_row) * 8;
    if (row >= rows_pad) return;
    uint32_t h[8], l[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const float x = (row < rows && k0 + u < d) ? X[row * d + k0 + u] : 0.f;
        h[u] = bf16_round(x);
        const float rest = x - __uint_as_float(h[u] << 16);
        l[u] = (rest == rest) ? bf16_round(rest) : 0u;       // Inf - Inf: the hi part already carries it
    }
    uint4 H = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
    uint4 L = make_uint4(l[0] | (l[1] << 16), l[2] | (l[3] << 16), l[4] | (l[5] << 16), l[6] | (l[7] << 16));
    const size_t at = ((size_t)(k0 / BK) * rows_pad + row) * BK + (k0 % BK);
    *reinterpret_cast<uint4*>(hi + at) = H;
    *reinterpret_cast<uint4*>(lo + at) = L;
}

// Inserts x into the ascending triple (m1, m2, m3) of the smallest values seen: three instructions.
__device__ inline uint32_t umed3(uint32_t a, uint32_t b, uint32_t c) {
    uint32_t r;
    asm("v_med3_u32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
__device__ inline void low3_insert(Low3& m, uint32_t x) {
    m.m3 = umed3(m.m2, x, m.m3);
    m.m2 = umed3(m.m1, x, m.m2);
    m.m1 = umin32(m.m1, x);
}

// Staging of one operand slice in LDS for the bf16 kernel: 128 rows x 16 components = 32 bytes per row, no
// padding; the two 16-byte pieces of a row swap places in every second group of four rows, so that the
// 16-byte reads of eight consecutive rows (one piece each) cover all 32 banks.
__device__ inline int split_piece_at(int row, int piece) { return row * 16 + ((piece ^ ((row >> 2) & 1)) << 3); }   // in bf16

// 128 x 128 outputs per workgroup, 4 waves 2 x 2, each 2 x 2 blocks of v_mfma_f32_32x32x16_bf16; wave w stages
// operand array w (Qh, Ql, Ch, Cl) of a slice of 16 components.  Two LDS buffers, one barrier per slice: slice
// s + 1 is stored while slice s is multiplied, slice s + 2 travels in registers.
// STRIPS = false: rows of the accumulator blocks are queries, columns clusters; every key is stored
// (rank_store).  STRIPS = true: the matrix roles are swapped -- rows are clusters, columns queries -- so that a
// lane holds, for ONE query (its column), 32 of the 64 clusters of a strip in registers: the three smallest
// tagged keys of the strip come from an in-register insertion (three instructions per key) and a single
// exchange with the lane 32 further, instead of a fold across 32 lanes.
template <bool STRIPS>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4)))
coarse_rank_split_kernel(const uint16_t* __restrict__ Qh, const uint16_t* __restrict__ Ql,
                         const uint16_t* __restrict__ Ch, const uint16_t* __restrict__ Cl,
                         const float* __restrict__ centroid_norms, int nq, int n_lists, int dp,
                         uint32_t* __restrict__ A, StripSummary* __restrict__ S) {
    __shared__ __attribute__((aligned(16))) uint16_t tile[2][4][128 * BK];
    __shared__ __attribute__((aligned(16))) float cn_s[128];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave >> 1, wc = wave & 1, half = lane >> 5, l32 = lane & 31;
    // Workgroup b runs on XCD b % 8.  Every XCD owns one eighth of the query tiles, whose operands then stay in
    // its L2, and walks the cluster tiles in the outer loop, so that a cluster tile is fetched into that L2 once
    // per pass and used by all of the XCD's query tiles in turn (one query tile row after the other re-reads
    // every cluster tile from beyond the L2 instead).
    const int q_tiles = (nq + 127) / 128, per_xcd = (q_tiles + 7) / 8;
    const int rank = blockIdx.x >> 3, c_tile = rank / per_xcd, q_tile = (blockIdx.x & 7) + 8 * (rank % per_xcd);
    if (q_tile >= q_tiles) return;                 // the grid is padded to 8 x per_xcd query tiles
    const int q0 = q_tile * 128, l0 = c_tile * 128;
    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const uint16_t* src = wave == 0 ? Qh : (wave == 1 ? Ql : (wave == 2 ? Ch : Cl));
    const int row0 = wave < 2 ? q0 : l0, n_rows = wave < 2 ? nq : n_lists;
    if (STRIPS && tid < 128) cn_s[tid] = l0 + tid < n_lists ? centroid_norms[l0 + tid] : 0.f;   // read after the loop's barriers
    uint4 pre[4];
    // a slice of one operand array, 128 rows x 32 bytes, is 256 consecutive 16-byte pieces: four per lane
    const size_t rows_pad = split_rows_padded((size_t)n_rows);
    const uint16_t* src0 = src + (size_t)row0 * BK + lane * 8;
    auto fetch = [&](int slice) __attribute__((always_inline)) {
        const uint16_t* at = src0 + (size_t)slice * rows_pad * BK;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint4* pp = reinterpret_cast<const uint4*>(at + c * 512);
            pre[c] = make_uint4(pp->x, pp->y, pp->z, pp->w);
        }
    };
    auto stash = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int piece = c * 64 + lane;
            *reinterpret_cast<uint4*>(&tile[buf][wave][split_piece_at(piece >> 1, piece & 1)]) = pre[c];
        }
    };
    // the operand arrays of the accumulator's rows and columns
    constexpr int RH = STRIPS ? 2 : 0, RL = STRIPS ? 3 : 1, CH = STRIPS ? 0 : 2, CL = STRIPS ? 1 : 3;
    const int n_slices = dp / BK;
    fetch(0);
    stash(0);
    if (n_slices > 1) fetch(1);
    __syncthreads();
    for (int sl = 0; sl < n_slices; ++sl) {
        const int buf = sl & 1;
        if (sl + 1 < n_slices) stash(buf ^ 1);                 // its last readers passed the barrier that ended slice sl - 1
        if (sl + 2 < n_slices) fetch(sl + 2);
        // operand of lane L: row L % 32, components 8 * (L / 32) .. + 7
        bf16x8 ah[2], al[2], bh[2], bl[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int at = split_piece_at((wr * 2 + i) * 32 + l32, half);
            ah[i] = *reinterpret_cast<const bf16x8*>(&tile[buf][RH][at]);
            al[i] = *reinterpret_cast<const bf16x8*>(&tile[buf][RL][at]);
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int at = split_piece_at((wc * 2 + j) * 32 + l32, half);
            bh[j] = *reinterpret_cast<const bf16x8*>(&tile[buf][CH][at]);
            bl[j] = *reinterpret_cast<const bf16x8*>(&tile[buf][CL][at]);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[i], bh[j], acc[i][j], 0, 0, 0);
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bl[j], acc[i][j], 0, 0, 0);
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bh[j], acc[i][j], 0, 0, 0);
            }
        __syncthreads();
    }
    if constexpr (!STRIPS) {
        rank_store<2>(acc, q0, l0, nq, n_lists, centroid_norms, A, S, reinterpret_cast<StripSummary*>(&tile[0][0][0]));
    } else {
        // Register v of lane L of block (i, j): cluster l0 + 64 wr + 32 i + 8 (v / 4) + 4 (L / 32) + v % 4, query
        // q0 + 64 wc + 32 j + L % 32.  The tag of a key is the cluster's position in the wave's strip of 64.
        const int strip = c_tile * 2 + wr, n_strips = (n_lists + 63) / 64;
        const int n_valid = n_lists - (l0 + wr * 64);              // clusters of this strip that exist
        const float* cn = cn_s + wr * 64 + 4 * half;
        // the three smallest tagged keys among this lane's 32 clusters of query block j
        auto lane_low3 = [&](int j, auto partial) __attribute__((always_inline)) {
            Low3 m{0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu};
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const float4 c4 = *reinterpret_cast<const float4*>(cn + i * 32 + 8 * g);
                    const float cv[4] = {c4.x, c4.y, c4.z, c4.w};
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int pos = i * 32 + 8 * g + u;        // + 4 * half, added once by the caller
                        const uint32_t key = ordered_key(__builtin_fmaf(-2.f, acc[i][j][4 * g + u], cv[u]));
                        uint32_t tagged = (key & ~63u) | (uint32_t)pos;
                        if (decltype(partial)::value && pos + 4 * half >= n_valid) tagged = 0xFFFFFFFFu;
                        low3_insert(m, tagged);
                    }
                }
            return m;
        };
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            // only the last strip of all can be short of clusters
            Low3 m = n_valid >= 64 ? lane_low3(j, std::false_type{}) : lane_low3(j, std::true_type{});
            // all-ones stays all-ones; every other key of this lane gets the half-wave's bit of the position
            m.m1 |= 4u * half; m.m2 |= 4u * half; m.m3 |= 4u * half;
            const Low3 other{(uint32_t)__shfl_xor((int)m.m1, 32, kWave), (uint32_t)__shfl_xor((int)m.m2, 32, kWave),
                             (uint32_t)__shfl_xor((int)m.m3, 32, kWave)};
            m = merge_low3(m, other);
            const int qi = q0 + wc * 64 + j * 32 + l32;
            if (half == 0 && qi < nq && strip < n_strips)
                S[(size_t)strip * nq + qi] = make_uint4(m.m1, m.m2, m.m3, 0xFFFFFFFFu);
        }
    }
}

// |a_computed - a_exact| <= this, for either ranking kernel (qn = |q|^2, cmax = max |c|^2): the split
// remainders, 3.02 * 2^-16 |q||c| on the dot product, so 3.02 * 2^-16 (|q|^2 + |c|^2) on a; the fp32 sum
// of up to 3 d exact products in any order (3 d 2^-24 relative to the sum of their magnitudes, taken with
// a factor 4 of slack for whatever rounding the matrix unit applies); the rounding of |c|^2 and of the
// final multiply-add (the + 8).
__device__ inline float rank_error_bound(int d, float qn, float cmax) {
    return ((float)(3 * d + 8) * 2.3841858e-07f + 5.0e-05f) * (qn + cmax);
}

// Tile choice: 128 x 128 tiles on the bf16 kernel when they still cover the chip, else 64 x 64 in fp32.
// The kernels store either every key, A[nq][n_lists] (S null), or only the strip summaries
// S[n_strips][nq] for strips of coarse_strip_width() clusters (see rank_store).
// split_ws: coarse_split_bytes() bytes of device scratch for the bf16 operands.
inline bool coarse_big_tiles(int nq, int n_lists) {
    return (long)((n_lists + 127) / 128) * ((nq + 127) / 128) >= 1024;
}
inline int coarse_strip_width(int nq, int n_lists) { return coarse_big_tiles(nq, n_lists) ? 64 : 32; }
// whether a selection of the k smallest per row should work from strip summaries instead of all keys
inline bool coarse_use_strips(int nq, int n_lists, int k) {
    const int w = coarse_strip_width(nq, n_lists);
    return n_lists > 1024 && (n_lists + w - 1) / w >= 2 * k;
}
inline int coarse_padded_dim(int d) { return (d + BK - 1) / BK * BK; }
inline size_t coarse_split_bytes(size_t nq_max, size_t n_lists, int d) {
    return 2 * (align_up(split_rows_padded(nq_max) * coarse_padded_dim(d) * 2) + align_up(split_rows_padded(n_lists) * coarse_padded_dim(d) * 2));
}

int launch_coarse(const float* q, const float* centroids, const float* centroid_norms, int nq, int n_lists, int d,
                  uint32_t* A, StripSummary* S, void* split_ws, hipStream_t st) {
    if (coarse_big_tiles(nq, n_lists)) {
        const int dp = coarse_padded_dim(d);
        const size_t q_pad = split_rows_padded((size_t)nq), c_pad = split_rows_padded((size_t)n_lists);
        const size_t q_bytes = align_up(q_pad * dp * 2), c_bytes = align_up(c_pad * dp * 2);
        uint16_t* qh = (uint16_t*)split_ws;
        uint16_t* ql = (uint16_t*)((unsigned char*)split_ws + q_bytes);
        uint16_t* ch = (uint16_t*)((unsigned char*)split_ws + 2 * q_bytes);
        uint16_t* cl = (uint16_t*)((unsigned char*)split_ws + 2 * q_bytes + c_bytes);
        const size_t q_threads = q_pad * (dp / 8), c_threads = c_pad * (dp / 8);
        hipLaunchKernelGGL(split_bf16_kernel, dim3((unsigned)((q_threads + 255) / 256)), dim3(256), 0, st, q, (size_t)nq, q_pad, d, dp, qh, ql);
        hipLaunchKernelGGL(split_bf16_kernel, dim3((unsigned)((c_threads + 255) / 256)), dim3(256), 0, st, centroids, (size_t)n_lists, c_pad, d, dp, ch, cl);
        const size_t blocks = (size_t)((n_lists + 127) / 128) * 8 * (((nq + 127) / 128 + 7) / 8);
        if (blocks > 0x7FFFFFFFull) return fail(IVFPQ_EINVAL, "ranking grid of %zu workgroups exceeds the launch limit", blocks);
        dim3 grid((unsigned)blocks);
        if (S) hipLaunchKernelGGL(coarse_rank_split_kernel<true>, grid, dim3(256), 0, st, qh, ql, ch, cl, centroid_norms, nq, n_lists, dp, A, S);
        else hipLaunchKernelGGL(coarse_rank_split_kernel<false>, grid, dim3(256), 0, st, qh, ql, ch, cl, centroid_norms, nq, n_lists, dp, A, S);
    } else {
        dim3 grid((n_lists + 63) / 64, (nq + 63) / 64);
        hipLaunchKernelGGL(coarse_rank_kernel<1>, grid, dim3(256), 0, st, q, centroids, centroid_norms, nq, n_lists, d, A, S);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(IVFPQ_EHIP, "coarse_rank_kernel launch failed: %s", hipGetErrorString(e));
    return IVFPQ_OK;
}

}  // namespace
