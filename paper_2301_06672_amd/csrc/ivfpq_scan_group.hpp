// The filtered scan for up to G (query, probe) pairs of ONE cluster per workgroup (8-bit or 4-bit codes in
// 16-byte chunks, every table dtype).  Included by ivfpq_device.hip after the table helpers it uses.
//
// In the cluster-grouped order neighbouring pairs share their cluster, and everything that depends on the
// cluster alone is then done once for all of them: a codebook entry is loaded once and becomes R table
// entries, a code chunk is loaded once, and -- the point of this kernel -- one LDS read serves R lookups:
// the R tables are interleaved ENTRY BY ENTRY, entry (sub-space j, code c, query g) at byte
//     ((j * 2^pq_bits + c) * R + g) * entry_bytes,
// so the R entries a code selects are adjacent and come back from a single ds_read of R * entry_bytes
// (four e5m3 entries in one 32-bit bank word; two halves in one; two floats in a 64-bit read).  What the LDS
// spends per lookup therefore falls with the entry size (Sec. I-D's argument, carried over from "fewer
// distinct bank words per table row" to "more lookups per bank word"), and the vector ALU extracts a code
// byte once per R lookups.
//
// Decode and accumulate, per query:
//   8-bit formats   the FP32 pattern of a code, (b << shift) + lo (Sec. II), has its low 16 bits clear, so its
//                   upper half is a bf16 number with the same value.  The bytes of two consecutive sub-spaces
//                   are gathered into the two halves of a register with one byte permute, one shift-add turns
//                   both into bf16 ((b << (shift - 16)) + (lo >> 16) in each half), and one dot-product
//                   instruction with (1, 1) adds both to the FP32 sum: 1.5 vector instructions per lookup.
//   half            fused multiply-add with 1.0 that converts its half operand (either half of a register) in
//                   the same instruction (add_half_lo / add_half_hi): 1 per lookup.
//   float           one add.
// Per query the sub-spaces are added in ascending order, as scan_kernel does.
// 4-bit codes: a byte holds the codes of sub-spaces 2b (low nibble) and 2b + 1; the low and the high nibbles of a
// code word are masked and shifted to entry offsets four at a time (two instructions per four offsets), so that
// byte b of the one result is the LDS offset for sub-space 2b and byte b of the other that for 2b + 1.
//
// A run of 1, 2, 3 or 4 pairs of one cluster is processed at once (3 in the 4-wide layout with one byte of
// every entry unused).  A workgroup takes G consecutive pairs of the grouped order and cuts them into
// such runs at the seams between clusters.
// LDS: the slot's pair descriptors | tables | R residuals of d floats | per wave kGroupStageAll staged survivors |
// a flag and, per wave, kAliveCap group numbers of the split scan.
#pragma once

constexpr int kGroupStageAll = 128;  // survivors a wave stages before it appends them, over all queries of a run: 128 / R per query
                                     // (a 64-vector group with more survivors than that goes straight to the list)
constexpr int kGroupHead = 128;      // bytes at the start of the kernel's LDS that hold the slot's pair descriptors

// 4 * R table entries -- codes u = 0..3 of one lane, queries g = 0..R-1, f[u * R + g] -- converted to the
// table dtype and stored at `dst` (their place in the interleaved table: 4 * R * entry_bytes contiguous bytes)
template <int LUT, int R>
__device__ __forceinline__ void store_packed(unsigned char* dst, const float (&f)[4 * R], const Fp8Params fp8, int hi_v) {
    if constexpr (LUT == IVFPQ_LUT_FP32) {
#pragma unroll
        for (int i = 0; i < R; ++i)
            reinterpret_cast<float4*>(dst)[i] = make_float4(f[4 * i], f[4 * i + 1], f[4 * i + 2], f[4 * i + 3]);
    } else if constexpr (LUT == IVFPQ_LUT_FP16) {
        uint32_t w[2 * R];
#pragma unroll
        for (int i = 0; i < 2 * R; ++i) w[i] = half_bits_from_f32(f[2 * i]) | (half_bits_from_f32(f[2 * i + 1]) << 16);
        if constexpr (R == 1) *reinterpret_cast<uint2*>(dst) = make_uint2(w[0], w[1]);
        else
#pragma unroll
            for (int i = 0; i < R / 2; ++i) reinterpret_cast<uint4*>(dst)[i] = make_uint4(w[4 * i], w[4 * i + 1], w[4 * i + 2], w[4 * i + 3]);
    } else {
        constexpr int SH = Fp8Format<LUT>::shift;
        uint32_t w[R];
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const float g4[4] = {f[4 * i], f[4 * i + 1], f[4 * i + 2], f[4 * i + 3]};
            w[i] = fp8_pack4<SH>(g4, fp8, hi_v);
        }
        if constexpr (R == 1) *reinterpret_cast<uint32_t*>(dst) = w[0];
        else if constexpr (R == 2) *reinterpret_cast<uint2*>(dst) = make_uint2(w[0], w[1]);
        else *reinterpret_cast<uint4*>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// Q pairs of one cluster, q[g], pair[g], with tables interleaved R >= Q wide (Q < R: the entries of the missing
// queries are zero bytes that nobody decodes; three pairs run as Q = 3 in the R = 4 layout)
template <int LUT, int NCH, int R, int Q, int BITS, bool SPLIT>
__device__ __forceinline__ void group_run(const ScanArgs& a, unsigned char* smem, const int (&q)[Q], const uint4 (&pair)[Q]) {
    static_assert(Q >= 1 && Q <= R, "queries of a run fit its interleave width");
    static_assert(BITS == 8 || BITS == 4, "codes of 8 or 4 bits");
    constexpr int E = LutTraits<LUT>::bytes, W = E * R, LOGW = ilog2(W), KSUB = 1 << BITS;
    static_assert(BITS == 8 || 15 * W < 256, "a 4-bit code's entry offset fits a byte");
    constexpr int kGroupStage = kGroupStageAll / R;
    const uint32_t len = pair[0].y;
    if (len == 0) return;
    const int l = (int)pair[0].x;
    unsigned char* lut = smem;
    float* rq = reinterpret_cast<float*>(smem + (size_t)a.pq_dim * KSUB * W);
    unsigned char* after_rq = reinterpret_cast<unsigned char*>(rq) + (((size_t)Q * a.d * 4 + 15) & ~(size_t)15);
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));      // the same for the whole wave: loop counters and group addresses stay scalar
    const int n_waves = blockDim.x >> 6;
    const Fp8Params fp8 = a.fp8.fixed;
    uint32_t bound[Q], seg0[Q], row_pos0[Q], staged[Q];
    uint2* stage[Q];
#pragma unroll
    for (int g = 0; g < Q; ++g) {
        bound[g] = a.bounds[q[g]];
        seg0[g] = a.pairs[(size_t)q[g] * a.n_probes + 1].w;
        row_pos0[g] = pair[g].w;
        staged[g] = 0;
        stage[g] = reinterpret_cast<uint2*>(after_rq) + ((size_t)wave * Q + g) * kGroupStage;
    }
    const int n_groups = (int)((len + 63u) >> 6);
    const uint4* cbase = reinterpret_cast<const uint4*>(a.codes + (size_t)pair[0].z * 64 * ((size_t)NCH * 16));
    auto load_group = [&](uint4 (&buf)[NCH], int grp) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) buf[c] = cbase[((size_t)grp * NCH + c) * 64 + lane];
    };
    uint4 buf_a[NCH], buf_b[NCH];
    int grp = wave;
    if (grp < n_groups) load_group(buf_a, grp);       // HBM latency overlaps the table build

    // step 2: the residuals against the cluster's centroid
    for (int t = threadIdx.x; t < a.d; t += blockDim.x) {
        const float c = a.centroids[(size_t)l * a.d + t];
#pragma unroll
        for (int g = 0; g < Q; ++g) rq[g * a.d + t] = a.queries[(size_t)q[g] * a.d + t] - c;
    }
    __syncthreads();
    // step 3: all R tables from one pass over the codebooks.  A wave takes blocks of 256 consecutive entries of the
    // table, 4 codes per lane: one row of an 8-bit sub-space, 16 rows of 4-bit sub-spaces (a lane's four codes
    // then belong to sub-space 16 block + lane / 4; the host admits only tables that are whole blocks)
    // 64 sub-spaces of 8-bit codes with the early exit on: most groups are over every bound after half of the
    // sub-spaces, so only the first 32 rows are built now; the rest follows if some group is still in the race
    // (scan_kernel's split scan, for a run of queries)
    static_assert(!SPLIT || (BITS == 8 && NCH == 4), "the split scan is for 64 sub-spaces of 8-bit codes");
    constexpr bool lazy = SPLIT;
    uint32_t* any_alive = reinterpret_cast<uint32_t*>(after_rq + (size_t)n_waves * kGroupStageAll * 8);
    uint16_t* alive = reinterpret_cast<uint16_t*>(any_alive + 4) + (size_t)wave * kAliveCap;
    if (threadIdx.x == 0) *any_alive = 0u;
    auto build = [&](int block0, int block1) __attribute__((always_inline)) {
        int hi_v = fp8.hi;
        asm volatile("" : "+v"(hi_v));
        auto rows = [&](auto m_tag) {
            constexpr int M = decltype(m_tag)::value;
            auto load_row = [&](int j, float (&cbv)[4 * M]) {
                const float4* src = reinterpret_cast<const float4*>(a.codebooks + ((size_t)j * 256 + lane * 4) * M);
#pragma unroll
                for (int v = 0; v < M; ++v) {
                    const float4 x = src[v];
                    cbv[4 * v] = x.x; cbv[4 * v + 1] = x.y; cbv[4 * v + 2] = x.z; cbv[4 * v + 3] = x.w;
                }
            };
            auto finish_row = [&](int j, const float (&cbv)[4 * M]) {
                float f[4 * R];
#pragma unroll
                for (int i = 0; i < 4 * R; ++i) f[i] = 0.f;
#pragma unroll
                for (int g = 0; g < Q; ++g) {
                    float r[M];
                    const int sub = BITS == 8 ? j : j * 16 + (lane >> 2);
#pragma unroll
                    for (int t = 0; t < M; ++t) r[t] = rq[g * a.d + sub * M + t];
#pragma unroll
                    for (int u = 0; u < 4; ++u) f[u * R + g] = lut_entry<M>(cbv + u * M, r);
                }
                store_packed<LUT, R>(lut + ((size_t)j * 256 + lane * 4) * W, f, fp8, hi_v);
            };
            // two rows per trip: both rows' loads are in flight before either is used
            const int n_blocks = block1;
            int j = block0 + wave;
            for (; j + n_waves < n_blocks; j += 2 * n_waves) {
                float c0[4 * M], c1[4 * M];
                load_row(j, c0);
                load_row(j + n_waves, c1);
                finish_row(j, c0);
                finish_row(j + n_waves, c1);
            }
            for (; j < n_blocks; j += n_waves) {
                float c0[4 * M];
                load_row(j, c0);
                finish_row(j, c0);
            }
        };
        switch (a.m) {
            case 1: rows(std::integral_constant<int, 1>{}); break;
            case 2: rows(std::integral_constant<int, 2>{}); break;
            default: rows(std::integral_constant<int, 4>{}); break;      // the host admits m = 1, 2, 4 only
        }
    };
    build(0, lazy ? 32 : a.pq_dim * KSUB / 256);
    __syncthreads();

    // step 4: Eq. (1) for all R queries
    // The tables are read through LDS addresses formed as plain integers: `off` comes out of a sub-dword
    // shift and the row's constant goes into the read's immediate offset, with no add between them.  This
    // takes the dynamic LDS of the kernel to start at LDS address 0, i.e. the kernel to have no static LDS;
    // the host verifies that before the first launch (require_no_static_lds).
    using word_t = typename LdsWord<W>::type;
    auto lds_word = [&](int row, uint32_t off) __attribute__((always_inline)) -> word_t {
        return LdsWord<W>::load(off + ((uint32_t)kGroupHead + (uint32_t)row * ((uint32_t)KSUB * W)));
    };
    // both halves of a register hold the bf16 pattern of 1.0; decode constant of the 8-bit formats per half
    const bf16x2_t ones = __builtin_bit_cast(bf16x2_t, 0x3F803F80u);
    const uint32_t k2 = ((uint32_t)fp8.lo >> 16) * 0x10001u;
    // adds the entries of two consecutive sub-spaces, x0 then x1 (the words of all R queries), to every query's sum
    auto add_two = [&](const word_t& x0, const word_t& x1, float (&acc)[Q]) __attribute__((always_inline)) {
        if constexpr (kIsFp8<LUT>) {
            constexpr int S = Fp8Format<LUT>::shift - 16;
#pragma unroll
            for (int g = 0; g < Q; ++g) {
                // bytes g of x0 and x1 into the low bytes of the two halves
                uint32_t p = __builtin_amdgcn_perm((uint32_t)x1, (uint32_t)x0, 0x0c000c00u | ((4u + g) << 16) | (uint32_t)g);
                p = (p << S) + k2;
                acc[g] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, p), ones, acc[g], false);
            }
        } else if constexpr (LUT == IVFPQ_LUT_FP16) {
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const word_t& x = b == 0 ? x0 : x1;
                if constexpr (R == 1) {
                    acc[0] = add_half_lo(acc[0], x);
                } else if constexpr (R == 2) {
                    acc[0] = add_half_lo(acc[0], x);
                    acc[1] = add_half_hi(acc[1], x);
                } else {
                    const uint32_t lo = x.x, hi = x.y;
                    acc[0] = add_half_lo(acc[0], lo);
                    acc[1] = add_half_hi(acc[1], lo);
                    acc[2] = add_half_lo(acc[2], hi);
                    if constexpr (Q > 3) acc[3] = add_half_hi(acc[3], hi);
                }
            }
        } else {
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const word_t& x = b == 0 ? x0 : x1;
                if constexpr (R == 1) {
                    acc[0] += __uint_as_float(x);
                } else if constexpr (R == 2) {
                    acc[0] += __uint_as_float(x.x); acc[1] += __uint_as_float(x.y);
                } else {
                    acc[0] += __uint_as_float(x.x); acc[1] += __uint_as_float(x.y);
                    acc[2] += __uint_as_float(x.z);
                    if constexpr (Q > 3) acc[3] += __uint_as_float(x.w);
                }
            }
        }
    };
    auto chunk = [&](const uint4& v, int c, float (&acc)[Q]) __attribute__((always_inline)) {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if constexpr (BITS == 8) {
                // the table words of two code words (eight sub-spaces) are read before the first is used
                if (u & 1) continue;
                word_t x[8];
#pragma unroll
                for (int v2 = 0; v2 < 2; ++v2) {
                    const uint32_t cw = w[u + v2];
                    const int row = (c * 4 + u + v2) * 4;
                    const uint32_t off[4] = {byte_shl<0, LOGW>(cw), byte_shl<1, LOGW>(cw), byte_shl<2, LOGW>(cw), byte_shl<3, LOGW>(cw)};
#pragma unroll
                    for (int b = 0; b < 4; ++b) x[4 * v2 + b] = lds_word(row + b, off[b]);
                }
#pragma unroll
                for (int pr = 0; pr < 4; ++pr) add_two(x[2 * pr], x[2 * pr + 1], acc);
            } else {
                // byte b of lo4 / hi4: the entry offset of the code in the low / high nibble of byte b
                constexpr uint32_t kNibbles = 0x0F0F0F0Fu << LOGW;
                const uint32_t lo4 = (w[u] << LOGW) & kNibbles, hi4 = (w[u] >> (4 - LOGW)) & kNibbles;
                const int row = (c * 4 + u) * 8;
                const uint32_t off_lo[4] = {byte_shl<0, 0>(lo4), byte_shl<1, 0>(lo4), byte_shl<2, 0>(lo4), byte_shl<3, 0>(lo4)};
                const uint32_t off_hi[4] = {byte_shl<0, 0>(hi4), byte_shl<1, 0>(hi4), byte_shl<2, 0>(hi4), byte_shl<3, 0>(hi4)};
                word_t x[8];             // read before the first is used, like the eight words of 8-bit codes above
#pragma unroll
                for (int b = 0; b < 4; ++b) { x[2 * b] = lds_word(row + 2 * b, off_lo[b]); x[2 * b + 1] = lds_word(row + 2 * b + 1, off_hi[b]); }
#pragma unroll
                for (int pr = 0; pr < 4; ++pr) add_two(x[2 * pr], x[2 * pr + 1], acc);
            }
        }
    };
    // Table entries are never negative, so the partial sums only grow: once all 64 x R of them are over their
    // queries' bounds no vector of the group can survive for any of the queries, and the remaining chunks are
    // skipped (the partial sums then fail the filter as the full sums would).
    auto accumulate = [&](const uint4 (&buf)[NCH], float (&acc)[Q], auto chunks_tag) __attribute__((always_inline)) {
        constexpr int CHUNKS = decltype(chunks_tag)::value;      // the leading chunks to add; NCH = all
#pragma unroll
        for (int g = 0; g < Q; ++g) acc[g] = 0.f;
        bool over = false;                  // wave-uniform
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c) {
            if (over) continue;
            chunk(buf[c], c, acc);
            if (c + 1 < CHUNKS && a.early_exit) {
                unsigned long long in_race = 0;
#pragma unroll
                for (int g = 0; g < Q; ++g) in_race |= ballot64(__float_as_uint(acc[g]) <= bound[g]);
                over = in_race == 0;
            }
        }
    };
    auto flush = [&](auto g_tag) __attribute__((always_inline)) {
        constexpr int g = decltype(g_tag)::value;
        if (staged[g] == 0) return;
        uint32_t base = 0;
        if (lane == 0) base = atomicAdd(&a.counts[q[g]], staged[g]);
        base = (uint32_t)__builtin_amdgcn_readfirstlane((int)base);
        uint32_t* dst_key = reinterpret_cast<uint32_t*>(a.R) + (size_t)q[g] * a.stride + seg0[g] + base;
        uint32_t* dst_pos = a.Rpos + (size_t)q[g] * a.stride + seg0[g] + base;
        for (uint32_t j = lane; j < staged[g]; j += kWave) {
            const uint2 e = stage[g][j];
            dst_key[j] = e.x;
            dst_pos[j] = e.y;
        }
        staged[g] = 0;
    };
    // end of the run: what every query still has staged.  The slots of all queries are requested first (one atomic
    // each, all in flight together), then the copies follow: one wait for the counters instead of one per query.
    auto flush_all = [&]() __attribute__((always_inline)) {
        uint32_t base[Q];
#pragma unroll
        for (int g = 0; g < Q; ++g) {
            base[g] = 0;
            if (staged[g] != 0 && lane == 0) base[g] = atomicAdd(&a.counts[q[g]], staged[g]);
        }
        static_for<Q>([&](auto g_tag) __attribute__((always_inline)) {
            constexpr int g = decltype(g_tag)::value;
            if (staged[g] == 0) return;
            const uint32_t at = (uint32_t)__builtin_amdgcn_readfirstlane((int)base[g]);
            uint32_t* dst_key = reinterpret_cast<uint32_t*>(a.R) + (size_t)q[g] * a.stride + seg0[g] + at;
            uint32_t* dst_pos = a.Rpos + (size_t)q[g] * a.stride + seg0[g] + at;
            for (uint32_t j = lane; j < staged[g]; j += kWave) {
                const uint2 e = stage[g][j];
                dst_key[j] = e.x;
                dst_pos[j] = e.y;
            }
            staged[g] = 0;
        });
    };
    auto keep = [&](int grp_i, const float (&acc)[Q]) __attribute__((always_inline)) {
        const uint32_t i = (uint32_t)grp_i * 64u + lane;
        const bool real = i < len;                  // the last group is padded with zero codes
        const unsigned long long m_real = ballot64(real);
        static_for<Q>([&](auto g_tag) __attribute__((always_inline)) {
            constexpr int g = decltype(g_tag)::value;
            // (the mask is the AND of two compares' results; a ballot of their conjunction goes through a 0/1 value)
            const bool under = __float_as_uint(acc[g]) <= bound[g];
            const unsigned long long m = ballot64(under) & m_real;
            const bool ok = real && under;
            if (m != 0) {
                const uint32_t cnt = (uint32_t)__popcll(m), rank = lanes_below(m);
                if (staged[g] + cnt > (uint32_t)kGroupStage) flush(g_tag);
                if (cnt > (uint32_t)kGroupStage) {
                    // more survivors in one group than the staging area holds: appended directly
                    uint32_t base = 0;
                    if (lane == 0) base = atomicAdd(&a.counts[q[g]], cnt);
                    base = (uint32_t)__builtin_amdgcn_readfirstlane((int)base);
                    if (ok) {
                        const size_t at = (size_t)q[g] * a.stride + seg0[g] + base + rank;
                        reinterpret_cast<uint32_t*>(a.R)[at] = __float_as_uint(acc[g]);
                        a.Rpos[at] = row_pos0[g] + i;
                    }
                } else {
                    if (ok) stage[g][staged[g] + rank] = make_uint2(__float_as_uint(acc[g]), row_pos0[g] + i);
                    staged[g] += cnt;
                }
            }
        });
    };
    float acc[Q];
    constexpr std::integral_constant<int, NCH> kAllChunks{};
    if constexpr (SPLIT) {
        {
            constexpr int HCH = NCH / 2;            // chunks of the first pass: the codes of the 32 leading sub-spaces
            uint32_t n_alive = 0;                   // wave-uniform
            bool redo_all = false;                  // more groups in the race than the list holds: take them all again
            auto load_head = [&](uint4 (&buf)[NCH], int g) __attribute__((always_inline)) {
#pragma unroll
                for (int c = 0; c < HCH; ++c) buf[c] = cbase[((size_t)g * NCH + c) * 64 + lane];
            };
            auto first_pass = [&](int g, const uint4 (&buf)[NCH]) __attribute__((always_inline)) {
                accumulate(buf, acc, std::integral_constant<int, HCH>{});
                unsigned long long in_race = 0;
#pragma unroll
                for (int gq = 0; gq < Q; ++gq) in_race |= ballot64(__float_as_uint(acc[gq]) <= bound[gq]);
                in_race &= ballot64((uint32_t)g * 64u + lane < len);
                if (in_race != 0) {
                    if (n_alive < (uint32_t)kAliveCap && g / n_waves < 65536) { if (lane == 0) alive[n_alive] = (uint16_t)(g / n_waves); ++n_alive; }
                    else redo_all = true;
                }
            };
            // (the loads of the wave's first group were issued in full before the build; later groups load the head only)
            while (grp < n_groups) {
                const int gn = grp + n_waves;
                if (gn < n_groups) load_head(buf_b, gn);
                first_pass(grp, buf_a);
                if (gn >= n_groups) break;
                grp = gn + n_waves;
                if (grp < n_groups) load_head(buf_a, grp);
                first_pass(gn, buf_b);
            }
            if (lane == 0 && (n_alive != 0 || redo_all)) atomicOr(any_alive, 1u);
            __syncthreads();
            if (*any_alive == 0u) return;           // the same for every wave
            build(32, a.pq_dim * KSUB / 256);
            __syncthreads();
            if (redo_all) {
                for (grp = wave; grp < n_groups; grp += n_waves) {
                    load_group(buf_a, grp);
                    accumulate(buf_a, acc, kAllChunks);
                    keep(grp, acc);
                }
            } else {
                for (uint32_t t = 0; t < n_alive; ++t) {
                    grp = (int)alive[t] * n_waves + wave;
                    load_group(buf_a, grp);
                    accumulate(buf_a, acc, kAllChunks);
                    keep(grp, acc);
                }
            }
            flush_all();
            return;
        }
    }
    while (grp < n_groups) {
        const int gn = grp + n_waves;
        if (gn < n_groups) load_group(buf_b, gn);
        accumulate(buf_a, acc, kAllChunks);
        keep(grp, acc);
        if (gn >= n_groups) break;
        grp = gn + n_waves;
        if (grp < n_groups) load_group(buf_a, grp);
        accumulate(buf_b, acc, kAllChunks);
        keep(gn, acc);
    }
    flush_all();
}

// Workgroup `slot` takes pairs [G slot, G slot + G) of the cluster-grouped order; the slots are dealt to the
// XCDs in blocks of order_block / G, which is the dealing of scan_kernel's pairs in blocks of order_block.
// The first kGroupHead bytes of the LDS hold the slot's pair descriptors (the runs read them by position);
// group_run's `smem` starts behind them.
template <int LUT, int NCH, int G, int BITS, bool SPLIT>
__global__ void __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(4, 8)))
scan_group_kernel(ScanArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    static_assert(G * 20 <= kGroupHead, "descriptors of a slot must fit the head of the LDS");
    const uint32_t n_slots = (a.n_pairs + (uint32_t)G - 1u) / (uint32_t)G, blk = a.order_block / (uint32_t)G;
    const uint32_t xcd = blockIdx.x & 7u, rank = blockIdx.x >> 3;
    const uint32_t slot = ((rank / blk) * 8u + xcd) * blk + rank % blk;
    if (slot >= n_slots) return;
    const uint32_t first = slot * (uint32_t)G;
    const int n_here = (int)(a.n_pairs - first < (uint32_t)G ? a.n_pairs - first : (uint32_t)G);
    uint4* s_pair = reinterpret_cast<uint4*>(smem);
    int* s_q = reinterpret_cast<int*>(smem + G * 16);
    if ((int)threadIdx.x < n_here) {
        const uint32_t lin = a.order[first + threadIdx.x];
        const int qi = (int)(lin / (uint32_t)(a.n_probes - 1));
        s_q[threadIdx.x] = qi;
        s_pair[threadIdx.x] = a.pairs[(size_t)qi * a.n_probes + 1 + (lin - (uint32_t)qi * (uint32_t)(a.n_probes - 1))];
    }
    __syncthreads();
    auto uni = [](uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); };
    auto q_at = [&](int i) { return (int)uni((uint32_t)s_q[i]); };
    auto pair_at = [&](int i) { const uint4 p = s_pair[i]; return make_uint4(uni(p.x), uni(p.y), uni(p.z), uni(p.w)); };
    unsigned char* body = smem + kGroupHead;
    // runs of pairs that name the same cluster, each processed at once
    int i = 0;
    while (i < n_here) {
        int r = 1;
        const uint32_t cl = uni(s_pair[i].x);
        while (i + r < n_here && uni(s_pair[i + r].x) == cl) ++r;
        if (i > 0) __syncthreads();          // the previous run's tables are still being read by slower waves
        bool done = false;
        if constexpr (G >= 4) {
            if (r == 4) {
                const int qq[4] = {q_at(i), q_at(i + 1), q_at(i + 2), q_at(i + 3)};
                const uint4 pp[4] = {pair_at(i), pair_at(i + 1), pair_at(i + 2), pair_at(i + 3)};
                group_run<LUT, NCH, 4, 4, BITS, SPLIT>(a, body, qq, pp);
                done = true;
            } else if (r == 3) {
                const int qq[3] = {q_at(i), q_at(i + 1), q_at(i + 2)};
                const uint4 pp[3] = {pair_at(i), pair_at(i + 1), pair_at(i + 2)};
                group_run<LUT, NCH, 4, 3, BITS, SPLIT>(a, body, qq, pp);
                done = true;
            }
        }
        if (!done) {
            if (r == 2) {
                const int qq[2] = {q_at(i), q_at(i + 1)};
                const uint4 pp[2] = {pair_at(i), pair_at(i + 1)};
                group_run<LUT, NCH, 2, 2, BITS, SPLIT>(a, body, qq, pp);
            } else {
                const int qq[1] = {q_at(i)};
                const uint4 pp[1] = {pair_at(i)};
                group_run<LUT, NCH, 1, 1, BITS, SPLIT>(a, body, qq, pp);
            }
        }
        i += r;
    }
}
