/*
 * ivfpq_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct CPU rendering of the IVFPQ index build and
 * search phases of arXiv 2301.06672 (Sec. I-B, I-C, II), used only by the test
 * suite, the smoke check and the benchmark's cpu_baseline leg.  It shares no
 * code with the HIP library; nothing in the product path may call it.
 *
 * Every function names the passage of the paper it follows.  Where the paper
 * is silent (Figs. 1-4 with the bit layouts and conversions are not in the
 * text) the reading taken is stated at the function.
 *
 * Arithmetic: float64 wherever the paper does not fix a precision (exact k-NN,
 * k-means, probe selection); fp32 in a fixed operation order for the lookup
 * table and for Eq. (1), because the table is *stored* in fp32/fp16/8-bit and
 * its entries must be reproducible bit for bit.
 *
 * Build: gcc -O2 -std=c11 -fopenmp -ffp-contract=off -fPIC -shared (oracle/build.py).
 * Parallelism: OpenMP over independent queries / rows only; no blocking,
 * fusion or reordering inside one query.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ */
/* small helpers                                                        */
/* ------------------------------------------------------------------ */

typedef struct { double key; int64_t id; } pair_d;
typedef struct { float key; int64_t id; } pair_f;

static int cmp_pair_d(const void* a, const void* b) {
    const pair_d* x = (const pair_d*)a; const pair_d* y = (const pair_d*)b;
    if (x->key < y->key) return -1;
    if (x->key > y->key) return 1;
    if (x->id < y->id) return -1;
    if (x->id > y->id) return 1;
    return 0;
}
static int cmp_pair_f(const void* a, const void* b) {
    const pair_f* x = (const pair_f*)a; const pair_f* y = (const pair_f*)b;
    if (x->key < y->key) return -1;
    if (x->key > y->key) return 1;
    if (x->id < y->id) return -1;
    if (x->id > y->id) return 1;
    return 0;
}

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
void orc_set_num_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* squared L2 distance, float64 accumulation of fp32 inputs */
static double sqdist_f64(const float* a, const float* b, int d) {
    double acc = 0.0;
    for (int t = 0; t < d; ++t) {
        double diff = (double)a[t] - (double)b[t];
        acc += diff * diff;
    }
    return acc;
}

/* ------------------------------------------------------------------ */
/* Sec. I-B: exact k nearest neighbours (the ground truth of "recall")  */
/* ------------------------------------------------------------------ */
/* ids/d2: [nq][k]; sorted ascending by (distance, id); padded with -1/+inf
 * when n < k. */
void orc_exact_knn(const float* data, int64_t n, int d,
                   const float* queries, int64_t nq, int k,
                   int64_t* ids, double* d2) {
    #pragma omp parallel
    {
        pair_d* buf = (pair_d*)malloc((size_t)(n > 0 ? n : 1) * sizeof(pair_d));
        #pragma omp for schedule(dynamic, 1)
        for (int64_t q = 0; q < nq; ++q) {
            for (int64_t i = 0; i < n; ++i) {
                buf[i].key = sqdist_f64(queries + q * d, data + i * d, d);
                buf[i].id = i;
            }
            qsort(buf, (size_t)n, sizeof(pair_d), cmp_pair_d);
            for (int j = 0; j < k; ++j) {
                if (j < n) { ids[q * k + j] = buf[j].id; d2[q * k + j] = buf[j].key; }
                else       { ids[q * k + j] = -1;        d2[q * k + j] = INFINITY; }
            }
        }
        free(buf);
    }
}

/* ------------------------------------------------------------------ */
/* Sec. I-C build step 1 (and the per-sub-space quantiser of step 3):   */
/* Lloyd's k-means.  Reading: nearest centre under squared L2 in         */
/* float64, ties to the lowest centre index; centre = float64 mean cast   */
/* to fp32; an empty cluster keeps its previous centre.                   */
/* ------------------------------------------------------------------ */
/* labels[i] = arg min_c |x_i - centre_c|^2 ; returns the summed minimum */
double orc_assign(const float* x, int64_t n, int dim,
                  const float* centres, int n_centres, int32_t* labels) {
    double total = 0.0;
    #pragma omp parallel for schedule(static) reduction(+:total)
    for (int64_t i = 0; i < n; ++i) {
        double best = INFINITY; int32_t arg = 0;
        for (int c = 0; c < n_centres; ++c) {
            double dist = sqdist_f64(x + i * dim, centres + (int64_t)c * dim, dim);
            if (dist < best) { best = dist; arg = c; }   /* strict: ties keep the lower index */
        }
        labels[i] = arg;
        total += best;
    }
    return total;
}

/* init_rows: n_centres distinct row indices drawn by the caller's seeded
 * generator (the method's random numbers are inputs, not drawn here).
 * inertia[it] = sum of squared distances to the centres the assignment of
 * iteration `it` used (non-increasing over iterations). */
void orc_kmeans(const float* x, int64_t n, int dim, int n_centres, int iters,
                const int64_t* init_rows, float* centres, double* inertia) {
    for (int c = 0; c < n_centres; ++c)
        memcpy(centres + (int64_t)c * dim, x + init_rows[c] * dim, (size_t)dim * sizeof(float));
    int32_t* labels = (int32_t*)malloc((size_t)(n > 0 ? n : 1) * sizeof(int32_t));
    double* sums = (double*)malloc((size_t)n_centres * dim * sizeof(double));
    int64_t* counts = (int64_t*)malloc((size_t)n_centres * sizeof(int64_t));
    for (int it = 0; it < iters; ++it) {
        double total = orc_assign(x, n, dim, centres, n_centres, labels);
        if (inertia) inertia[it] = total;
        memset(sums, 0, (size_t)n_centres * dim * sizeof(double));
        memset(counts, 0, (size_t)n_centres * sizeof(int64_t));
        for (int64_t i = 0; i < n; ++i) {
            int32_t c = labels[i];
            counts[c] += 1;
            for (int t = 0; t < dim; ++t) sums[(int64_t)c * dim + t] += (double)x[i * dim + t];
        }
        for (int c = 0; c < n_centres; ++c) {
            if (counts[c] == 0) continue;
            for (int t = 0; t < dim; ++t)
                centres[(int64_t)c * dim + t] = (float)(sums[(int64_t)c * dim + t] / (double)counts[c]);
        }
    }
    free(labels); free(sums); free(counts);
}

/* ------------------------------------------------------------------ */
/* Sec. II: the sign-less 8-bit float "e5m3" (and "e4m4").               */
/* Reading (Figs. 1-4 are not in the text): E exponent bits on top, M     */
/* mantissa bits below, no sign, every code a normal number:               */
/*     value(b) = (1 + mant / 2^M) * 2^(exp - bias),                       */
/* with exp = b >> M, mant = b & (2^M - 1).  e5m3 takes bias 15 so that    */
/* its 32 binades 2^-15 .. 2^16 contain the FP16 normal range.             */
/* Encoding: nearest representable value, a tie going to the larger one;   */
/* anything below the smallest value (zero and negatives included) gives   */
/* code 0, anything above the largest (+Inf included) gives code 255; a    */
/* NaN follows its sign bit (the clamp acts on the bit pattern as a signed */
/* integer).  `truncate` selects the alternate reading: the largest        */
/* representable value not above x.                                        */
/* The oracle works from this definition in float64, not from bit tricks.  */
/* ------------------------------------------------------------------ */
double orc_fp8_value(int b, int mant_bits, int bias) {
    int e = b >> mant_bits;
    int m = b & ((1 << mant_bits) - 1);
    return ldexp(1.0 + (double)m / (double)(1 << mant_bits), e - bias);
}

/* the 256 representable values, ascending (value(b) is strictly increasing in b) */
static void fp8_table(int mant_bits, int bias, double* table) {
    for (int b = 0; b < 256; ++b) table[b] = orc_fp8_value(b, mant_bits, bias);
}

static uint8_t fp8_encode_with_table(float x, const double* table, int truncate) {
    if (isnan(x)) return signbit(x) ? 0x00 : 0xFF;
    double v = (double)x;
    if (!(v > table[0])) return 0x00;
    if (v >= table[255]) return 0xFF;
    /* largest code whose value is <= v (bisection on the sorted table) */
    int lo = 0, hi = 255;              /* table[lo] <= v < table[hi] */
    while (hi - lo > 1) {
        int mid = (lo + hi) / 2;
        if (table[mid] <= v) lo = mid; else hi = mid;
    }
    if (truncate) return (uint8_t)lo;
    /* both gaps are exact in float64 (fp32 input, <= 5 significant bits in the codes) */
    return (uint8_t)((v - table[lo]) >= (table[lo + 1] - v) ? lo + 1 : lo);
}

uint8_t orc_fp8_encode(float x, int mant_bits, int bias, int truncate) {
    double table[256];
    fp8_table(mant_bits, bias, table);
    return fp8_encode_with_table(x, table, truncate);
}

float orc_fp8_decode(uint8_t b, int mant_bits, int bias) {
    return (float)orc_fp8_value((int)b, mant_bits, bias);
}

uint8_t orc_e5m3_encode(float x, int truncate) { return orc_fp8_encode(x, 3, 15, truncate); }
float orc_e5m3_decode(uint8_t b) { return orc_fp8_decode(b, 3, 15); }

/* IEEE binary16 storage (the "half" table of Sec. I-D / Sec. III), written
 * from the format's definition: round to nearest, ties to even, subnormals
 * kept.  Values above the largest finite half saturate to it (the paper is
 * silent on overflow; a distance table must not hold +Inf). */
uint16_t orc_fp16_encode(float x) {
    if (isnan(x)) return 0x7E00;
    uint16_t sign = signbit(x) ? 0x8000 : 0;
    double a = fabs((double)x);
    if (a > 65504.0) a = 65504.0;
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);                /* a = fr * 2^e, fr in [0.5, 1) */
    int exp = e - 1;                   /* a = (2 fr) * 2^exp, 2 fr in [1, 2) */
    double scaled;                     /* a in units of the half's last place */
    if (exp < -14) { exp = -14; }
    scaled = ldexp(a, 10 - exp);       /* exact: power-of-two scaling */
    double fl = floor(scaled);
    double rem = scaled - fl;
    uint32_t m = (uint32_t)fl;
    if (rem > 0.5 || (rem == 0.5 && (m & 1u))) m += 1;
    /* m is in [0, 2048]; 1024..2047 normal at `exp`, 2048 carries into exp+1, <1024 subnormal */
    uint32_t biased;
    if (exp == -14 && m < 1024) { biased = 0; }
    else {
        if (m == 2048) { m = 1024; exp += 1; }
        biased = (uint32_t)(exp + 15);
        m -= 1024;
    }
    return (uint16_t)(sign | (biased << 10) | m);
}

float orc_fp16_decode(uint16_t h) {
    int sign = (h >> 15) & 1, e = (h >> 10) & 31, m = h & 1023;
    double v;
    if (e == 31) v = m ? NAN : INFINITY;
    else if (e == 0) v = ldexp((double)m, -24);
    else v = ldexp(1.0 + (double)m / 1024.0, e - 15);
    return (float)(sign ? -v : v);
}

void orc_e5m3_encode_array(const float* x, int64_t n, int truncate, uint8_t* out) {
    double table[256];
    fp8_table(3, 15, table);
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) out[i] = fp8_encode_with_table(x[i], table, truncate);
}
/* general (mantissa bits, bias) variant, for the 4+4 split of Sec. II */
void orc_fp8_encode_array(const float* x, int64_t n, int mant_bits, int bias, int truncate, uint8_t* out) {
    double table[256];
    fp8_table(mant_bits, bias, table);
    for (int64_t i = 0; i < n; ++i) out[i] = fp8_encode_with_table(x[i], table, truncate);
}
void orc_fp8_decode_array(const uint8_t* b, int64_t n, int mant_bits, int bias, float* out) {
    for (int64_t i = 0; i < n; ++i) out[i] = orc_fp8_decode(b[i], mant_bits, bias);
}
void orc_e5m3_decode_array(const uint8_t* b, int64_t n, float* out) {
    for (int64_t i = 0; i < n; ++i) out[i] = orc_e5m3_decode(b[i]);
}
void orc_fp16_encode_array(const float* x, int64_t n, uint16_t* out) {
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) out[i] = orc_fp16_encode(x[i]);
}
void orc_fp16_decode_array(const uint16_t* h, int64_t n, float* out) {
    for (int64_t i = 0; i < n; ++i) out[i] = orc_fp16_decode(h[i]);
}

/* ------------------------------------------------------------------ */
/* Sec. I-C search step 1: the n_probes clusters whose centroids are     */
/* nearest to the query (float64 distances, ascending, ties to the lower  */
/* cluster index).                                                        */
/* ------------------------------------------------------------------ */
void orc_select_probes(const float* centroids, int n_lists, int d,
                       const float* queries, int64_t nq, int n_probes,
                       uint32_t* probes, double* probe_d2) {
    #pragma omp parallel
    {
        pair_d* buf = (pair_d*)malloc((size_t)n_lists * sizeof(pair_d));
        #pragma omp for schedule(static)
        for (int64_t q = 0; q < nq; ++q) {
            for (int l = 0; l < n_lists; ++l) {
                buf[l].key = sqdist_f64(queries + q * d, centroids + (int64_t)l * d, d);
                buf[l].id = l;
            }
            qsort(buf, (size_t)n_lists, sizeof(pair_d), cmp_pair_d);
            for (int p = 0; p < n_probes; ++p) {
                probes[q * n_probes + p] = (uint32_t)buf[p].id;
                if (probe_d2) probe_d2[q * n_probes + p] = buf[p].key;
            }
        }
        free(buf);
    }
}

/* ------------------------------------------------------------------ */
/* Sec. I-C search steps 2-3: residual of the query against one centroid  */
/* and the "norm2 fragment lookup table" F.  fp32, fixed order:           */
/*   rq[t] = fl(q[t] - c[t]);                                             */
/*   F[j][code] = sum over the sub-vector, left to right, of               */
/*                fma(diff, diff, acc) with diff = fl(cb[j][code][t]-rq[j*m+t]) */
/* codebooks: [pq_dim][ksub][m] fp32.                                      */
/* ------------------------------------------------------------------ */
void orc_lut_f32(const float* query, const float* centroid, const float* codebooks,
                 int d, int pq_dim, int ksub, float* F) {
    int m = d / pq_dim;
    float* rq = (float*)malloc((size_t)d * sizeof(float));
    for (int t = 0; t < d; ++t) rq[t] = query[t] - centroid[t];
    for (int j = 0; j < pq_dim; ++j) {
        for (int c = 0; c < ksub; ++c) {
            const float* cb = codebooks + ((int64_t)j * ksub + c) * m;
            float acc = 0.0f;
            for (int t = 0; t < m; ++t) {
                float diff = cb[t] - rq[j * m + t];
                acc = fmaf(diff, diff, acc);
            }
            F[(int64_t)j * ksub + c] = acc;
        }
    }
    free(rq);
}

/* Power-of-two scaling of a table stored in an 8-bit format (a reading that goes beyond Sec. II,
 * which fixes one bias per format): multiplying every entry by 2^s before the encode and dividing
 * by 2^s after the decode is the same as moving the format's exponent bias by s, so the scale is
 * expressed as a per-table bias.  It is chosen so that the binade of the table's largest entry is
 * the format's top binade: with e = floor(log2(max F)) and E = 2^exp_bits - 1 (the largest exponent
 * field), bias = E - e.  Entries below the FP32 normal range count as 2^-127 (e = -127; so does an
 * all-zero table), +Inf as 2^128; the result is clamped to [bias_min, bias_max]. */
int orc_fp8_table_bias(const float* F, int64_t n, int exp_bits, int bias_min, int bias_max) {
    double mx = 0.0;
    for (int64_t i = 0; i < n; ++i)
        if (!isnan(F[i]) && (double)F[i] > mx) mx = (double)F[i];
    int e;
    if (isinf(mx)) e = 128;
    else if (mx < ldexp(1.0, -126)) e = -127;
    else { (void)frexp(mx, &e); e -= 1; }       /* frexp: mx = f * 2^e with f in [0.5, 1) */
    int bias = ((1 << exp_bits) - 1) - e;
    if (bias < bias_min) bias = bias_min;
    if (bias > bias_max) bias = bias_max;
    return bias;
}

/* lut_dtype: 0 = fp32 (4 B little-endian), 1 = IEEE half (2 B), 2 = e5m3 (1 B), 3 = e4m4 (1 B; the
 * 4+4 split of Sec. II).  For the two 8-bit formats `bias` is the exponent bias (15 is the reading
 * taken for e5m3; the text gives none for e4m4) and `truncate` the rounding; per_table != 0 replaces
 * `bias` by orc_fp8_table_bias of this table, clamped to [bias_min, bias_max].
 * `stored` receives the table exactly as it sits in on-chip memory;
 * `decoded` (may be NULL) receives what a lookup returns, as fp32.  Returns the bias used. */
enum { ORC_LUT_FP32 = 0, ORC_LUT_FP16 = 1, ORC_LUT_E5M3 = 2, ORC_LUT_E4M4 = 3 };

static int lut_elem_bytes(int lut_dtype) { return lut_dtype == 0 ? 4 : (lut_dtype == 1 ? 2 : 1); }

int orc_lut_store(const float* F, int64_t n, int lut_dtype, int truncate, int bias, int per_table,
                  int bias_min, int bias_max, uint8_t* stored, float* decoded) {
    double table[256];
    const int mant_bits = lut_dtype == ORC_LUT_E4M4 ? 4 : 3;
    if ((lut_dtype == ORC_LUT_E5M3 || lut_dtype == ORC_LUT_E4M4) && per_table)
        bias = orc_fp8_table_bias(F, n, 8 - mant_bits, bias_min, bias_max);
    fp8_table(mant_bits, bias, table);
    for (int64_t i = 0; i < n; ++i) {
        float back;
        if (lut_dtype == ORC_LUT_FP32) {
            memcpy(stored + 4 * i, &F[i], 4); back = F[i];
        } else if (lut_dtype == ORC_LUT_FP16) {
            uint16_t h = orc_fp16_encode(F[i]);
            memcpy(stored + 2 * i, &h, 2); back = orc_fp16_decode(h);
        } else {
            uint8_t b = fp8_encode_with_table(F[i], table, truncate);
            stored[i] = b; back = orc_fp8_decode(b, mant_bits, bias);
        }
        if (decoded) decoded[i] = back;
    }
    return bias;
}

/* PQ code of sub-space j of one stored vector.  The paper treats p = 8 only (byte j); reading for
 * 4 <= p <= 8: the codes of a vector form one string of pq_dim * p bits, sub-space j in bits
 * [j*p, (j+1)*p), bit i of the string being bit (i mod 8) of byte (i div 8).  For p = 4 that puts the
 * even sub-space in the low nibble of byte j/2 and the odd one in the high nibble. */
static int code_at(const uint8_t* codes, int j, int pq_bits) {
    int code = 0;
    for (int b = 0; b < pq_bits; ++b) {
        int64_t i = (int64_t)j * pq_bits + b;
        code |= ((codes[i >> 3] >> (i & 7)) & 1) << b;
    }
    return code;
}

/* ------------------------------------------------------------------ */
/* Sec. I-C search step 4, Eq. (1): R = sum_{j=1..s} F(y_j) for every     */
/* coded vector of one cluster; fp32, j ascending, starting from +0.      */
/* R64 (may be NULL): the same sum in float64, for error reporting.       */
/* ------------------------------------------------------------------ */
void orc_scan_list(const float* lut_decoded, int pq_dim, int pq_bits,
                   const uint8_t* codes, int64_t n_vec, float* R, double* R64) {
    int ksub = 1 << pq_bits;
    int code_bytes = pq_dim * pq_bits / 8;
    for (int64_t i = 0; i < n_vec; ++i) {
        const uint8_t* y = codes + i * code_bytes;
        float acc = 0.0f; double acc64 = 0.0;
        for (int j = 0; j < pq_dim; ++j) {
            float f = lut_decoded[(int64_t)j * ksub + code_at(y, j, pq_bits)];
            acc = acc + f;
            acc64 += (double)f;
        }
        R[i] = acc;
        if (R64) R64[i] = acc64;
    }
}

/* ------------------------------------------------------------------ */
/* Sec. I-C search, steps 1-5 for a batch of queries on a saved index.    */
/* Index arrays (all host, the logical layout):                           */
/*   centroids [n_lists][d], codebooks [pq_dim][2^pq_bits][d/pq_dim],     */
/*   list_offsets [n_lists+1], codes [n][pq_dim*pq_bits/8] and ids [n]    */
/*   in list order.                                                       */
/* probes_in: NULL -> step 1 is done here; else [nq][n_probes] given.     */
/* Step 5: gather (R, id) of all probed clusters, full sort by (R, id),   */
/* first k; fewer than k candidates -> id -1, distance +inf.              */
/* stats (may be NULL) [2]: number of table entries that hit the lowest / */
/* highest code of an 8-bit format (floored / saturated), summed.        */
/* ------------------------------------------------------------------ */
void orc_search(int64_t n, int d, int n_lists, int pq_dim, int pq_bits,
                const float* centroids, const float* codebooks,
                const int64_t* list_offsets, const uint8_t* codes, const int64_t* ids,
                const float* queries, int64_t nq, int n_probes, int k,
                int lut_dtype, int truncate, int bias, int per_table, int bias_min, int bias_max,
                const uint32_t* probes_in,
                int64_t* out_ids, float* out_d, int64_t* stats) {
    (void)n;
    int ksub = 1 << pq_bits;
    int code_bytes = pq_dim * pq_bits / 8;
    int64_t lut_n = (int64_t)pq_dim * ksub;
    int64_t floored = 0, saturated = 0;
    #pragma omp parallel reduction(+:floored, saturated)
    {
        float* F = (float*)malloc((size_t)lut_n * sizeof(float));
        float* Fd = (float*)malloc((size_t)lut_n * sizeof(float));
        uint8_t* stored = (uint8_t*)malloc((size_t)lut_n * 4);
        uint32_t* probes = (uint32_t*)malloc((size_t)n_probes * sizeof(uint32_t));
        #pragma omp for schedule(dynamic, 1)
        for (int64_t q = 0; q < nq; ++q) {
            const float* qv = queries + q * d;
            if (probes_in) memcpy(probes, probes_in + q * n_probes, (size_t)n_probes * sizeof(uint32_t));
            else orc_select_probes(centroids, n_lists, d, qv, 1, n_probes, probes, NULL);
            int64_t n_cand = 0;
            for (int p = 0; p < n_probes; ++p)
                n_cand += list_offsets[probes[p] + 1] - list_offsets[probes[p]];
            pair_f* cand = (pair_f*)malloc((size_t)(n_cand > 0 ? n_cand : 1) * sizeof(pair_f));
            int64_t at = 0;
            for (int p = 0; p < n_probes; ++p) {
                uint32_t l = probes[p];
                int64_t lo = list_offsets[l], len = list_offsets[l + 1] - lo;
                orc_lut_f32(qv, centroids + (int64_t)l * d, codebooks, d, pq_dim, ksub, F);
                (void)orc_lut_store(F, lut_n, lut_dtype, truncate, bias, per_table, bias_min, bias_max, stored, Fd);
                if (lut_dtype == ORC_LUT_E5M3 || lut_dtype == ORC_LUT_E4M4)
                    for (int64_t e = 0; e < lut_n; ++e) {
                        floored += stored[e] == 0x00; saturated += stored[e] == 0xFF;
                    }
                float* R = (float*)malloc((size_t)(len > 0 ? len : 1) * sizeof(float));
                orc_scan_list(Fd, pq_dim, pq_bits, codes + lo * code_bytes, len, R, NULL);
                for (int64_t i = 0; i < len; ++i) { cand[at].key = R[i]; cand[at].id = ids[lo + i]; ++at; }
                free(R);
            }
            qsort(cand, (size_t)n_cand, sizeof(pair_f), cmp_pair_f);
            for (int j = 0; j < k; ++j) {
                if (j < n_cand) { out_ids[q * k + j] = cand[j].id; out_d[q * k + j] = cand[j].key; }
                else            { out_ids[q * k + j] = -1;         out_d[q * k + j] = INFINITY; }
            }
            free(cand);
        }
        free(F); free(Fd); free(stored); free(probes);
    }
    if (stats) { stats[0] = floored; stats[1] = saturated; }
}

/* ------------------------------------------------------------------ */
/* Re-ranking of candidates with the original vectors (not in the paper; */
/* the usual companion of a PQ search: Eq. (1) only approximates          */
/* |q - x|^2, the stored vectors give it exactly).  For each query the     */
/* float64 squared distance of every candidate id >= 0 (an id is a row of  */
/* `data`), sorted by (distance, id), first k; padded with -1 / +inf.      */
/* A candidate listed twice is ranked twice.                               */
/* ------------------------------------------------------------------ */
void orc_refine(const float* data, int64_t n, int d, const float* queries, int64_t nq,
                const int64_t* cand_ids, int n_cand, int k, int64_t* out_ids, double* out_d) {
    (void)n;
    #pragma omp parallel
    {
        pair_d* buf = (pair_d*)malloc((size_t)(n_cand > 0 ? n_cand : 1) * sizeof(pair_d));
        #pragma omp for schedule(static)
        for (int64_t q = 0; q < nq; ++q) {
            int m = 0;
            for (int c = 0; c < n_cand; ++c) {
                int64_t id = cand_ids[q * n_cand + c];
                if (id < 0) continue;
                buf[m].key = sqdist_f64(queries + q * d, data + id * d, d);
                buf[m].id = id;
                ++m;
            }
            qsort(buf, (size_t)m, sizeof(pair_d), cmp_pair_d);
            for (int j = 0; j < k; ++j) {
                if (j < m) { out_ids[q * k + j] = buf[j].id; out_d[q * k + j] = buf[j].key; }
                else       { out_ids[q * k + j] = -1;        out_d[q * k + j] = INFINITY; }
            }
        }
        free(buf);
    }
}

int orc_lut_elem_bytes(int lut_dtype) { return lut_elem_bytes(lut_dtype); }
