/*
 * ivfpq.h -- C ABI of the MI355X (gfx950) IVFPQ search library.
 *
 * The library implements the search phase of IVFPQ as described in
 * arXiv 2301.06672, Sec. I-C (second enumeration) and Sec. I-D, with the
 * "norm2 fragment lookup table" held in LDS as fp32, IEEE half or one of the
 * paper's sign-less 8-bit floats, e5m3 and e4m4 (Sec. II).  All compute of the search runs in
 * hand-written HIP kernels; this header is the only interface.
 *
 * Conventions
 *  - Every function returns an ivfpq_status (0 = OK, negative = error); nothing
 *    throws across the ABI.  ivfpq_last_error() gives a text for the last
 *    non-OK return on the calling thread.
 *  - "host" pointers are ordinary CPU memory, "device" pointers are HIP device
 *    memory of the current device.  The caller owns every buffer it passes; the
 *    library never allocates or frees device memory.
 *  - Row-major everywhere.  Distances are squared L2 (Sec. I-B).
 *  - hip_stream is a hipStream_t passed as void* (NULL = the default stream).
 *    Search calls only enqueue work; they do not synchronise.
 *  - The library reads no environment variable; launch heuristics can be overridden per index with
 *    ivfpq_set_tuning (for tuning experiments and tests only).
 *  - No function throws: a C++ exception inside the library (host memory exhausted) comes back as a status.
 */
#ifndef IVFPQ_H
#define IVFPQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ivfpq_index ivfpq_index_t; /* opaque; created by build/import, destroyed by ivfpq_free */

/* Storage type of the lookup-table entries F(y_v) in LDS (Sec. I-D, Sec. II). */
typedef enum {
    IVFPQ_LUT_FP32 = 0,     /* IEEE binary32 */
    IVFPQ_LUT_FP16 = 1,     /* IEEE binary16, round-to-nearest-even, saturating at 65504 */
    IVFPQ_LUT_FP8_E5M3 = 2, /* 5 exponent + 3 mantissa bits, no sign, bias 15, all codes normal:
                               value(b) = (1 + (b&7)/8) * 2^((b>>3) - 15); FP32 -> code: nearest, ties up,
                               clamped to [0x00, 0xFF]; code -> FP32 bits: (b << 20) + 0x38000000 */
    IVFPQ_LUT_FP8_E4M4 = 3  /* the paper's other split, 4 exponent + 4 mantissa bits, same rules:
                               value(b) = (1 + (b&15)/16) * 2^((b>>4) - bias), 16 binades from 2^-bias;
                               the bias is set per index with ivfpq_set_e4m4_bias (default 7) */
} ivfpq_lut_dtype_t;

/* Rounding of the FP32 -> 8-bit encode (Sec. II: "shift the bit string and adjust the exponent bias";
 * whether the shift rounds is left open by the text). */
typedef enum {
    IVFPQ_ROUND_NEAREST = 0, /* nearest representable value, ties to the larger one (the default) */
    IVFPQ_ROUND_TRUNCATE = 1 /* the largest representable value not above the input: a bare shift */
} ivfpq_fp8_rounding_t;

typedef enum {
    IVFPQ_OK = 0,
    IVFPQ_EINVAL = -1,       /* null pointer, bad shape or parameter */
    IVFPQ_ENOSPACE = -2,     /* a caller buffer is smaller than the matching *_bytes() query says */
    IVFPQ_EHIP = -3,         /* a HIP runtime call failed (text in ivfpq_last_error) */
    IVFPQ_EUNSUPPORTED = -4, /* shape outside what the kernels handle (e.g. table does not fit LDS) */
    IVFPQ_ESTATE = -5        /* index not uploaded, or uploaded to another device */
} ivfpq_status;

enum { IVFPQ_MAX_K = 1024, IVFPQ_MAX_PROBES = 1024 };

/* ---- index construction (Sec. I-C, first enumeration; host side, not timed) ---- */

/* Builds an index on the host CPU: (1) Lloyd k-means with n_lists clusters (kmeans_iters
 * iterations, start rows drawn from `seed`), (2) residuals to the own centroid, (3) product
 * quantisation of the residuals: pq_dim contiguous sub-vectors of d/pq_dim components, one
 * codebook of 2^pq_bits entries per sub-space, (4) the saved lists, codes and codebook.
 * data: host [n][d] fp32.  Requires d % pq_dim == 0, 4 <= pq_bits <= 8 (the paper treats 8),
 * (pq_dim*pq_bits/8) % 4 == 0, 1 <= n_lists <= n.  *out receives the new handle. */
int ivfpq_build_host(const float* data, int64_t n, int32_t d, int32_t n_lists, int32_t pq_dim,
                     int32_t pq_bits, int32_t kmeans_iters, uint64_t seed, ivfpq_index_t** out);

/* The same four build steps on the GPU (current device).  d_data: device [n][d] fp32, n < 2^31.
 * Every decision (nearest cluster centre, nearest codeword) is the arg-min of float64 squared
 * distances, ties to the lower index; every centre is the float64 mean of its members summed in
 * ascending row order, rounded to fp32 once; an empty cluster keeps its centre.
 * The random draws are inputs (host arrays; each may be NULL, then it is drawn from `seed` as
 * ivfpq_build_host does):
 *   coarse_train_rows [n_coarse_train]  rows of d_data the cluster k-means trains on
 *                                       (NULL: <= 256 rows per list at a fixed stride)
 *   coarse_init_rows  [n_lists]         positions in that training set whose rows start the k-means
 *   pq_train_rows     [n_pq_train]      rows of d_data whose residuals train the codebooks
 *                                       (NULL: <= 262144 rows at a fixed stride); n_pq_train * pq_dim < 2^32
 *   pq_init_rows      [pq_dim][2^pq_bits]  positions in that training set, per sub-space
 * d_workspace: device scratch of >= ivfpq_build_device_workspace_bytes(...) (pass the two counts, or 0
 * for the defaults), 256-byte aligned.  Synchronises the stream before it returns; the resulting handle
 * holds the logical arrays on the host, as after ivfpq_build_host (call ivfpq_upload next). */
size_t ivfpq_build_device_workspace_bytes(int64_t n, int32_t d, int32_t n_lists, int32_t pq_dim, int32_t pq_bits,
                                          int64_t n_coarse_train, int64_t n_pq_train);
int ivfpq_build_device(const float* d_data, int64_t n, int32_t d, int32_t n_lists, int32_t pq_dim, int32_t pq_bits,
                       int32_t kmeans_iters, const int64_t* coarse_train_rows, int64_t n_coarse_train,
                       const int64_t* coarse_init_rows, const int64_t* pq_train_rows, int64_t n_pq_train,
                       const int64_t* pq_init_rows, uint64_t seed, void* d_workspace, size_t workspace_bytes,
                       void* hip_stream, ivfpq_index_t** out);

/* Build step 1's assignment alone, for inspection: d_labels[i] (device, int32) = the centre nearest to
 * row i of d_rows (device [n_rows][d]) among d_centres (device [n_centres][d]), decided as above.
 * d_workspace >= ivfpq_assign_device_workspace_bytes(n_rows, d, n_centres).  Asynchronous. */
size_t ivfpq_assign_device_workspace_bytes(int64_t n_rows, int32_t d, int32_t n_centres);
int ivfpq_assign_device(const float* d_rows, int64_t n_rows, int32_t d, const float* d_centres, int32_t n_centres,
                        int32_t* d_labels, void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* Imports the logical saved index (Sec. I-C build step 4).  All host pointers; the library copies.
 *   centroids    [n_lists][d] f32
 *   codebooks    [pq_dim][2^pq_bits][d/pq_dim] f32
 *   list_offsets [n_lists+1] i64, non-decreasing, [0] = 0, [n_lists] = n
 *   codes        [n][pq_dim*pq_bits/8] u8 in list order: the codes of a vector are one string of
 *                pq_dim*pq_bits bits, sub-space j in bits [j*p, (j+1)*p), bit i of the string = bit
 *                (i mod 8) of byte (i div 8).  pq_bits = 8: byte j = code of sub-space j; pq_bits = 4:
 *                byte j holds sub-space 2j in its low and 2j+1 in its high nibble
 *   ids          [n] i64 in list order (the caller's labels; returned by search) */
int ivfpq_index_from_arrays(int64_t n, int32_t d, int32_t n_lists, int32_t pq_dim, int32_t pq_bits,
                            const float* centroids, const float* codebooks, const int64_t* list_offsets,
                            const uint8_t* codes, const int64_t* ids, ivfpq_index_t** out);

/* Shape of an index; any out pointer may be NULL. */
int ivfpq_index_info(const ivfpq_index_t* index, int64_t* n, int32_t* d, int32_t* n_lists,
                     int32_t* pq_dim, int32_t* pq_bits);

/* Copies the logical arrays (same layout as ivfpq_index_from_arrays) into caller host buffers of
 * the sizes ivfpq_index_info implies; any pointer may be NULL to skip that array. */
int ivfpq_index_export(const ivfpq_index_t* index, float* centroids, float* codebooks,
                       int64_t* list_offsets, uint8_t* codes, int64_t* ids);

/* Encoding of one of the two 8-bit table dtypes (lut_dtype = IVFPQ_LUT_FP8_E5M3 or _E4M4) for searches
 * on this index; takes effect at the next call.  Defaults: bias 15 (e5m3) / 7 (e4m4), nearest, fixed.
 *   bias            exponent bias B of the format: value(b) = (1 + mant/2^M) * 2^(exp - B).  Moving the
 *                   bias by s is a scale of the table by 2^s before the encode and 2^-s after the
 *                   decode; returned distances are always in the data's own units.
 *                   -96 <= B <= 110 (e5m3), -100 <= B <= 110 (e4m4): every code a normal FP32 number.
 *   rounding        an ivfpq_fp8_rounding_t
 *   per_table_bias  0: `bias` for every table.  1: per (query, cluster) table, the bias that puts the
 *                   binade of the table's largest entry on the format's top binade (with e the FP32
 *                   exponent of that entry, B = 31 - e for e5m3, 15 - e for e4m4, clamped to the range
 *                   above); `bias` is ignored.  Costs a second pass over the table's entries. */
int ivfpq_set_fp8_encoding(ivfpq_index_t* index, int32_t lut_dtype, int32_t bias, int32_t rounding,
                           int32_t per_table_bias);

/* Shorthand: sets only the exponent bias of the IVFPQ_LUT_FP8_E4M4 table dtype for searches on this index (Sec. II gives the
 * 4+4 split but not its bias): representable table values are 2^-bias .. 1.9375 * 2^(15-bias); what
 * falls outside is clamped to the nearest end.  -100 <= bias <= 110.  Takes effect at the next call. */
int ivfpq_set_e4m4_bias(ivfpq_index_t* index, int32_t bias);

void ivfpq_free(ivfpq_index_t* index);

/* ---- device residency ---- */

/* Bytes of device memory the uploaded index needs (lists are padded to 64 vectors and the codes
 * re-laid out for coalesced wave64 loads; see ivfpq_upload). */
size_t ivfpq_device_bytes(const ivfpq_index_t* index);

/* Writes the device image of the index into d_buf (device, >= ivfpq_device_bytes, 256-byte aligned)
 * on the current device and remembers the pointer.  Synchronous.  d_buf must stay alive and
 * unmodified while the handle is used for searches. */
int ivfpq_upload(ivfpq_index_t* index, void* d_buf, size_t bytes, void* hip_stream);

/* Bytes of device scratch one search call needs for these parameters (probe lists, per-pair
 * descriptors, cluster ranking values, the R rows and the positions of filtered candidates).
 * Large batches are processed in query tiles so that the figure stays near the index's workspace
 * limit (one query's share can exceed it: a tile holds at least one query). */
size_t ivfpq_search_workspace_bytes(const ivfpq_index_t* index, int64_t nq, int32_t n_probes,
                                    int32_t k, int32_t lut_dtype);

/* Overrides one launch heuristic of searches on this index (tuning experiments, tests); value 0 restores
 * the library's own choice.  No knob changes any result.  Takes effect at the next call. */
typedef enum {
    IVFPQ_TUNE_SCAN_THREADS = 0, /* workgroup size of the scan kernels: 64, 128, 256, 512 or 1024 */
    IVFPQ_TUNE_ORDER_BLOCK = 1,  /* consecutive (query, probe) pairs of the cluster-grouped order that stay on one
                                    XCD (>= 1; the scan that shares a workgroup between pairs needs an even value) */
    IVFPQ_TUNE_SCAN_SHARE = 2,   /* 1: one (query, probe) pair per scan workgroup; 2 or 4: up to that many pairs of
                                    one cluster per workgroup wherever the kernel for it applies (8- and 4-bit codes) */
    IVFPQ_TUNE_EARLY_EXIT = 3,   /* 1: on (the default: a 64-vector group stops adding once all its partial sums are
                                    over the query's bound); -1: off, every lookup of Eq. (1) is made */
    IVFPQ_TUNE_LDS_PAD = 4       /* extra bytes of LDS requested per scan workgroup (lowers occupancy without
                                    changing the table: separates the two effects of a smaller table dtype) */
} ivfpq_tuning_t;
int ivfpq_set_tuning(ivfpq_index_t* index, int32_t knob, int32_t value);

/* The workspace limit of searches on this index, in bytes (default 32 GiB; at least 1 MiB).  A query's
 * share of the scratch is sized for the worst case (every vector of its n_probes largest clusters kept),
 * so big indexes split a batch into tiles; fewer, larger tiles run faster (measured: 10,000 queries on
 * 10^8 vectors take 15.3 ms with 2 GiB, 14.0 ms with 8 GiB, 13.5 ms with 32 GiB), smaller limits suit
 * many concurrent callers.  Takes effect at the next ivfpq_search_workspace_bytes / search call. */
int ivfpq_set_workspace_limit(ivfpq_index_t* index, size_t bytes);

/* ---- search (Sec. I-C, second enumeration, steps 1-5) ---- */

/* For each of nq queries: picks the n_probes clusters with the nearest centroids (step 1), and for
 * each picked cluster forms the query residual (step 2), builds the lookup table F in LDS in
 * lut_dtype (step 3), accumulates R = sum_j F(y_j) (Eq. 1) over every coded vector of the cluster
 * (step 4); then keeps the k smallest R over all picked clusters (step 5).
 *   d_queries [nq][d] f32 (device)          d_ids [nq][k] i64 (device, out)
 *   d_dists   [nq][k] f32 (device, out): R of the returned vectors, ascending; ties ordered by id.
 * Rows with fewer than k candidates are padded with id -1, distance +inf.
 * 1 <= n_probes <= min(n_lists, IVFPQ_MAX_PROBES), 1 <= k <= IVFPQ_MAX_K.
 * d_workspace: device scratch of >= ivfpq_search_workspace_bytes(...), 256-byte aligned; calls that
 * may overlap in time need distinct workspaces. */
int ivfpq_search(const ivfpq_index_t* index, const float* d_queries, int64_t nq, int32_t n_probes,
                 int32_t k, int32_t lut_dtype, int64_t* d_ids, float* d_dists,
                 void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* ivfpq_search for callers that cannot allocate device memory or provide a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and kernels as
 * ivfpq_search, but the scratch is a fixed array of IVFPQ_STATIC_SCRATCH_BYTES inside the library's device
 * image (each GPU the library runs on holds it until the process ends); the call allocates and frees nothing.
 * A batch is processed in as many query tiles as the array requires; if a single query's share does not fit
 * (its n_probes largest clusters hold too many vectors) the call returns IVFPQ_ENOSPACE and touches nothing.
 * All calls on one GPU share that GPU's array, whatever the index or stream: calls that overlap in time race,
 * so issue them on one stream or order them yourself.  Nothing in the array needs to survive between calls. */
#define IVFPQ_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
int ivfpq_search_static(const ivfpq_index_t* index, const float* d_queries, int64_t nq, int32_t n_probes,
                        int32_t k, int32_t lut_dtype, int64_t* d_ids, float* d_dists, void* hip_stream);

/* Step 1 alone: d_probes [nq][n_probes] u32 (device, out), nearest first, ties to the lower
 * cluster index; d_probe_dists [nq][n_probes] f32 (device, out, may be NULL). */
int ivfpq_select_probes(const ivfpq_index_t* index, const float* d_queries, int64_t nq,
                        int32_t n_probes, uint32_t* d_probes, float* d_probe_dists,
                        void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* Steps 2-5 on caller-chosen clusters: d_probes [nq][n_probes] u32 (device, in), every entry
 * < n_lists; a cluster listed twice for one query is scanned twice. */
int ivfpq_search_with_probes(const ivfpq_index_t* index, const float* d_queries, int64_t nq,
                             const uint32_t* d_probes, int32_t n_probes, int32_t k, int32_t lut_dtype,
                             int64_t* d_ids, float* d_dists,
                             void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* Steps 2-3 alone, for inspection: builds the table of one (query, cluster) pair exactly as the
 * search kernel stages it in LDS and copies the raw bytes out.
 * d_query [d] f32 (device); d_lut_out (device) [pq_dim][2^pq_bits] entries of lut_dtype,
 * i.e. pq_dim * 2^pq_bits * {4, 2, 1, 1} bytes for the four dtypes. */
int ivfpq_dump_lut(const ivfpq_index_t* index, const float* d_query, uint32_t list_id,
                   int32_t lut_dtype, void* d_lut_out, void* hip_stream);

/* Step 4 alone, for inspection: R of every coded vector of one cluster for one query, in list
 * order.  d_R_out (device) [list length] f32. */
int ivfpq_scan_list(const ivfpq_index_t* index, const float* d_query, uint32_t list_id,
                    int32_t lut_dtype, float* d_R_out, void* hip_stream);

/* ---- re-ranking with the stored vectors (not part of the paper's path; the usual companion of a PQ
 * search, whose Eq. (1) only approximates |q - x|^2) ---- */

/* For each of nq queries: the exact squared distance (fp32, direct form) to each of its n_cand candidate
 * vectors, and the k smallest, ascending, ties ordered by id.  A candidate id is a row of d_data
 * (device [n_data][d] fp32: the vectors the index was built from, when their ids are their row numbers);
 * ids outside [0, n_data) -- the -1 padding of a search result -- are skipped; an id listed twice is
 * ranked twice.  d_cand_ids [nq][n_cand] i64 (device), e.g. the ids of ivfpq_search with a larger k.
 * d_ids [nq][k] i64, d_dists [nq][k] f32 (device, out); short rows are padded with -1 / +inf.
 * 1 <= n_cand <= IVFPQ_MAX_K, 1 <= k <= IVFPQ_MAX_K.  Asynchronous; needs no workspace. */
int ivfpq_refine(const float* d_data, int64_t n_data, int32_t d, const float* d_queries, int64_t nq,
                 const int64_t* d_cand_ids, int32_t n_cand, int32_t k, int64_t* d_ids, float* d_dists,
                 void* hip_stream);

/* ---- measurement aid ---- */

/* When enabled, search calls record HIP events around their stages on the stream they run on (the events
 * and their bookkeeping live in the handle: while enabled, search calls on one index must not overlap).
 * After the stream has been synchronised, ivfpq_stage_times_ms reports the last call's
 * milliseconds, summed over query tiles: ms[0] = probe selection (step 1: ranking GEMM + selection),
 * ms[1] = table build + code scan (steps 2-4: the scan kernel over the nearest probe, the bound kernel,
 * the grouping of the other pairs by cluster, the scan kernel over the remaining probes), ms[2] = top-k
 * (step 5), ms[3] = whole call; and single launches inside those stages: ms[4] = the ranking GEMM of
 * step 1, ms[5] = the scan kernel over the nearest probes, ms[6] = the scan kernel over the remaining
 * probes (the dominant kernel), ms[7] = 0 (reserved). */
int ivfpq_set_stage_timing(ivfpq_index_t* index, int32_t enabled);
int ivfpq_stage_times_ms(ivfpq_index_t* index, float ms[8]);

/* Writes into buf (host, buf_bytes > 0, always terminated) the name, workgroup size and LDS request of the
 * kernel that scans the probes other than the nearest one (the dominant kernel of a search) for this index,
 * table dtype and current tuning: what to look for in a profiler's kernel list. */
int ivfpq_scan_kernel_info(const ivfpq_index_t* index, int32_t lut_dtype, char* buf, size_t buf_bytes);

/* Measurement aid, not a step of the method: a plain streaming read of `bytes` bytes of device memory
 * (16-byte loads, grid-strided, n_out workgroups of 256 threads), the achievable HBM read rate that a
 * code scan (Sec. I-C, search step 4, Eq. 1) streaming every byte from HBM is priced against.  d_buf: device,
 * 16-byte aligned, bytes a multiple of 16; d_out: device, n_out words (1..65536), word b = XOR of all
 * 32-bit words workgroup b read.  Asynchronous on hip_stream; allocates nothing. */
int ivfpq_stream_read(const void* d_buf, size_t bytes, uint32_t* d_out, int32_t n_out, void* hip_stream);

const char* ivfpq_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* IVFPQ_H */
