"""CPU oracle for the IVFPQ build and search phases -- TEST INFRASTRUCTURE.

Thin ctypes wrapper over `oracle/ivfpq_oracle.c` plus the few numpy steps that
glue its primitives into the index build of Sec. I-C.  Only `tests/`, the smoke
check and the benchmark's cpu_baseline leg may import this package; the HIP
library never does, and this package never imports the library.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np

from .build import build as _build, LIB_PATH, SRC as _SRC

LUT_FP32, LUT_FP16, LUT_E5M3, LUT_E4M4 = 0, 1, 2, 3
LUT_NAMES = {LUT_FP32: "fp32", LUT_FP16: "fp16", LUT_E5M3: "e5m3", LUT_E4M4: "e4m4"}

_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if (not os.path.exists(LIB_PATH)
                or os.path.getmtime(LIB_PATH) < os.path.getmtime(_SRC)):
            _build()
        _lib = ctypes.CDLL(LIB_PATH)
        _declare(_lib)
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _declare(L):
    c = ctypes
    vp, i64, i32, f32, f64 = c.c_void_p, c.c_int64, c.c_int, c.c_float, c.c_double
    L.orc_num_threads.restype = i32
    L.orc_set_num_threads.argtypes = [i32]
    L.orc_exact_knn.argtypes = [vp, i64, i32, vp, i64, i32, vp, vp]
    L.orc_assign.argtypes = [vp, i64, i32, vp, i32, vp]
    L.orc_assign.restype = f64
    L.orc_kmeans.argtypes = [vp, i64, i32, i32, i32, vp, vp, vp]
    L.orc_fp8_value.argtypes = [i32, i32, i32]
    L.orc_fp8_value.restype = f64
    L.orc_e5m3_encode.argtypes = [f32, i32]
    L.orc_e5m3_encode.restype = c.c_uint8
    L.orc_e5m3_decode.argtypes = [c.c_uint8]
    L.orc_e5m3_decode.restype = f32
    L.orc_fp16_encode.argtypes = [f32]
    L.orc_fp16_encode.restype = c.c_uint16
    L.orc_fp16_decode.argtypes = [c.c_uint16]
    L.orc_fp16_decode.restype = f32
    L.orc_e5m3_encode_array.argtypes = [vp, i64, i32, vp]
    L.orc_e5m3_decode_array.argtypes = [vp, i64, vp]
    L.orc_fp8_encode_array.argtypes = [vp, i64, i32, i32, i32, vp]
    L.orc_fp8_decode_array.argtypes = [vp, i64, i32, i32, vp]
    L.orc_fp16_encode_array.argtypes = [vp, i64, vp]
    L.orc_fp16_decode_array.argtypes = [vp, i64, vp]
    L.orc_select_probes.argtypes = [vp, i32, i32, vp, i64, i32, vp, vp]
    L.orc_lut_f32.argtypes = [vp, vp, vp, i32, i32, i32, vp]
    L.orc_lut_store.argtypes = [vp, i64, i32, i32, i32, i32, i32, i32, vp, vp]
    L.orc_lut_store.restype = i32
    L.orc_fp8_table_bias.argtypes = [vp, i64, i32, i32, i32]
    L.orc_fp8_table_bias.restype = i32
    L.orc_scan_list.argtypes = [vp, i32, i32, vp, i64, vp, vp]
    L.orc_search.argtypes = [i64, i32, i32, i32, i32, vp, vp, vp, vp, vp,
                             vp, i64, i32, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp]
    L.orc_lut_elem_bytes.argtypes = [i32]
    L.orc_refine.argtypes = [vp, i64, i32, vp, i64, vp, i32, i32, vp, vp]
    L.orc_lut_elem_bytes.restype = i32


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


# ---------------------------------------------------------------- number formats (Sec. II)

def e5m3_encode(x, truncate: bool = False) -> np.ndarray:
    x = _f32(np.atleast_1d(x))
    out = np.empty(x.shape, dtype=np.uint8)
    lib().orc_e5m3_encode_array(_p(x), x.size, int(truncate), _p(out))
    return out


def e5m3_decode(b) -> np.ndarray:
    b = np.ascontiguousarray(np.atleast_1d(b), dtype=np.uint8)
    out = np.empty(b.shape, dtype=np.float32)
    lib().orc_e5m3_decode_array(_p(b), b.size, _p(out))
    return out


def fp8_encode(x, mant_bits: int, bias: int, truncate: bool = False) -> np.ndarray:
    x = _f32(np.atleast_1d(x))
    out = np.empty(x.shape, dtype=np.uint8)
    lib().orc_fp8_encode_array(_p(x), x.size, mant_bits, bias, int(truncate), _p(out))
    return out


def fp8_decode(b, mant_bits: int, bias: int) -> np.ndarray:
    b = np.ascontiguousarray(np.atleast_1d(b), dtype=np.uint8)
    out = np.empty(b.shape, dtype=np.float32)
    lib().orc_fp8_decode_array(_p(b), b.size, mant_bits, bias, _p(out))
    return out


def fp16_encode(x) -> np.ndarray:
    x = _f32(np.atleast_1d(x))
    out = np.empty(x.shape, dtype=np.uint16)
    lib().orc_fp16_encode_array(_p(x), x.size, _p(out))
    return out


def fp16_decode(h) -> np.ndarray:
    h = np.ascontiguousarray(np.atleast_1d(h), dtype=np.uint16)
    out = np.empty(h.shape, dtype=np.float32)
    lib().orc_fp16_decode_array(_p(h), h.size, _p(out))
    return out


# ---------------------------------------------------------------- exact k-NN (Sec. I-B)

def exact_knn(data, queries, k: int):
    data, queries = _f32(data), _f32(queries)
    n, d = data.shape
    nq = queries.shape[0]
    ids = np.empty((nq, k), dtype=np.int64)
    d2 = np.empty((nq, k), dtype=np.float64)
    lib().orc_exact_knn(_p(data), n, d, _p(queries), nq, k, _p(ids), _p(d2))
    return ids, d2


def recall(found_ids: np.ndarray, true_ids: np.ndarray) -> float:
    """|V intersect V_GT| / |V_GT| averaged over queries (Sec. I-B)."""
    hits = 0
    for f, t in zip(found_ids, true_ids):
        hits += len(set(int(v) for v in f if v >= 0) & set(int(v) for v in t))
    return hits / float(true_ids.size)


# ---------------------------------------------------------------- k-means (Sec. I-C, build step 1)

def assign(x, centres):
    x, centres = _f32(x), _f32(centres)
    labels = np.empty(x.shape[0], dtype=np.int32)
    total = lib().orc_assign(_p(x), x.shape[0], x.shape[1], _p(centres), centres.shape[0], _p(labels))
    return labels, total


def kmeans(x, n_centres: int, iters: int, init_rows):
    x = _f32(x)
    init_rows = np.ascontiguousarray(init_rows, dtype=np.int64)
    assert init_rows.shape == (n_centres,)
    centres = np.empty((n_centres, x.shape[1]), dtype=np.float32)
    inertia = np.empty(max(iters, 1), dtype=np.float64)
    lib().orc_kmeans(_p(x), x.shape[0], x.shape[1], n_centres, iters, _p(init_rows), _p(centres), _p(inertia))
    return centres, inertia[:iters]


# ---------------------------------------------------------------- the saved index (Sec. I-C, build step 4)

@dataclass
class Index:
    """The logical saved index: cluster membership, PQ codes, PQ codebook."""
    d: int
    n_lists: int
    pq_dim: int
    pq_bits: int
    centroids: np.ndarray      # [n_lists][d] f32
    codebooks: np.ndarray      # [pq_dim][2^pq_bits][d/pq_dim] f32
    list_offsets: np.ndarray   # [n_lists+1] i64
    codes: np.ndarray          # [n][pq_dim*pq_bits/8] u8, list order
    ids: np.ndarray            # [n] i64, list order

    @property
    def n(self) -> int:
        return int(self.ids.shape[0])

    @property
    def ksub(self) -> int:
        return 1 << self.pq_bits

    @property
    def m(self) -> int:
        return self.d // self.pq_dim


def make_index(d, n_lists, pq_dim, pq_bits, centroids, codebooks, list_offsets, codes, ids) -> Index:
    return Index(d, n_lists, pq_dim, pq_bits, _f32(centroids), _f32(codebooks),
                 np.ascontiguousarray(list_offsets, dtype=np.int64),
                 np.ascontiguousarray(codes, dtype=np.uint8),
                 np.ascontiguousarray(ids, dtype=np.int64))


def pack_codes(codes_per_subspace: np.ndarray, pq_bits: int) -> np.ndarray:
    """[n][pq_dim] code values -> [n][pq_dim*pq_bits/8] bytes: sub-space j in bits [j*p, (j+1)*p) of
    the vector's bit string, least significant bit first inside every byte (p=8: one byte per
    sub-space; p=4: low nibble = even sub-space, high nibble = odd sub-space)."""
    c = np.ascontiguousarray(codes_per_subspace, dtype=np.uint8)
    assert 4 <= pq_bits <= 8 and (c.shape[1] * pq_bits) % 8 == 0
    bits = (c[:, :, None] >> np.arange(pq_bits, dtype=np.uint8)[None, None, :]) & 1      # [n][pq_dim][p], LSB first
    return np.packbits(bits.reshape(c.shape[0], -1), axis=1, bitorder="little")


def unpack_codes(packed: np.ndarray, pq_bits: int) -> np.ndarray:
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    bits = np.unpackbits(packed, axis=1, bitorder="little")
    pq_dim = bits.shape[1] // pq_bits
    bits = bits[:, :pq_dim * pq_bits].reshape(packed.shape[0], pq_dim, pq_bits)
    return (bits << np.arange(pq_bits, dtype=np.uint8)[None, None, :]).sum(axis=2).astype(np.uint8)


def build_index(data, n_lists: int, pq_dim: int, pq_bits: int, kmeans_iters: int,
                coarse_init_rows, pq_init_rows, coarse_train_rows=None, pq_train_rows=None) -> Index:
    """Index build of Sec. I-C: (1) k-means clusters, (2) residuals to the own
    centroid, (3) product quantisation of the residuals, one codebook per
    sub-space of d/pq_dim contiguous components, (4) the saved arrays.

    coarse_init_rows: [n_lists] rows of the coarse training set; pq_init_rows:
    [pq_dim][2^pq_bits] rows of the PQ training set (the random draws are inputs).
    *_train_rows: row subsets used for training (None = all rows)."""
    data = _f32(data)
    n, d = data.shape
    m = d // pq_dim
    ksub = 1 << pq_bits
    train = data if coarse_train_rows is None else data[np.asarray(coarse_train_rows)]
    centroids, _ = kmeans(train, n_lists, kmeans_iters, coarse_init_rows)
    labels, _ = assign(data, centroids)                       # membership of every row
    residual = data - centroids[labels]                        # fp32, step 2
    rtrain = residual if pq_train_rows is None else residual[np.asarray(pq_train_rows)]
    codebooks = np.empty((pq_dim, ksub, m), dtype=np.float32)
    sub_codes = np.empty((n, pq_dim), dtype=np.uint8)
    pq_init_rows = np.asarray(pq_init_rows)
    for j in range(pq_dim):
        sub_train = np.ascontiguousarray(rtrain[:, j * m:(j + 1) * m])
        codebooks[j], _ = kmeans(sub_train, ksub, kmeans_iters, pq_init_rows[j])
        sub_all = np.ascontiguousarray(residual[:, j * m:(j + 1) * m])
        sub_codes[:, j] = assign(sub_all, codebooks[j])[0].astype(np.uint8)
    order = np.argsort(labels, kind="stable")                  # list order, ascending id inside a list
    counts = np.bincount(labels, minlength=n_lists)
    list_offsets = np.zeros(n_lists + 1, dtype=np.int64)
    np.cumsum(counts, out=list_offsets[1:])
    codes = pack_codes(sub_codes[order], pq_bits)
    return make_index(d, n_lists, pq_dim, pq_bits, centroids, codebooks, list_offsets, codes,
                      order.astype(np.int64))


# ---------------------------------------------------------------- search (Sec. I-C, search steps 1-5)

def select_probes(index: Index, queries, n_probes: int):
    queries = _f32(queries)
    nq = queries.shape[0]
    probes = np.empty((nq, n_probes), dtype=np.uint32)
    d2 = np.empty((nq, n_probes), dtype=np.float64)
    lib().orc_select_probes(_p(index.centroids), index.n_lists, index.d, _p(queries), nq, n_probes,
                            _p(probes), _p(d2))
    return probes, d2


def lut_f32(index: Index, query, list_id: int) -> np.ndarray:
    """F[pq_dim][2^pq_bits] in fp32 for one (query, cluster) pair (search steps 2-3)."""
    query = _f32(query)
    F = np.empty((index.pq_dim, index.ksub), dtype=np.float32)
    centroid = np.ascontiguousarray(index.centroids[list_id])
    lib().orc_lut_f32(_p(query), _p(centroid), _p(index.codebooks), index.d, index.pq_dim, index.ksub, _p(F))
    return F


# Range of the exponent bias of the two 8-bit formats (every code stays a finite, normal FP32 number)
FP8_BIAS_RANGE = {2: (-96, 110), 3: (-100, 110)}
FP8_DEFAULT_BIAS = {2: 15, 3: 7}


def _fp8_bias(lut_dtype: int, bias, e4m4_bias: int) -> int:
    if bias is not None:
        return int(bias)
    return int(e4m4_bias) if lut_dtype == LUT_E4M4 else FP8_DEFAULT_BIAS.get(lut_dtype, 0)


def fp8_table_bias(F: np.ndarray, lut_dtype: int) -> int:
    """Exponent bias that puts the binade of the table's largest entry on the format's top binade."""
    F = _f32(F)
    lo, hi = FP8_BIAS_RANGE[lut_dtype]
    return int(lib().orc_fp8_table_bias(_p(F), F.size, 5 if lut_dtype == LUT_E5M3 else 4, lo, hi))


def lut_store(F: np.ndarray, lut_dtype: int, truncate: bool = False, e4m4_bias: int = 7, bias=None,
              per_table: bool = False, return_bias: bool = False):
    """-> (bytes as stored on chip, decoded fp32 values a lookup returns).

    bias: exponent bias of the 8-bit format in use (default 15 for e5m3, e4m4_bias for e4m4);
    per_table: choose the bias from the table's largest entry instead (power-of-two table scaling)."""
    F = _f32(F)
    eb = lib().orc_lut_elem_bytes(lut_dtype)
    stored = np.empty(F.size * eb, dtype=np.uint8)
    decoded = np.empty(F.shape, dtype=np.float32)
    lo, hi = FP8_BIAS_RANGE.get(lut_dtype, (0, 0))
    used = lib().orc_lut_store(_p(F), F.size, lut_dtype, int(truncate), _fp8_bias(lut_dtype, bias, e4m4_bias),
                               int(per_table), lo, hi, _p(stored), _p(decoded))
    if return_bias:
        return stored, decoded, int(used)
    return stored, decoded


def scan_list(index: Index, lut_decoded: np.ndarray, list_id: int):
    """Eq. (1) for every coded vector of one cluster -> (R fp32, R float64 shadow)."""
    lo, hi = int(index.list_offsets[list_id]), int(index.list_offsets[list_id + 1])
    codes = np.ascontiguousarray(index.codes[lo:hi])
    lut_decoded = _f32(lut_decoded)
    R = np.empty(hi - lo, dtype=np.float32)
    R64 = np.empty(hi - lo, dtype=np.float64)
    lib().orc_scan_list(_p(lut_decoded), index.pq_dim, index.pq_bits, _p(codes), hi - lo, _p(R), _p(R64))
    return R, R64


def search(index: Index, queries, n_probes: int, k: int, lut_dtype: int = LUT_FP32,
           truncate: bool = False, probes=None, return_stats: bool = False, e4m4_bias: int = 7, bias=None,
           per_table: bool = False):
    queries = _f32(queries)
    nq = queries.shape[0]
    out_ids = np.empty((nq, k), dtype=np.int64)
    out_d = np.empty((nq, k), dtype=np.float32)
    stats = np.zeros(2, dtype=np.int64)
    pr = None
    if probes is not None:
        pr = np.ascontiguousarray(probes, dtype=np.uint32)
        assert pr.shape == (nq, n_probes)
    lib().orc_search(index.n, index.d, index.n_lists, index.pq_dim, index.pq_bits,
                     _p(index.centroids), _p(index.codebooks), _p(index.list_offsets),
                     _p(index.codes), _p(index.ids), _p(queries), nq, n_probes, k,
                     lut_dtype, int(truncate), _fp8_bias(lut_dtype, bias, e4m4_bias), int(per_table),
                     *FP8_BIAS_RANGE.get(lut_dtype, (0, 0)), _p(pr) if pr is not None else None,
                     _p(out_ids), _p(out_d), _p(stats))
    if return_stats:
        return out_ids, out_d, {"floored": int(stats[0]), "saturated": int(stats[1])}
    return out_ids, out_d


def refine(data, queries, cand_ids, k: int):
    """Exact re-ranking: float64 distances of the candidate rows, the k smallest by (distance, id)."""
    data, queries = _f32(data), _f32(queries)
    cand = np.ascontiguousarray(cand_ids, dtype=np.int64)
    nq, n_cand = cand.shape
    assert queries.shape[0] == nq and (cand < data.shape[0]).all()
    out_ids = np.empty((nq, k), dtype=np.int64)
    out_d = np.empty((nq, k), dtype=np.float64)
    lib().orc_refine(_p(data), data.shape[0], data.shape[1], _p(queries), nq, _p(cand), n_cand, k, _p(out_ids), _p(out_d))
    return out_ids, out_d


def num_threads() -> int:
    return int(lib().orc_num_threads())


def set_num_threads(n: int) -> None:
    lib().orc_set_num_threads(int(n))
