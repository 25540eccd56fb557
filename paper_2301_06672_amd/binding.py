"""ctypes binding of libivfpq.so: argument marshalling only.

Function names mirror the C ABI in include/ivfpq.h.  PyTorch is used for device memory
(`torch.empty(..., device="cuda")`) and for the current HIP stream -- nothing is computed here.
There is no CPU fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np
import torch  # imported before the library so that both share one HIP runtime

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libivfpq.so")

LUT_FP32, LUT_FP16, LUT_FP8_E5M3, LUT_FP8_E4M4 = 0, 1, 2, 3
LUT_NAMES = {LUT_FP32: "fp32", LUT_FP16: "fp16", LUT_FP8_E5M3: "e5m3", LUT_FP8_E4M4: "e4m4"}
LUT_BYTES = {LUT_FP32: 4, LUT_FP16: 2, LUT_FP8_E5M3: 1, LUT_FP8_E4M4: 1}
ROUND_NEAREST, ROUND_TRUNCATE = 0, 1
MAX_K = 1024
MAX_PROBES = 1024
STATIC_SCRATCH_BYTES = 64 << 20
TUNE_SCAN_THREADS, TUNE_ORDER_BLOCK, TUNE_SCAN_SHARE, TUNE_EARLY_EXIT, TUNE_LDS_PAD = 0, 1, 2, 3, 4

OK, EINVAL, ENOSPACE, EHIP, EUNSUPPORTED, ESTATE = 0, -1, -2, -3, -4, -5

# every symbol include/ivfpq.h declares
EXPORTS = (
    "ivfpq_build_host", "ivfpq_build_device", "ivfpq_build_device_workspace_bytes", "ivfpq_assign_device",
    "ivfpq_assign_device_workspace_bytes", "ivfpq_index_from_arrays", "ivfpq_index_info", "ivfpq_index_export", "ivfpq_free",
    "ivfpq_set_e4m4_bias", "ivfpq_set_fp8_encoding", "ivfpq_set_workspace_limit", "ivfpq_set_tuning",
    "ivfpq_device_bytes", "ivfpq_upload", "ivfpq_search_workspace_bytes", "ivfpq_search", "ivfpq_search_static",
    "ivfpq_select_probes", "ivfpq_search_with_probes", "ivfpq_dump_lut", "ivfpq_scan_list", "ivfpq_refine",
    "ivfpq_set_stage_timing", "ivfpq_stage_times_ms", "ivfpq_scan_kernel_info", "ivfpq_stream_read", "ivfpq_last_error",
)


class IvfpqError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"ivfpq status {status}: {message}")
        self.status = status


_lib: Optional[ctypes.CDLL] = None


def lib() -> ctypes.CDLL:
    """Loads libivfpq.so (built by `python -m paper_2301_06672_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not found: build it with `python -m paper_2301_06672_amd.build` "
                "(there is no fallback implementation)")
        L = ctypes.CDLL(LIB_PATH)
        _declare(L)
        _lib = L
    return _lib


def _declare(L):
    c = ctypes
    vp, i64, i32, u32, u64, sz = c.c_void_p, c.c_int64, c.c_int32, c.c_uint32, c.c_uint64, c.c_size_t
    pp = c.POINTER(c.c_void_p)
    L.ivfpq_build_host.argtypes = [vp, i64, i32, i32, i32, i32, i32, u64, pp]
    L.ivfpq_build_device_workspace_bytes.argtypes = [i64, i32, i32, i32, i32, i64, i64]
    L.ivfpq_build_device_workspace_bytes.restype = sz
    L.ivfpq_build_device.argtypes = [vp, i64, i32, i32, i32, i32, i32, vp, i64, vp, vp, i64, vp, u64, vp, sz, vp, pp]
    L.ivfpq_assign_device_workspace_bytes.argtypes = [i64, i32, i32]
    L.ivfpq_assign_device_workspace_bytes.restype = sz
    L.ivfpq_assign_device.argtypes = [vp, i64, i32, vp, i32, vp, vp, sz, vp]
    L.ivfpq_index_from_arrays.argtypes = [i64, i32, i32, i32, i32, vp, vp, vp, vp, vp, pp]
    L.ivfpq_index_info.argtypes = [vp, c.POINTER(i64), c.POINTER(i32), c.POINTER(i32), c.POINTER(i32), c.POINTER(i32)]
    L.ivfpq_index_export.argtypes = [vp, vp, vp, vp, vp, vp]
    L.ivfpq_free.argtypes = [vp]
    L.ivfpq_set_e4m4_bias.argtypes = [vp, i32]
    L.ivfpq_set_workspace_limit.argtypes = [vp, sz]
    L.ivfpq_set_fp8_encoding.argtypes = [vp, i32, i32, i32, i32]
    L.ivfpq_set_tuning.argtypes = [vp, i32, i32]
    L.ivfpq_search_static.argtypes = [vp, vp, i64, i32, i32, i32, vp, vp, vp]
    L.ivfpq_free.restype = None
    L.ivfpq_device_bytes.argtypes = [vp]
    L.ivfpq_device_bytes.restype = sz
    L.ivfpq_upload.argtypes = [vp, vp, sz, vp]
    L.ivfpq_search_workspace_bytes.argtypes = [vp, i64, i32, i32, i32]
    L.ivfpq_search_workspace_bytes.restype = sz
    L.ivfpq_search.argtypes = [vp, vp, i64, i32, i32, i32, vp, vp, vp, sz, vp]
    L.ivfpq_select_probes.argtypes = [vp, vp, i64, i32, vp, vp, vp, sz, vp]
    L.ivfpq_search_with_probes.argtypes = [vp, vp, i64, vp, i32, i32, i32, vp, vp, vp, sz, vp]
    L.ivfpq_dump_lut.argtypes = [vp, vp, u32, i32, vp, vp]
    L.ivfpq_refine.argtypes = [vp, i64, i32, vp, i64, vp, i32, i32, vp, vp, vp]
    L.ivfpq_scan_list.argtypes = [vp, vp, u32, i32, vp, vp]
    L.ivfpq_set_stage_timing.argtypes = [vp, i32]
    L.ivfpq_stage_times_ms.argtypes = [vp, c.POINTER(c.c_float * 8)]
    L.ivfpq_scan_kernel_info.argtypes = [vp, i32, c.c_char_p, sz]
    L.ivfpq_stream_read.argtypes = [vp, sz, vp, i32, vp]
    L.ivfpq_last_error.restype = c.c_char_p
    for name in EXPORTS:
        fn = getattr(L, name)
        if fn.restype is c.c_int:      # default: status code
            fn.restype = c.c_int


def _check(status: int):
    if status != OK:
        raise IvfpqError(status, lib().ivfpq_last_error().decode("utf-8", "replace"))


def _np(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def _hp(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _dp(t: Optional[torch.Tensor]):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev_f32(x) -> torch.Tensor:
    if isinstance(x, torch.Tensor):
        assert x.is_cuda and x.dtype == torch.float32
        return x.contiguous()
    return torch.from_numpy(_np(x, np.float32)).cuda()


def ivfpq_assign_device(rows, centres) -> torch.Tensor:
    """-> int32 CUDA tensor: the nearest centre of every row (k-means assignment step)."""
    x, c = _dev_f32(rows), _dev_f32(centres)
    assert x.shape[1] == c.shape[1]
    need = lib().ivfpq_assign_device_workspace_bytes(int(x.shape[0]), int(x.shape[1]), int(c.shape[0]))
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
    labels = torch.empty(int(x.shape[0]), dtype=torch.int32, device="cuda")
    _check(lib().ivfpq_assign_device(_dp(x), int(x.shape[0]), int(x.shape[1]), _dp(c), int(c.shape[0]), _dp(labels),
                                     _dp(ws), need, _stream()))
    torch.cuda.current_stream().synchronize()
    return labels


def ivfpq_refine(data: torch.Tensor, queries, cand_ids: torch.Tensor, k: int):
    """-> (ids [nq][k] int64, dists [nq][k] fp32): candidates re-ranked by exact distance to rows of `data` (CUDA)."""
    assert data.is_cuda and data.dtype == torch.float32 and data.is_contiguous()
    q = _dev_f32(queries)
    cand = cand_ids.contiguous()
    assert cand.is_cuda and cand.dtype == torch.int64 and cand.shape[0] == q.shape[0]
    ids = torch.empty((q.shape[0], k), dtype=torch.int64, device="cuda")
    dists = torch.empty((q.shape[0], k), dtype=torch.float32, device="cuda")
    _check(lib().ivfpq_refine(_dp(data), int(data.shape[0]), int(data.shape[1]), _dp(q), int(q.shape[0]), _dp(cand),
                              int(cand.shape[1]), int(k), _dp(ids), _dp(dists), _stream()))
    return ids, dists


def ivfpq_stream_read(buf: torch.Tensor, n_out: int = 8192) -> torch.Tensor:
    """-> uint32-as-int32 [n_out]: per-workgroup XOR of the 32-bit words of `buf` (CUDA, size a multiple of 16 bytes)."""
    assert buf.is_cuda and buf.is_contiguous()
    out = torch.empty(n_out, dtype=torch.int32, device="cuda")
    _check(lib().ivfpq_stream_read(_dp(buf), buf.numel() * buf.element_size(), _dp(out), int(n_out), _stream()))
    return out


class Index:
    """Owns one ivfpq_index_t handle plus the torch tensors that back its device image and scratch."""

    def __init__(self, handle: ctypes.c_void_p):
        self._h = handle
        self._image: Optional[torch.Tensor] = None
        self._ws: Optional[torch.Tensor] = None
        n, d, nl, s, p = ctypes.c_int64(), ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
        _check(lib().ivfpq_index_info(self._h, n, d, nl, s, p))
        self.n, self.d, self.n_lists, self.pq_dim, self.pq_bits = n.value, d.value, nl.value, s.value, p.value

    # ---- construction
    @staticmethod
    def ivfpq_build_host(data, n_lists: int, pq_dim: int, pq_bits: int, kmeans_iters: int = 10, seed: int = 0) -> "Index":
        data = _np(data, np.float32)
        h = ctypes.c_void_p()
        _check(lib().ivfpq_build_host(_hp(data), data.shape[0], data.shape[1], n_lists, pq_dim, pq_bits,
                                      kmeans_iters, seed, ctypes.byref(h)))
        return Index(h)

    @staticmethod
    def ivfpq_build_device(data, n_lists: int, pq_dim: int, pq_bits: int, kmeans_iters: int = 10, seed: int = 0,
                           coarse_train_rows=None, coarse_init_rows=None, pq_train_rows=None,
                           pq_init_rows=None) -> "Index":
        """data: a CUDA tensor or a numpy array (copied to the device) [n][d] fp32."""
        x = _dev_f32(data)
        n, d = int(x.shape[0]), int(x.shape[1])
        opt = lambda a: None if a is None else _np(a, np.int64)
        ctr, cir, ptr, pir = opt(coarse_train_rows), opt(coarse_init_rows), opt(pq_train_rows), opt(pq_init_rows)
        n_ct = 0 if ctr is None else int(ctr.size)
        n_pt = 0 if ptr is None else int(ptr.size)
        if cir is not None:
            assert cir.size == n_lists
        if pir is not None:
            assert pir.size == pq_dim * (1 << pq_bits)
        need = lib().ivfpq_build_device_workspace_bytes(n, d, n_lists, pq_dim, pq_bits, n_ct, n_pt)
        if need == 0:
            raise IvfpqError(EINVAL, lib().ivfpq_last_error().decode("utf-8", "replace"))
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        h = ctypes.c_void_p()
        hp = lambda a: None if a is None else _hp(a)
        _check(lib().ivfpq_build_device(_dp(x), n, d, n_lists, pq_dim, pq_bits, kmeans_iters, hp(ctr), n_ct, hp(cir),
                                        hp(ptr), n_pt, hp(pir), seed, _dp(ws), need, _stream(), ctypes.byref(h)))
        del ws
        return Index(h)

    @staticmethod
    def ivfpq_index_from_arrays(d: int, n_lists: int, pq_dim: int, pq_bits: int, centroids, codebooks,
                                list_offsets, codes, ids) -> "Index":
        centroids, codebooks = _np(centroids, np.float32), _np(codebooks, np.float32)
        list_offsets, codes, ids = _np(list_offsets, np.int64), _np(codes, np.uint8), _np(ids, np.int64)
        ksub, m, cb = 1 << pq_bits, d // max(pq_dim, 1), pq_dim * pq_bits // 8
        n = int(ids.shape[0])
        assert centroids.size == n_lists * d and codebooks.size == pq_dim * ksub * m
        assert list_offsets.size == n_lists + 1 and codes.size == n * cb
        h = ctypes.c_void_p()
        _check(lib().ivfpq_index_from_arrays(n, d, n_lists, pq_dim, pq_bits, _hp(centroids), _hp(codebooks),
                                             _hp(list_offsets), _hp(codes), _hp(ids), ctypes.byref(h)))
        return Index(h)

    def ivfpq_index_export(self):
        ksub, m, cb = 1 << self.pq_bits, self.d // self.pq_dim, self.pq_dim * self.pq_bits // 8
        centroids = np.empty((self.n_lists, self.d), np.float32)
        codebooks = np.empty((self.pq_dim, ksub, m), np.float32)
        list_offsets = np.empty(self.n_lists + 1, np.int64)
        codes = np.empty((self.n, cb), np.uint8)
        ids = np.empty(self.n, np.int64)
        _check(lib().ivfpq_index_export(self._h, _hp(centroids), _hp(codebooks), _hp(list_offsets), _hp(codes), _hp(ids)))
        return centroids, codebooks, list_offsets, codes, ids

    def ivfpq_set_fp8_encoding(self, lut_dtype: int, bias: int, rounding: int = ROUND_NEAREST, per_table_bias: bool = False):
        _check(lib().ivfpq_set_fp8_encoding(self._h, int(lut_dtype), int(bias), int(rounding), int(per_table_bias)))

    def ivfpq_set_workspace_limit(self, nbytes: int):
        _check(lib().ivfpq_set_workspace_limit(self._h, int(nbytes)))
        self._ws = None

    def ivfpq_set_tuning(self, knob: int, value: int):
        _check(lib().ivfpq_set_tuning(self._h, int(knob), int(value)))

    def ivfpq_set_e4m4_bias(self, bias: int):
        _check(lib().ivfpq_set_e4m4_bias(self._h, int(bias)))

    def ivfpq_free(self):
        if self._h:
            lib().ivfpq_free(self._h)
            self._h = None
            self._image = None
            self._ws = None

    def __del__(self):
        try:
            self.ivfpq_free()
        except Exception:
            pass

    # ---- device residency
    def ivfpq_device_bytes(self) -> int:
        return int(lib().ivfpq_device_bytes(self._h))

    def ivfpq_upload(self) -> "Index":
        nbytes = self.ivfpq_device_bytes()
        self._image = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        _check(lib().ivfpq_upload(self._h, _dp(self._image), nbytes, _stream()))
        return self

    def ivfpq_search_workspace_bytes(self, nq: int, n_probes: int, k: int, lut_dtype: int) -> int:
        return int(lib().ivfpq_search_workspace_bytes(self._h, nq, n_probes, k, lut_dtype))

    def _workspace(self, nq, n_probes, k, lut_dtype) -> torch.Tensor:
        need = self.ivfpq_search_workspace_bytes(nq, n_probes, k, lut_dtype)
        if self._ws is None or self._ws.numel() < need:
            self._ws = None
            self._ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
        return self._ws

    # ---- search
    def ivfpq_search(self, queries, n_probes: int, k: int, lut_dtype: int = LUT_FP8_E5M3, out=None):
        q = _dev_f32(queries)
        nq = q.shape[0]
        ids, dists = out if out is not None else (
            torch.empty((nq, k), dtype=torch.int64, device="cuda"),
            torch.empty((nq, k), dtype=torch.float32, device="cuda"))
        ws = self._workspace(nq, n_probes, k, lut_dtype)
        _check(lib().ivfpq_search(self._h, _dp(q), nq, n_probes, k, lut_dtype, _dp(ids), _dp(dists),
                                  _dp(ws), ws.numel(), _stream()))
        return ids, dists

    def ivfpq_search_static(self, queries, n_probes: int, k: int, lut_dtype: int = LUT_FP8_E5M3, out=None):
        """ivfpq_search on the library's fixed scratch: no workspace is allocated or passed."""
        q = _dev_f32(queries)
        nq = q.shape[0]
        ids, dists = out if out is not None else (
            torch.empty((nq, k), dtype=torch.int64, device="cuda"),
            torch.empty((nq, k), dtype=torch.float32, device="cuda"))
        _check(lib().ivfpq_search_static(self._h, _dp(q), nq, n_probes, k, lut_dtype, _dp(ids), _dp(dists), _stream()))
        return ids, dists

    def ivfpq_select_probes(self, queries, n_probes: int):
        q = _dev_f32(queries)
        nq = q.shape[0]
        probes = torch.empty((nq, n_probes), dtype=torch.int32, device="cuda")   # u32 payload
        pd = torch.empty((nq, n_probes), dtype=torch.float32, device="cuda")
        ws = self._workspace(nq, n_probes, 1, LUT_FP32)
        _check(lib().ivfpq_select_probes(self._h, _dp(q), nq, n_probes, _dp(probes), _dp(pd), _dp(ws),
                                         ws.numel(), _stream()))
        return probes, pd

    def ivfpq_search_with_probes(self, queries, probes, k: int, lut_dtype: int = LUT_FP8_E5M3):
        q = _dev_f32(queries)
        nq = q.shape[0]
        if not isinstance(probes, torch.Tensor):
            probes = torch.from_numpy(_np(probes, np.uint32).view(np.int32)).cuda()
        probes = probes.contiguous()
        assert probes.is_cuda and probes.dtype == torch.int32 and probes.shape[0] == nq
        n_probes = probes.shape[1]
        ids = torch.empty((nq, k), dtype=torch.int64, device="cuda")
        dists = torch.empty((nq, k), dtype=torch.float32, device="cuda")
        ws = self._workspace(nq, n_probes, k, lut_dtype)
        _check(lib().ivfpq_search_with_probes(self._h, _dp(q), nq, _dp(probes), n_probes, k, lut_dtype,
                                              _dp(ids), _dp(dists), _dp(ws), ws.numel(), _stream()))
        return ids, dists

    def ivfpq_dump_lut(self, query, list_id: int, lut_dtype: int) -> torch.Tensor:
        q = _dev_f32(query).reshape(-1)
        nbytes = self.pq_dim * (1 << self.pq_bits) * LUT_BYTES[lut_dtype]
        out = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        _check(lib().ivfpq_dump_lut(self._h, _dp(q), list_id, lut_dtype, _dp(out), _stream()))
        return out

    def ivfpq_scan_list(self, query, list_id: int, lut_dtype: int, list_len: int) -> torch.Tensor:
        q = _dev_f32(query).reshape(-1)
        out = torch.empty(max(list_len, 1), dtype=torch.float32, device="cuda")
        _check(lib().ivfpq_scan_list(self._h, _dp(q), list_id, lut_dtype, _dp(out), _stream()))
        return out[:list_len]

    # ---- measurement aid
    def ivfpq_set_stage_timing(self, enabled: bool):
        _check(lib().ivfpq_set_stage_timing(self._h, int(enabled)))

    def ivfpq_scan_kernel_info(self, lut_dtype: int) -> str:
        buf = ctypes.create_string_buffer(256)
        _check(lib().ivfpq_scan_kernel_info(self._h, int(lut_dtype), buf, 256))
        return buf.value.decode()

    def ivfpq_stage_times_ms(self):
        ms = (ctypes.c_float * 8)()
        _check(lib().ivfpq_stage_times_ms(self._h, ctypes.byref(ms)))
        return {"probe_select": ms[0], "scan": ms[1], "topk": ms[2], "total": ms[3],
                "rank_gemm": ms[4], "scan_nearest_kernel": ms[5], "scan_filtered_kernel": ms[6]}
