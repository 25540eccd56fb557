"""CPU-only checks of libivfpq.so: it loads, exports every symbol the header declares, and its
host-side logic (import/export, validation, the CPU index builder) behaves.  No kernel is
launched here."""
import os
import re

import numpy as np
import pytest

import oracle
import synth_inputs as si

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def P():
    import paper_2301_06672_amd as pkg
    if not os.path.exists(pkg.LIB_PATH):
        from paper_2301_06672_amd.build import build
        build()
    pkg.lib()
    return pkg


def test_library_exports_every_declared_symbol(P):
    header = open(os.path.join(ROOT, "include", "ivfpq.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(ivfpq_[a-z_0-9]+)\s*\(", header))
    assert declared == set(P.EXPORTS)
    L = P.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_header_is_plain_c_and_links(P, tmp_path):
    # strict C99 compile of a translation unit that uses the header, then a link against the library
    import subprocess
    src = os.path.join(ROOT, "tests", "abi_smoke.c")
    obj = str(tmp_path / "abi_smoke.o")
    subprocess.run(["gcc", "-std=c99", "-pedantic-errors", "-Wall", "-Werror", "-c", src, "-o", obj], check=True)
    so = str(tmp_path / "libabi_smoke.so")
    subprocess.run(["gcc", "-shared", "-o", so, obj, P.LIB_PATH], check=True)


def test_import_export_round_trip(P):
    arrays = si.random_index_arrays(777, 32, 9, 16, 4, salt=1, empty_lists=(3,))
    idx = P.Index.ivfpq_index_from_arrays(32, 9, 16, 4, *arrays)
    assert (idx.n, idx.d, idx.n_lists, idx.pq_dim, idx.pq_bits) == (777, 32, 9, 16, 4)
    out = idx.ivfpq_index_export()
    for a, b in zip(arrays, out):
        np.testing.assert_array_equal(np.asarray(a).reshape(b.shape), b)
    # device image: every list padded to 64 vectors, all arrays 256-byte aligned
    sizes = np.diff(arrays[2])
    padded = ((sizes + 63) // 64 * 64).sum()
    assert idx.ivfpq_device_bytes() >= padded * 8 + 777 * 8 + 9 * 32 * 4 + 16 * 16 * 2 * 4
    assert idx.ivfpq_device_bytes() % 256 == 0
    assert idx.ivfpq_search_workspace_bytes(100, 3, 10, 0) > 0
    idx.ivfpq_free()
    idx.ivfpq_free()   # idempotent


@pytest.mark.parametrize("kw,needle", [
    (dict(d=30, pq_dim=16), "multiple of pq_dim"),
    (dict(pq_bits=3), "pq_bits"),
    (dict(pq_bits=9), "pq_bits"),
    (dict(pq_bits=5), "multiple of 4"),
    (dict(d=6, pq_dim=6, pq_bits=4), "multiple of 4"),
    (dict(n_lists=0), "bad shape"),
])
def test_shape_validation(P, kw, needle):
    args = dict(d=32, n_lists=4, pq_dim=16, pq_bits=8)
    args.update(kw)
    d, L, s, p = args["d"], args["n_lists"], args["pq_dim"], args["pq_bits"]
    cent = np.zeros((max(L, 1), d), np.float32)
    cb = np.zeros((s, 1 << p, max(d // s, 1)), np.float32)
    with pytest.raises((P.IvfpqError, AssertionError)) as e:
        import ctypes
        h = ctypes.c_void_p()
        st = P.lib().ivfpq_index_from_arrays(0, d, L, s, p, cent.ctypes.data, cb.ctypes.data,
                                             np.zeros(max(L, 0) + 1, np.int64).ctypes.data, None, None, ctypes.byref(h))
        assert st == P.EINVAL
        raise P.IvfpqError(st, P.lib().ivfpq_last_error().decode())
    assert needle in str(e.value)


def test_bad_list_offsets_rejected(P):
    cent, cb, offs, codes, ids = si.random_index_arrays(50, 8, 3, 4, 8, salt=2)
    bad = offs.copy()
    bad[1], bad[2] = bad[2], bad[1] - 1 if bad[1] > 0 else 0
    bad[1] = offs[3] + 5
    with pytest.raises(P.IvfpqError):
        P.Index.ivfpq_index_from_arrays(8, 3, 4, 8, cent, cb, bad, codes, ids)
    bad = offs.copy()
    bad[-1] += 1
    with pytest.raises(P.IvfpqError):
        P.Index.ivfpq_index_from_arrays(8, 3, 4, 8, cent, cb, bad, codes, ids)


def test_fp8_encoding_setter_validates(P):
    idx = P.Index.ivfpq_index_from_arrays(32, 9, 16, 4, *si.random_index_arrays(100, 32, 9, 16, 4, salt=2))
    idx.ivfpq_set_fp8_encoding(P.LUT_FP8_E5M3, -96, P.ROUND_TRUNCATE, True)
    idx.ivfpq_set_fp8_encoding(P.LUT_FP8_E4M4, 110)
    idx.ivfpq_set_e4m4_bias(-100)
    for bad, needle in (((P.LUT_FP32, 15, 0, 0), "8-bit"), ((P.LUT_FP8_E5M3, -97, 0, 0), "outside"),
                        ((P.LUT_FP8_E4M4, 111, 0, 0), "outside"), ((P.LUT_FP8_E4M4, 7, 2, 0), "rounding"),
                        ((P.LUT_FP8_E5M3, 15, 0, 2), "per_table")):
        with pytest.raises(P.IvfpqError) as e:
            idx.ivfpq_set_fp8_encoding(*bad)
        assert e.value.status == P.EINVAL and needle in str(e.value)


def test_tuning_setter_validates(P):
    idx = P.Index.ivfpq_index_from_arrays(32, 9, 16, 4, *si.random_index_arrays(100, 32, 9, 16, 4, salt=2))
    for knob, good in ((P.TUNE_SCAN_THREADS, (0, 64, 1024)), (P.TUNE_ORDER_BLOCK, (0, 1, 64)), (P.TUNE_SCAN_SHARE, (0, 1, 2)),
                       (P.TUNE_EARLY_EXIT, (-1, 0, 1)), (P.TUNE_LDS_PAD, (0, 16, 65536))):
        for v in good:
            idx.ivfpq_set_tuning(knob, v)
        idx.ivfpq_set_tuning(knob, 0)
    for knob, bad in ((P.TUNE_SCAN_THREADS, 100), (P.TUNE_ORDER_BLOCK, -1), (P.TUNE_SCAN_SHARE, 3), (P.TUNE_EARLY_EXIT, 2),
                      (P.TUNE_LDS_PAD, 8), (P.TUNE_LDS_PAD, 1 << 20), (99, 0)):
        with pytest.raises(P.IvfpqError) as e:
            idx.ivfpq_set_tuning(knob, bad)
        assert e.value.status == P.EINVAL


def test_library_reads_no_environment_variable():
    # tuning is per index (ivfpq_set_tuning): no hidden process-global state
    for name in ("ivfpq_device.hip", "ivfpq_build.hip", "ivfpq_host.cpp", "ivfpq_rank.hpp", "ivfpq_internal.hpp"):
        text = open(os.path.join(ROOT, "paper_2301_06672_amd", "csrc", name)).read()
        assert "getenv" not in text, name


def test_static_scratch_search_refuses_what_does_not_fit(P):
    # one query on one cluster of 9 million vectors needs 2 x 9e6 x 8 bytes of scratch: more than the fixed
    # array.  The refusal comes before anything touches a device, so it is checked here without a GPU.
    n, d, s, p = 9_000_000, 4, 4, 8
    cent = np.zeros((1, d), np.float32)
    cb = np.zeros((s, 1 << p, 1), np.float32)
    offs = np.array([0, n], np.int64)
    idx = P.Index.ivfpq_index_from_arrays(d, 1, s, p, cent, cb, offs, np.zeros((n, 4), np.uint8), np.arange(n, dtype=np.int64))
    import ctypes
    dummy = ctypes.c_void_p(256)
    st = P.lib().ivfpq_search_static(idx._h, dummy, 1, 1, 10, P.LUT_FP8_E5M3, dummy, dummy, None)
    assert st == P.ENOSPACE
    msg = P.lib().ivfpq_last_error().decode()
    assert "static" in msg and str(P.STATIC_SCRATCH_BYTES) in msg
    # what fits is refused only for the missing device image
    small = P.Index.ivfpq_index_from_arrays(8, 3, 4, 8, *si.random_index_arrays(100, 8, 3, 4, 8, salt=3))
    assert P.lib().ivfpq_search_static(small._h, dummy, 1, 1, 1, 0, dummy, dummy, None) == P.ESTATE
    header = open(os.path.join(ROOT, "include", "ivfpq.h")).read()
    assert "((size_t)64 << 20)" in header and P.STATIC_SCRATCH_BYTES == 64 << 20


def test_device_builder_plan_is_checked_on_the_host(P):
    # the launch geometry and workspace layout of ivfpq_build_device are validated before the first launch;
    # the size query runs the same check, so it can be exercised without a GPU
    L = P.lib()
    need = L.ivfpq_build_device_workspace_bytes(100_000_000, 128, 50_000, 32, 8, 0, 0)      # the 10^8-vector workload
    n_ct = 256 * 50_000
    floor = n_ct * 128 * 4 + 100_000_000 * (4 + 4 + 4 + 32) + 262_144 * 128 * 4      # training rows, labels, order, tmp, codes, residuals
    assert floor < need < floor + (4 << 30)
    assert need % 256 == 0
    assert L.ivfpq_build_device_workspace_bytes(100_000_000, 128, 50_000, 64, 4, 0, 0) > 0
    # a shape whose row gather would need more workgroups than a grid dimension holds is refused, not truncated
    assert L.ivfpq_build_device_workspace_bytes(2_000_000_000, 4096, 1_000_000, 1024, 8, 0, 0) == 0
    assert b"workgroups" in L.ivfpq_last_error()


def test_stream_read_validates_before_launching(P):
    L = P.lib()
    for args in ((None, 64, 16, 4), (16, 64, None, 4), (16, 64, 32, 0), (16, 64, 32, 1 << 20), (8, 64, 32, 4), (16, 60, 32, 4)):
        assert L.ivfpq_stream_read(args[0], args[1], args[2], args[3], None) == P.EINVAL


def test_search_without_device_image_is_a_state_error(P):
    arrays = si.random_index_arrays(100, 8, 3, 4, 8, salt=3)
    idx = P.Index.ivfpq_index_from_arrays(8, 3, 4, 8, *arrays)
    import ctypes
    dummy = ctypes.c_void_p(256)
    st = P.lib().ivfpq_search(idx._h, dummy, 1, 1, 1, 0, dummy, dummy, dummy, 1 << 20, None)
    assert st == P.ESTATE
    assert b"ivfpq_upload" in P.lib().ivfpq_last_error()


def test_host_builder_structure_and_recall(P):
    w = si.WORKLOADS["tiny"]
    data = si.dataset(w)
    idx = P.Index.ivfpq_build_host(data, w.n_lists, w.pq_dim, w.pq_bits, w.kmeans_iters, seed=7)
    cent, cb, offs, codes, ids = idx.ivfpq_index_export()
    assert offs[0] == 0 and offs[-1] == w.n and np.all(np.diff(offs) >= 0)
    np.testing.assert_array_equal(np.sort(ids), np.arange(w.n))
    # membership is the nearest centroid (checked with the oracle's float64 assignment; a handful of
    # near-ties may differ because the builder ranks in fp32)
    labels, _ = oracle.assign(data, cent)
    lab_lib = np.empty(w.n, np.int64)
    lab_lib[ids] = np.repeat(np.arange(w.n_lists), np.diff(offs))
    assert (labels == lab_lib).mean() > 0.999
    for l in range(w.n_lists):
        assert np.all(np.diff(ids[offs[l]:offs[l + 1]]) > 0)
    # the index it builds is as good as the oracle's builder, judged by recall through the oracle's search
    oidx = oracle.make_index(w.d, w.n_lists, w.pq_dim, w.pq_bits, cent, cb, offs, codes, ids)
    q = si.queries(w, 300)
    gt, _ = oracle.exact_knn(data, q, w.k)
    recs = [oracle.recall(oracle.search(oidx, q, w.n_probes, w.k)[0], gt)]
    for seed in (8, 9):       # k-means starts differ: average the builder over a few seeds
        a = P.Index.ivfpq_build_host(data, w.n_lists, w.pq_dim, w.pq_bits, w.kmeans_iters, seed=seed).ivfpq_index_export()
        recs.append(oracle.recall(oracle.search(oracle.make_index(w.d, w.n_lists, w.pq_dim, w.pq_bits, *a),
                                                q, w.n_probes, w.k)[0], gt))
    from util_parity import oracle_tiny_index
    _, _, ref = oracle_tiny_index()
    rec_ref = oracle.recall(oracle.search(ref, q, w.n_probes, w.k)[0], gt)
    assert abs(np.mean(recs) - rec_ref) < 0.04 and min(recs) > 0.7
    # same seed, same index; another seed, another index
    again = P.Index.ivfpq_build_host(data, w.n_lists, w.pq_dim, w.pq_bits, w.kmeans_iters, seed=7).ivfpq_index_export()
    np.testing.assert_array_equal(again[0], cent)
    np.testing.assert_array_equal(again[3], codes)
    other = P.Index.ivfpq_build_host(data, w.n_lists, w.pq_dim, w.pq_bits, w.kmeans_iters, seed=8).ivfpq_index_export()
    assert not np.array_equal(other[0], cent)


@pytest.mark.parametrize("pq_bits", [5, 6, 7])
def test_host_builder_bit_packed_codes(P, pq_bits):
    # the host builder packs p-bit codes as one little-endian bit string: unpacked with the oracle's
    # reader, each code is the nearest codeword of its residual sub-vector
    w = si.WORKLOADS["tiny"].with_(n=1500)
    data = si.dataset(w)                        # d = 32
    idx = P.Index.ivfpq_build_host(data, 6, 32, pq_bits, 3, seed=2)
    cent, cb, offs, codes, ids = idx.ivfpq_index_export()
    assert codes.shape == (1500, 32 * pq_bits // 8) and cb.shape == (32, 1 << pq_bits, 1)
    labels = np.repeat(np.arange(6), np.diff(offs))
    res = data[ids] - cent[labels]
    sub = oracle.unpack_codes(codes, pq_bits)
    assert sub.max() < (1 << pq_bits)
    rows = np.random.default_rng(1).choice(1500, 60, replace=False)
    agree = 0
    for r in rows:
        for j in range(32):
            dist = (cb[j, :, 0].astype(np.float64) - res[r, j]) ** 2
            agree += int(sub[r, j] == dist.argmin())
    assert agree >= 0.99 * 60 * 32


def test_host_builder_4bit_codes_pack_low_nibble_first(P):
    w = si.WORKLOADS["tiny"].with_(n=2000)
    data = si.dataset(w)
    idx = P.Index.ivfpq_build_host(data, 8, 16, 4, 5, seed=1)
    cent, cb, offs, codes, ids = idx.ivfpq_index_export()
    assert codes.shape == (2000, 8) and cb.shape == (16, 16, 2)
    labels = np.repeat(np.arange(8), np.diff(offs))
    res = data[ids] - cent[labels]
    sub = oracle.unpack_codes(codes, 4)
    rows = np.random.default_rng(0).choice(2000, 100, replace=False)
    agree = 0
    for r in rows:
        for j in range(16):
            dist = ((cb[j].astype(np.float64) - res[r, 2 * j:2 * j + 2]) ** 2).sum(1)
            agree += int(sub[r, j] == dist.argmin())
    assert agree >= 0.99 * 1600
