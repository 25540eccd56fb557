"""GPU parity: the HIP library against the CPU oracle, element by element, on the same seeded
inputs, through the C ABI (ctypes binding).  Every test here needs an MI355X.

Bars (stated here, used below):
  * table entries for half and e5m3: the stored bytes are identical to the oracle's;
    the fp32 table too (same fp32 operation order on both sides);
  * accumulated distances R: within 1e-5 relative (fp32 adds of <= 64 non-negative terms in the
    same order; the tolerance leaves room for a different summation order);
  * top-k ids: equal except inside ties within that tolerance; padding identical;
  * probe lists: same clusters rank by rank, swaps only between clusters whose float64
    distances agree to 1e-5 relative.
"""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from util_parity import (RTOL, assert_probes_match, assert_topk_matches, oracle_tiny_index, random_pair,
                         to_library)

pytestmark = pytest.mark.gpu

DTYPES = [oracle.LUT_FP32, oracle.LUT_FP16, oracle.LUT_E5M3]


@pytest.fixture(scope="module")
def P():
    import paper_2301_06672_amd as pkg
    pkg.lib()
    assert torch.cuda.is_available()
    return pkg


@pytest.fixture(scope="module")
def tiny(P):
    w, data, oidx = oracle_tiny_index()
    return w, data, oidx, to_library(P, oidx)


def _step(msg):
    print(f"[parity] {msg}", flush=True)


# ---------------------------------------------------------------- table entries (search steps 2-3)

@pytest.mark.parametrize("dtype", DTYPES)
def test_lut_bytes_identical_tiny(P, tiny, dtype):
    w, data, oidx, gidx = tiny
    q = si.queries(w, 16)
    for qi in range(0, 16, 3):
        for l in (0, 7, 63):
            _step(f"dump_lut dtype={dtype} q={qi} list={l}")
            got = gidx.ivfpq_dump_lut(q[qi], l, dtype).cpu().numpy()
            want, _ = oracle.lut_store(oracle.lut_f32(oidx, q[qi], l), dtype)
            np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("d,pq_dim,pq_bits", [(32, 32, 8), (32, 16, 8), (32, 8, 8), (48, 16, 8), (24, 8, 4),
                                              (128, 64, 8), (96, 48, 8), (128, 64, 4), (128, 32, 8),
                                              (64, 32, 5), (96, 16, 6), (128, 64, 6), (64, 32, 7), (128, 64, 7)])
def test_lut_bytes_identical_shapes_and_ranges(P, d, pq_dim, pq_bits):
    # sub-vector lengths 1, 2, 4 (templated) and 3 (generic); value scales that reach below the
    # smallest e5m3 value, into the half subnormals, and above the largest half / e5m3 value
    for scale in (1e-3, 1.0, 300.0):
        oidx, gidx = random_pair(P, 300, d, 3, pq_dim, pq_bits, salt=100 + d + pq_dim, scale=scale)
        q = (scale * np.random.default_rng(d).standard_normal(d)).astype(np.float32)
        for dtype in DTYPES:
            _step(f"dump_lut d={d} s={pq_dim} p={pq_bits} scale={scale} dtype={dtype}")
            got = gidx.ivfpq_dump_lut(q, 1, dtype).cpu().numpy()
            F = oracle.lut_f32(oidx, q, 1)
            want, _ = oracle.lut_store(F, dtype)
            np.testing.assert_array_equal(got, want)
        if scale == 300.0:
            assert F.max() > 122880.0      # the saturating end was exercised
        if scale == 1e-3:
            assert F.min() < 2.0 ** -15     # and the flooring end


@pytest.mark.parametrize("bias", [-2, 1, 7, 14])
def test_e4m4_lut_bytes_and_search(P, tiny, bias):
    # the 4+4 split with a caller-chosen exponent bias: table bytes identical, search results as the oracle's
    w, data, oidx, gidx = tiny
    gidx.ivfpq_set_e4m4_bias(bias)
    q = si.queries(w, 40)
    for l in (3, 40):
        _step(f"e4m4 bias={bias} dump_lut list={l}")
        got = gidx.ivfpq_dump_lut(q[2], l, P.LUT_FP8_E4M4).cpu().numpy()
        want, _ = oracle.lut_store(oracle.lut_f32(oidx, q[2], l), oracle.LUT_E4M4, e4m4_bias=bias)
        np.testing.assert_array_equal(got, want)
    ids_g, d_g = gidx.ivfpq_search(q, w.n_probes, w.k, P.LUT_FP8_E4M4)
    probes, _ = gidx.ivfpq_select_probes(q, w.n_probes)
    ids_o, d_o = oracle.search(oidx, q, w.n_probes, w.k, oracle.LUT_E4M4, probes=probes.cpu().numpy().view(np.uint32),
                               e4m4_bias=bias)
    assert_topk_matches(ids_g.cpu().numpy(), d_g.cpu().numpy(), ids_o, d_o, context=f"e4m4 bias={bias}")
    gidx.ivfpq_set_e4m4_bias(7)


def test_e4m4_other_shapes(P):
    for d, pq_dim, pq_bits in ((128, 64, 4), (128, 32, 8), (24, 8, 4)):
        oidx, gidx = random_pair(P, 2000, d, 5, pq_dim, pq_bits, salt=900 + d + pq_bits)
        gidx.ivfpq_set_e4m4_bias(5)
        q = np.random.default_rng(900).standard_normal((20, d)).astype(np.float32)
        _step(f"e4m4 d={d} s={pq_dim} p={pq_bits}")
        ids_g, d_g = gidx.ivfpq_search(q, 3, 20, P.LUT_FP8_E4M4)
        probes, _ = gidx.ivfpq_select_probes(q, 3)
        ids_o, d_o = oracle.search(oidx, q, 3, 20, oracle.LUT_E4M4, probes=probes.cpu().numpy().view(np.uint32), e4m4_bias=5)
        assert_topk_matches(ids_g.cpu().numpy(), d_g.cpu().numpy(), ids_o, d_o, context=f"e4m4 d={d} p={pq_bits}")


FP8 = {oracle.LUT_E5M3: "e5m3", oracle.LUT_E4M4: "e4m4"}


def _reset_fp8(P, gidx):
    gidx.ivfpq_set_fp8_encoding(P.LUT_FP8_E5M3, 15)
    gidx.ivfpq_set_fp8_encoding(P.LUT_FP8_E4M4, 7)


@pytest.mark.parametrize("dtype", list(FP8))
@pytest.mark.parametrize("bias,trunc,per_table", [(15, True, False), (22, False, False), (3, True, False),
                                                  (0, False, True), (0, True, True)])
def test_fp8_encoding_options_lut_bytes_and_search(P, tiny, dtype, bias, trunc, per_table):
    # general exponent bias, truncating encode and per-table bias of both 8-bit formats: the table
    # bytes are identical to the oracle's and the search returns what the oracle returns
    w, data, oidx, gidx = tiny
    gidx.ivfpq_set_fp8_encoding(dtype, bias, P.ROUND_TRUNCATE if trunc else P.ROUND_NEAREST, per_table)
    try:
        q = si.queries(w, 40)
        kw = dict(truncate=trunc, bias=bias, per_table=per_table)
        for qi, l in ((2, 3), (5, 40), (11, 63)):
            _step(f"{FP8[dtype]} {kw} dump_lut q={qi} list={l}")
            got = gidx.ivfpq_dump_lut(q[qi], l, dtype).cpu().numpy()
            want, _ = oracle.lut_store(oracle.lut_f32(oidx, q[qi], l), dtype, **kw)
            np.testing.assert_array_equal(got, want)
        _step(f"{FP8[dtype]} {kw} search")
        ids_g, d_g = gidx.ivfpq_search(q, w.n_probes, w.k, dtype)
        probes, _ = gidx.ivfpq_select_probes(q, w.n_probes)
        ids_o, d_o = oracle.search(oidx, q, w.n_probes, w.k, dtype, probes=probes.cpu().numpy().view(np.uint32), **kw)
        assert_topk_matches(ids_g.cpu().numpy(), d_g.cpu().numpy(), ids_o, d_o, context=f"{FP8[dtype]} {kw}")
    finally:
        _reset_fp8(P, gidx)


@pytest.mark.parametrize("d,pq_dim,pq_bits", [(32, 32, 8), (48, 16, 8), (24, 8, 4), (128, 64, 4), (96, 48, 8)])
def test_per_table_bias_shapes_and_ranges(P, d, pq_dim, pq_bits):
    # every table-building code path (sub-vector lengths 1, 2, 3, 4; 4- and 8-bit codes) at value scales
    # from far below to far above the fixed formats' ranges; with a per-table bias the bytes follow the scale
    ref = {}
    for scale in (2.0 ** -30, 1.0, 2.0 ** 20):
        oidx = oracle.make_index(d, 3, pq_dim, pq_bits, *si.random_index_arrays(300, d, 3, pq_dim, pq_bits, salt=100 + d + pq_dim))
        s = np.float32(scale)
        oidx_s = oracle.make_index(d, 3, pq_dim, pq_bits, oidx.centroids * s, oidx.codebooks * s, oidx.list_offsets,
                                   oidx.codes, oidx.ids)
        gidx = to_library(P, oidx_s)
        q = (np.random.default_rng(d).standard_normal(d)).astype(np.float32) * s
        F = oracle.lut_f32(oidx_s, q, 1)
        for dtype in FP8:
            for trunc in (False, True):
                gidx.ivfpq_set_fp8_encoding(dtype, 0, int(trunc), True)
                _step(f"per-table d={d} s={pq_dim} p={pq_bits} scale={scale} {FP8[dtype]} trunc={trunc}")
                got = gidx.ivfpq_dump_lut(q, 1, dtype).cpu().numpy()
                want, _ = oracle.lut_store(F, dtype, truncate=trunc, per_table=True)
                np.testing.assert_array_equal(got, want)
                key = (dtype, trunc)
                if key in ref:
                    np.testing.assert_array_equal(got, ref[key])     # scale invariance, on the GPU side too
                ref[key] = got
                R_g = gidx.ivfpq_scan_list(q, 1, dtype, int(oidx.list_offsets[2] - oidx.list_offsets[1])).cpu().numpy()
                _, dec = oracle.lut_store(F, dtype, truncate=trunc, per_table=True)
                R_o, _ = oracle.scan_list(oidx_s, dec, 1)
                np.testing.assert_allclose(R_g, R_o, rtol=RTOL, atol=0)


# ---------------------------------------------------------------- Eq. (1) over one cluster (step 4)

@pytest.mark.parametrize("dtype", DTYPES)
def test_scan_list_R_tiny(P, tiny, dtype):
    w, data, oidx, gidx = tiny
    q = si.queries(w, 4)
    sizes = np.diff(oidx.list_offsets)
    for l in (int(np.argmax(sizes)), int(np.argmin(sizes)), 5):
        _step(f"scan_list dtype={dtype} list={l} len={sizes[l]}")
        _, dec = oracle.lut_store(oracle.lut_f32(oidx, q[1], l), dtype)
        want, _ = oracle.scan_list(oidx, dec, l)
        got = gidx.ivfpq_scan_list(q[1], l, dtype, int(sizes[l])).cpu().numpy()
        np.testing.assert_allclose(got, want, rtol=RTOL, atol=0)


@pytest.mark.parametrize("d,pq_dim,pq_bits", [(128, 64, 8), (96, 48, 8), (128, 64, 4), (128, 32, 8), (32, 16, 8),
                                              (24, 24, 8), (24, 8, 4), (160, 80, 8),
                                              (64, 32, 5), (96, 16, 6), (128, 64, 6), (64, 32, 7), (128, 64, 7), (256, 128, 5)])
def test_scan_list_R_code_widths(P, d, pq_dim, pq_bits):
    # 64/48/32/16-byte codes (16-byte chunk kernels) and 24/4/80-byte codes (generic 4-byte path);
    # bit-packed 5/6/7-bit codes whose fields straddle words (20/12/28/56/80 bytes on the 4-byte path,
    # 48 bytes of 6-bit codes on the 16-byte path);
    # list lengths that span several 64-vector groups with a ragged tail
    oidx, gidx = random_pair(P, 1500, d, 4, pq_dim, pq_bits, salt=200 + d + pq_bits)
    q = np.random.default_rng(pq_dim).standard_normal(d).astype(np.float32)
    sizes = np.diff(oidx.list_offsets)
    for dtype in DTYPES:
        for l in range(4):
            _step(f"scan_list d={d} s={pq_dim} p={pq_bits} dtype={dtype} list={l} len={sizes[l]}")
            _, dec = oracle.lut_store(oracle.lut_f32(oidx, q, l), dtype)
            want, _ = oracle.scan_list(oidx, dec, l)
            got = gidx.ivfpq_scan_list(q, l, dtype, int(sizes[l])).cpu().numpy()
            np.testing.assert_allclose(got, want, rtol=RTOL, atol=0)


# ---------------------------------------------------------------- probe selection (step 1)

@pytest.mark.parametrize("n_probes", [1, 8, 64])
def test_select_probes_tiny(P, tiny, n_probes):
    w, data, oidx, gidx = tiny
    q = si.queries(w, 300)
    _step(f"select_probes P={n_probes}")
    probes, pd = gidx.ivfpq_select_probes(q, n_probes)
    probes = probes.cpu().numpy().view(np.uint32)
    assert_probes_match(probes, oidx.centroids, q, n_probes)
    want, want_d = oracle.select_probes(oidx, q, n_probes)
    np.testing.assert_allclose(pd.cpu().numpy(), want_d, rtol=RTOL)
    assert (probes == want).mean() > 0.999


def test_select_probes_many_lists_and_exact_ties(P):
    # 3000 clusters (does not fit one pass of anything), 96 dims, duplicated centroids -> exact ties
    arrays = list(si.random_index_arrays(64, 96, 3000, 48, 8, salt=300))
    arrays[0][100:110] = arrays[0][50]          # ten copies of centroid 50
    oidx = oracle.make_index(96, 3000, 48, 8, *arrays)
    gidx = to_library(P, oidx)
    rng = np.random.default_rng(300)
    q = rng.standard_normal((40, 96)).astype(np.float32)
    q[:5] = arrays[0][50] + 0.01 * rng.standard_normal((5, 96)).astype(np.float32)
    for n_probes in (5, 200, 1000):
        _step(f"select_probes L=3000 P={n_probes}")
        probes, _ = gidx.ivfpq_select_probes(q, n_probes)
        probes = probes.cpu().numpy().view(np.uint32)
        assert_probes_match(probes, oidx.centroids, q, n_probes)
    # the tie group must come out in ascending cluster index
    probes, _ = gidx.ivfpq_select_probes(q[:5], 11)
    for row in probes.cpu().numpy().view(np.uint32):
        np.testing.assert_array_equal(row, [50] + list(range(100, 110)))


def test_select_probes_6000_lists_ties_and_outliers(P):
    # 6000 clusters: the bound of the n_probes-th ranking value comes from a sample of the row that grows
    # with n_probes.  Duplicated centroids far apart in the row give exact ties; a query far from
    # everything and one on a centroid are included.
    arrays = list(si.random_index_arrays(7000, 64, 6000, 32, 8, salt=310))
    arrays[0][5000:5006] = arrays[0][40]        # copies of a sampled centroid among the unsampled ones
    arrays[0][3000] = arrays[0][2999]
    oidx = oracle.make_index(64, 6000, 32, 8, *arrays)
    gidx = to_library(P, oidx)
    rng = np.random.default_rng(310)
    q = rng.standard_normal((70, 64)).astype(np.float32)
    q[:4] = arrays[0][40] + 0.01 * rng.standard_normal((4, 64)).astype(np.float32)
    q[4] = arrays[0][5500]
    q[5] = 50.0
    for n_probes in (1, 7, 64, 300, 1000):
        _step(f"select_probes L=6000 P={n_probes}")
        probes, pd = gidx.ivfpq_select_probes(q, n_probes)
        probes = probes.cpu().numpy().view(np.uint32)
        assert_probes_match(probes, oidx.centroids, q, n_probes)
        want, want_d = oracle.select_probes(oidx, q, n_probes)
        np.testing.assert_allclose(pd.cpu().numpy(), want_d, rtol=RTOL)
    probes, _ = gidx.ivfpq_select_probes(q[:4], 7)
    for row in probes.cpu().numpy().view(np.uint32):
        np.testing.assert_array_equal(row, [40] + list(range(5000, 5006)))
    for dtype in (oracle.LUT_FP32, oracle.LUT_E5M3):
        ids_g, d_g, ids_o, d_o = _search_both(gidx, oidx, q, 64, 20, dtype)
        assert_topk_matches(ids_g, d_g, ids_o, d_o, context=f"6000 lists dtype={dtype}")


def test_select_probes_strip_minima_large_batch(P):
    # enough queries x clusters that the ranking GEMM runs its 128 x 128 tiles and hands the selection
    # the minima of 64-cluster strips; n_probes on both sides of the rule that decides whether they are used
    arrays = list(si.random_index_arrays(7000, 32, 6000, 16, 8, salt=320))
    arrays[0][5990:5996] = arrays[0][17]        # exact ties across strips, one in the ragged last strip
    oidx = oracle.make_index(32, 6000, 16, 8, *arrays)
    gidx = to_library(P, oidx)
    rng = np.random.default_rng(320)
    q = rng.standard_normal((3000, 32)).astype(np.float32)
    q[:6] = arrays[0][17] + 0.01 * rng.standard_normal((6, 32)).astype(np.float32)
    for n_probes in (1, 7, 47, 48, 200):
        _step(f"select_probes strips L=6000 nq=3000 P={n_probes}")
        probes, pd = gidx.ivfpq_select_probes(q, n_probes)
        probes = probes.cpu().numpy().view(np.uint32)
        want, want_d = oracle.select_probes(oidx, q, n_probes)
        np.testing.assert_allclose(pd.cpu().numpy(), want_d, rtol=RTOL)
        assert (probes == want).mean() > 0.999
        assert all(len(set(r)) == n_probes for r in probes[:200])
    probes, _ = gidx.ivfpq_select_probes(q, 7)
    for row in probes.cpu().numpy().view(np.uint32)[:6]:
        np.testing.assert_array_equal(row, [17] + list(range(5990, 5996)))


def test_select_probes_bf16_tiles_with_padded_dimension(P):
    # d = 24 is not a multiple of the 16-component slices of the bf16 kernel: the split pads with zeros
    arrays = list(si.random_index_arrays(7000, 24, 6000, 12, 8, salt=340))
    oidx = oracle.make_index(24, 6000, 12, 8, *arrays)
    gidx = to_library(P, oidx)
    q = np.random.default_rng(340).standard_normal((3000, 24)).astype(np.float32)
    for n_probes in (5, 33):
        _step(f"select_probes d=24 L=6000 nq=3000 P={n_probes}")
        probes, pd = gidx.ivfpq_select_probes(q, n_probes)
        want, want_d = oracle.select_probes(oidx, q, n_probes)
        np.testing.assert_allclose(pd.cpu().numpy(), want_d, rtol=RTOL)
        assert (probes.cpu().numpy().view(np.uint32) == want).mean() > 0.999


@pytest.mark.parametrize("nq", [40, 3000])
def test_non_finite_queries_stay_in_range(P, nq):
    # NaN, infinite and huge queries: the call returns, every index it returns is valid, and the finite
    # queries of the same batch get their exact answer (40 queries: fp32 tiles and all ranking keys;
    # 3000: bf16 tiles and strip summaries)
    arrays = list(si.random_index_arrays(7000, 32, 6000, 16, 8, salt=350))
    oidx = oracle.make_index(32, 6000, 16, 8, *arrays)
    gidx = to_library(P, oidx)
    q = np.random.default_rng(350).standard_normal((nq, 32)).astype(np.float32)
    bad = [1, 7, 20, 33]
    q[1, 3] = np.nan
    q[7, :] = np.inf
    q[20, 0] = -np.inf
    q[33, :] = 3.0e38
    good = np.setdiff1d(np.arange(nq), bad)
    _step(f"non-finite queries nq={nq}: probes")
    probes, _ = gidx.ivfpq_select_probes(q, 12)
    probes = probes.cpu().numpy().view(np.uint32)
    assert probes.max() < 6000
    want, _ = oracle.select_probes(oidx, q[good], 12)
    assert (probes[good] == want).mean() > 0.999
    _step(f"non-finite queries nq={nq}: search")
    ids, dist = gidx.ivfpq_search(q, 12, 10, P.LUT_FP8_E5M3)
    ids = ids.cpu().numpy()
    assert ids.min() >= -1 and ids.max() < 7000
    ids_o, d_o = oracle.search(oidx, q[good], 12, 10, oracle.LUT_E5M3, probes=probes[good])
    assert_topk_matches(ids[good], dist.cpu().numpy()[good], ids_o, d_o, context="finite queries beside non-finite ones")


def test_select_probes_plateau_of_equal_centroids(P):
    # 40,000 clusters, all but three with the same centroid: every strip minimum equals the bound, more
    # strips qualify than the list holds, the whole row overflows the candidate buffer and the kernel
    # ends in its exact whole-row selection; ties come out by ascending cluster index
    arrays = list(si.random_index_arrays(41000, 8, 40000, 4, 8, salt=330))
    arrays[0][:] = arrays[0][0]
    arrays[0][[12345, 777, 39999]] += np.float32(0.25)
    oidx = oracle.make_index(8, 40000, 4, 8, *arrays)
    gidx = to_library(P, oidx)
    q = np.tile(arrays[0][12345], (3, 1)).astype(np.float32)
    q[1] = arrays[0][0]
    for n_probes in (1, 10, 300):
        _step(f"select_probes plateau P={n_probes}")
        probes, pd = gidx.ivfpq_select_probes(q, n_probes)
        probes = probes.cpu().numpy().view(np.uint32)
        want, want_d = oracle.select_probes(oidx, q, n_probes)
        np.testing.assert_array_equal(probes, want)
        np.testing.assert_allclose(pd.cpu().numpy(), want_d, rtol=RTOL)


# ---------------------------------------------------------------- whole search (steps 1-5)

def _search_both(gidx, oidx, q, n_probes, k, dtype):
    """GPU search; the oracle is run on the GPU's probe lists so that a near-tie in step 1 does not
    turn into a different (and equally valid) candidate set downstream."""
    ids_g, d_g = gidx.ivfpq_search(q, n_probes, k, dtype)
    probes, _ = gidx.ivfpq_select_probes(q, n_probes)
    probes = probes.cpu().numpy().view(np.uint32)
    ids_o, d_o = oracle.search(oidx, q, n_probes, k, dtype, probes=probes)
    return ids_g.cpu().numpy(), d_g.cpu().numpy(), ids_o, d_o


@pytest.mark.parametrize("dtype", DTYPES)
def test_search_tiny_config(P, tiny, dtype):
    w, data, oidx, gidx = tiny
    q = si.queries(w)                            # all 1,000 queries of the configuration
    _step(f"search tiny dtype={dtype}")
    ids_g, d_g, ids_o, d_o = _search_both(gidx, oidx, q, w.n_probes, w.k, dtype)
    swapped = assert_topk_matches(ids_g, d_g, ids_o, d_o, context=f"tiny dtype={dtype}")
    assert swapped <= 0.01 * ids_o.size
    # and against the oracle's own probe selection: same answer for (nearly) every query
    ids_oo, _ = oracle.search(oidx, q, w.n_probes, w.k, dtype)
    assert (ids_oo == ids_g).all(axis=1).mean() > 0.99
    gt, _ = oracle.exact_knn(data, q[:200], w.k)
    assert abs(oracle.recall(ids_g[:200], gt) - oracle.recall(ids_oo[:200], gt)) < 1e-3


@pytest.mark.parametrize("n_probes,k", [(1, 1), (3, 100), (64, 10), (8, 1024)])
def test_search_tiny_probe_and_k_range(P, tiny, n_probes, k):
    w, data, oidx, gidx = tiny
    q = si.queries(w, 64)
    for dtype in (oracle.LUT_FP32, oracle.LUT_E5M3):
        _step(f"search tiny P={n_probes} k={k} dtype={dtype}")
        ids_g, d_g, ids_o, d_o = _search_both(gidx, oidx, q, n_probes, k, dtype)
        assert_topk_matches(ids_g, d_g, ids_o, d_o, context=f"P={n_probes} k={k} dtype={dtype}")


@pytest.mark.parametrize("d,pq_dim,pq_bits", [(128, 64, 8), (96, 48, 8), (128, 64, 4), (128, 32, 8), (24, 8, 4),
                                              (64, 32, 5), (128, 64, 6), (32, 16, 6), (128, 64, 7)])
def test_search_random_index_ragged_and_empty_lists(P, d, pq_dim, pq_bits):
    oidx, gidx = random_pair(P, 5000, d, 37, pq_dim, pq_bits, salt=400 + d + pq_bits, empty_lists=(0, 5, 36))
    q = np.random.default_rng(400).standard_normal((50, d)).astype(np.float32)
    for dtype in DTYPES:
        for n_probes, k in ((4, 10), (37, 100)):
            _step(f"search random d={d} s={pq_dim} p={pq_bits} dtype={dtype} P={n_probes} k={k}")
            ids_g, d_g, ids_o, d_o = _search_both(gidx, oidx, q, n_probes, k, dtype)
            assert_topk_matches(ids_g, d_g, ids_o, d_o, context=f"d={d} p={pq_bits} dtype={dtype}")


def test_search_fewer_candidates_than_k_pads(P):
    oidx, gidx = random_pair(P, 70, 32, 9, 16, 8, salt=500, empty_lists=(1, 2))
    q = np.random.default_rng(500).standard_normal((8, 32)).astype(np.float32)
    probes = np.tile(np.array([[1, 2, 3]], dtype=np.uint32), (8, 1))      # two empty clusters and a small one
    ids_g, d_g = gidx.ivfpq_search_with_probes(q, probes, 50, oracle.LUT_FP16)
    ids_o, d_o = oracle.search(oidx, q, 3, 50, oracle.LUT_FP16, probes=probes)
    assert_topk_matches(ids_g.cpu().numpy(), d_g.cpu().numpy(), ids_o, d_o, context="padding")
    assert (ids_o == -1).any()
    probes = np.tile(np.array([[1, 2]], dtype=np.uint32), (8, 1))         # nothing to scan at all
    ids_g, d_g = gidx.ivfpq_search_with_probes(q, probes, 5, oracle.LUT_FP32)
    assert (ids_g.cpu().numpy() == -1).all() and np.isinf(d_g.cpu().numpy()).all()


def test_search_massive_ties_order_by_id(P):
    # 6000 identical codes in one cluster: every R is equal, the answer is the k smallest ids
    # (more ties than the selection's LDS record capacity -> the 64-bit tie-key path)
    cent, cb, offs, codes, ids = si.random_index_arrays(6400, 32, 2, 16, 8, salt=600)
    codes[:] = codes[0]
    oidx = oracle.make_index(32, 2, 16, 8, cent, cb, offs, codes, ids)
    gidx = to_library(P, oidx)
    q = np.random.default_rng(600).standard_normal((3, 32)).astype(np.float32)
    for k in (1, 10, 1000):
        for n_probes in (1, 2):
            _step(f"massive ties k={k} P={n_probes}")
            ids_g, d_g, ids_o, d_o = _search_both(gidx, oidx, q, n_probes, k, oracle.LUT_E5M3)
            np.testing.assert_array_equal(ids_g, ids_o)
            np.testing.assert_array_equal(d_g, d_o)


def test_search_small_nearest_cluster_admits_everything(P):
    # the nearest probe holds fewer than k vectors, so its R values give no bound: every vector of
    # the large second cluster survives the filter (each wave appends several staged batches)
    n, d = 3300, 32
    cent, cb, _, codes, ids = si.random_index_arrays(n, d, 3, 16, 8, salt=800)
    offs = np.array([0, 40, 3240, 3300], dtype=np.int64)
    oidx = oracle.make_index(d, 3, 16, 8, cent, cb, offs, codes, ids)
    gidx = to_library(P, oidx)
    q = np.random.default_rng(800).standard_normal((6, d)).astype(np.float32)
    for probes_row, k in (([0, 1], 100), ([0, 1, 2], 1000), ([2, 1], 64), ([1, 0], 10)):
        probes = np.tile(np.array([probes_row], dtype=np.uint32), (6, 1))
        for dtype in (oracle.LUT_FP32, oracle.LUT_E5M3):
            _step(f"small nearest cluster probes={probes_row} k={k} dtype={dtype}")
            ids_g, d_g = gidx.ivfpq_search_with_probes(q, probes, k, dtype)
            ids_o, d_o = oracle.search(oidx, q, len(probes_row), k, dtype, probes=probes)
            assert_topk_matches(ids_g.cpu().numpy(), d_g.cpu().numpy(), ids_o, d_o, context=f"probes={probes_row} k={k}")


def test_search_cluster_listed_twice_is_scanned_twice(P, tiny):
    w, data, oidx, gidx = tiny
    q = si.queries(w, 10)
    probes = np.tile(np.array([[4, 4, 9]], dtype=np.uint32), (10, 1))
    ids_g, d_g = gidx.ivfpq_search_with_probes(q, probes, 20, oracle.LUT_FP32)
    ids_o, d_o = oracle.search(oidx, q, 3, 20, oracle.LUT_FP32, probes=probes)
    assert_topk_matches(ids_g.cpu().numpy(), d_g.cpu().numpy(), ids_o, d_o, context="dup cluster")


def test_empty_inputs(P, tiny):
    w, data, oidx, gidx = tiny
    ids, d = gidx.ivfpq_search(np.zeros((0, w.d), np.float32), 4, 10, oracle.LUT_E5M3)
    assert ids.shape == (0, 10) and d.shape == (0, 10)
    # an index with no vectors at all
    cent, cb, offs, codes, ids0 = si.random_index_arrays(0, 32, 4, 16, 8, salt=700)
    oidx0 = oracle.make_index(32, 4, 16, 8, cent, cb, offs, codes, ids0)
    g0 = to_library(P, oidx0)
    q = np.ones((3, 32), np.float32)
    ids, d = g0.ivfpq_search(q, 2, 5, oracle.LUT_FP32)
    assert (ids.cpu().numpy() == -1).all() and np.isinf(d.cpu().numpy()).all()


def test_error_paths(P, tiny):
    w, data, oidx, gidx = tiny
    q = torch.from_numpy(si.queries(w, 4)).cuda()
    with pytest.raises(P.IvfpqError) as e:
        gidx.ivfpq_search(q, 0, 10, 0)
    assert e.value.status == P.EINVAL
    with pytest.raises(P.IvfpqError) as e:
        gidx.ivfpq_search(q, w.n_lists + 1, 10, 0)
    assert e.value.status == P.EINVAL
    with pytest.raises(P.IvfpqError) as e:
        gidx.ivfpq_search(q, 4, P.MAX_K + 1, 0)
    assert e.value.status == P.EINVAL
    with pytest.raises(P.IvfpqError) as e:
        gidx.ivfpq_search(q, 4, 10, 7)
    assert e.value.status == P.EINVAL
    with pytest.raises(P.IvfpqError) as e:
        gidx.ivfpq_set_e4m4_bias(500)
    assert e.value.status == P.EINVAL
    for bad in ((P.LUT_FP16, 15, 0, 0), (P.LUT_FP8_E5M3, -97, 0, 0), (P.LUT_FP8_E5M3, 111, 0, 0),
                (P.LUT_FP8_E4M4, 7, 2, 0), (P.LUT_FP8_E4M4, 7, 0, 3)):
        with pytest.raises(P.IvfpqError) as e:
            gidx.ivfpq_set_fp8_encoding(*bad)
        assert e.value.status == P.EINVAL
    # a workspace that is too small is refused before anything is launched
    import ctypes
    ids = torch.empty((4, 10), dtype=torch.int64, device="cuda")
    d = torch.empty((4, 10), dtype=torch.float32, device="cuda")
    ws = torch.empty(256, dtype=torch.uint8, device="cuda")
    st = P.lib().ivfpq_search(gidx._h, ctypes.c_void_p(q.data_ptr()), 4, 4, 10, 0, ctypes.c_void_p(ids.data_ptr()),
                              ctypes.c_void_p(d.data_ptr()), ctypes.c_void_p(ws.data_ptr()), 256, None)
    assert st == P.ENOSPACE
    # no device image yet
    fresh = P.Index.ivfpq_index_from_arrays(oidx.d, oidx.n_lists, oidx.pq_dim, oidx.pq_bits, oidx.centroids,
                                            oidx.codebooks, oidx.list_offsets, oidx.codes, oidx.ids)
    with pytest.raises(P.IvfpqError) as e:
        fresh.ivfpq_search(q, 4, 10, 0)
    assert e.value.status == P.ESTATE


def test_stage_timing_reports(P, tiny):
    w, data, oidx, gidx = tiny
    q = torch.from_numpy(si.queries(w, 256)).cuda()
    gidx.ivfpq_set_stage_timing(True)
    gidx.ivfpq_search(q, 8, 10, oracle.LUT_E5M3)
    torch.cuda.synchronize()
    ms = gidx.ivfpq_stage_times_ms()
    gidx.ivfpq_set_stage_timing(False)
    assert ms["total"] > 0 and ms["scan"] > 0
    assert ms["probe_select"] + ms["scan"] + ms["topk"] <= ms["total"] * 1.05 + 0.05
    # single launches inside the stages
    assert 0 < ms["rank_gemm"] <= ms["probe_select"] * 1.05 + 0.05
    assert ms["scan_nearest_kernel"] > 0 and ms["scan_filtered_kernel"] > 0
    assert ms["scan_nearest_kernel"] + ms["scan_filtered_kernel"] <= ms["scan"] * 1.05 + 0.05


def test_library_builder_index_searches_like_oracle_builder(P, tiny):
    # the two builders run different k-means code: compare them by recall only
    w, data, oidx, _ = tiny
    g = P.Index.ivfpq_build_host(data, w.n_lists, w.pq_dim, w.pq_bits, w.kmeans_iters, seed=3).ivfpq_upload()
    q = si.queries(w, 300)
    gt, _ = oracle.exact_knn(data, q, w.k)
    ids_lib, _ = g.ivfpq_search(q, w.n_probes, w.k, oracle.LUT_FP32)
    ids_orc, _ = oracle.search(oidx, q, w.n_probes, w.k, oracle.LUT_FP32)
    assert abs(oracle.recall(ids_lib.cpu().numpy(), gt) - oracle.recall(ids_orc, gt)) < 0.06


# ---------------------------------------------------------------- re-ranking with the stored vectors

def test_refine_matches_oracle(P, tiny):
    w, data, oidx, gidx = tiny
    q = si.queries(w, 200)
    x = torch.from_numpy(data).cuda()
    _step("refine: search k'=40, refine to 10")
    cand, _ = gidx.ivfpq_search(q, w.n_probes, 40, P.LUT_FP8_E5M3)
    ids_g, d_g = P.ivfpq_refine(x, q, cand, 10)
    ids_o, d_o = oracle.refine(data, q, cand.cpu().numpy(), 10)
    assert_topk_matches(ids_g.cpu().numpy(), d_g.cpu().numpy(), ids_o, d_o.astype(np.float32), context="refine")
    gt, _ = oracle.exact_knn(data, q, 10)
    ids10, _ = gidx.ivfpq_search(q, w.n_probes, 10, P.LUT_FP8_E5M3)
    r0, r1 = oracle.recall(ids10.cpu().numpy(), gt), oracle.recall(ids_g.cpu().numpy(), gt)
    _step(f"refine: recall@10 {r0:.3f} -> {r1:.3f}")
    assert r1 > r0 + 0.03


@pytest.mark.parametrize("n_cand,k", [(1, 1), (7, 10), (64, 64), (1000, 100), (1024, 1024)])
def test_refine_edge_cases(P, n_cand, k):
    rng = np.random.default_rng(n_cand)
    n, d, nq = 3000, 24, 33
    data = rng.integers(-3, 4, size=(n, d)).astype(np.float32)      # integer grid: many exactly equal distances
    q = rng.integers(-3, 4, size=(nq, d)).astype(np.float32)
    cand = rng.integers(0, n, size=(nq, n_cand)).astype(np.int64)   # with duplicates
    cand[rng.random(cand.shape) < 0.2] = -1                          # padding entries anywhere
    if n_cand > 3:
        cand[5, :] = -1                                              # a query with no candidate at all
        cand[6, 3] = n + 5                                           # an id beyond the data: skipped
    _step(f"refine edge n_cand={n_cand} k={k}")
    ids_g, d_g = P.ivfpq_refine(torch.from_numpy(data).cuda(), q, torch.from_numpy(cand).cuda(), k)
    cand_o = np.where(cand >= n, -1, cand)
    ids_o, d_o = oracle.refine(data, q, cand_o, k)
    # integer-valued data: fp32 distances are exact, so the result is identical, ties by id included
    np.testing.assert_array_equal(ids_g.cpu().numpy(), ids_o)
    np.testing.assert_array_equal(d_g.cpu().numpy().astype(np.float64), d_o)


def test_refine_rejects_bad_arguments(P):
    x = torch.zeros((10, 8), device="cuda")
    q = torch.zeros((2, 8), device="cuda")
    for n_cand, k in ((P.MAX_K + 1, 5), (4, 0), (4, P.MAX_K + 1)):
        with pytest.raises(P.IvfpqError) as e:
            P.ivfpq_refine(x, q, torch.zeros((2, n_cand), dtype=torch.int64, device="cuda"), k)
        assert e.value.status == P.EINVAL


# ---------------------------------------------------------------- the streaming-read measurement kernel

@pytest.mark.parametrize("n_words,n_wg", [(4, 1), (4 * 1000, 3), (4 * 300001, 64)])
def test_stream_read_folds_every_word_once(P, n_words, n_wg):
    rng = np.random.default_rng(n_words)
    words = rng.integers(0, 2**32, size=n_words, dtype=np.uint64).astype(np.uint32)
    _step(f"stream read {n_words} words, {n_wg} workgroups")
    out = P.ivfpq_stream_read(torch.from_numpy(words.view(np.int32)).cuda(), n_wg).cpu().numpy().view(np.uint32)
    # 16-byte word i belongs to workgroup (i // 256) % n_wg
    w16 = np.bitwise_xor.reduce(words.reshape(-1, 4), axis=1)
    owner = (np.arange(w16.size) // 256) % n_wg
    want = np.zeros(n_wg, dtype=np.uint32)
    np.bitwise_xor.at(want, owner, w16)
    np.testing.assert_array_equal(out, want)


# ---------------------------------------------------------------- several pairs of one cluster per workgroup

@pytest.mark.parametrize("d,pq_dim,pq_bits,n_lists,n_probes,k", [
    (32, 16, 8, 7, 5, 10),        # m = 2, few clusters: most neighbouring pairs share theirs (runs of 4, 3, 2 and 1)
    (64, 16, 8, 33, 8, 100),      # m = 4
    (48, 48, 8, 200, 40, 10),     # m = 1, three 16-byte chunks, many seams between clusters
    (128, 64, 8, 3, 3, 1000),     # four chunks; two pairs per query: odd and even runs
    (128, 32, 8, 20, 12, 100),    # two chunks, m = 4: the shape of the 10^8-vector workload with 8-bit codes
    (128, 64, 4, 20, 12, 100),    # 4-bit codes, two chunks, m = 2: the shape of the 10^8-vector workload with 4-bit codes
    (32, 32, 4, 7, 5, 10),        # 4-bit codes, one chunk, m = 1
    (128, 32, 4, 33, 8, 1000),    # 4-bit codes, one chunk, m = 4
    (96, 96, 4, 50, 20, 10),      # 4-bit codes, three chunks
    (128, 128, 4, 9, 6, 100),     # 4-bit codes, four chunks
])
@pytest.mark.parametrize("dtype_name", ["e5m3", "e4m4", "fp16", "fp32"])
def test_search_group_of_pairs_per_workgroup(P, d, pq_dim, pq_bits, n_lists, n_probes, k, dtype_name):
    # the kernel that interleaves the tables of two or four queries of one cluster is forced on; results must be
    # those of the oracle, and identical to the one-pair kernel's (same arithmetic per query, same order)
    dtype = {"e5m3": oracle.LUT_E5M3, "e4m4": oracle.LUT_E4M4, "fp16": oracle.LUT_FP16, "fp32": oracle.LUT_FP32}[dtype_name]
    oidx, gidx = random_pair(P, 9000, d, n_lists, pq_dim, pq_bits, salt=900 + d, empty_lists=(1,) if n_lists > 3 else ())
    q = np.random.default_rng(900 + d).standard_normal((257, d)).astype(np.float32)
    gidx.ivfpq_set_tuning(P.TUNE_SCAN_SHARE, 1)
    assert gidx.ivfpq_scan_kernel_info(dtype).startswith("scan_kernel")
    ids_one, d_one = gidx.ivfpq_search(q, n_probes, k, dtype)
    for share in (2, 4):
        gidx.ivfpq_set_tuning(P.TUNE_SCAN_SHARE, share)
        info = gidx.ivfpq_scan_kernel_info(dtype)
        _step(f"{share} pairs per workgroup d={d} s={pq_dim} p={pq_bits} L={n_lists} P={n_probes} k={k} {dtype_name}: {info}")
        if not info.startswith("scan_group_kernel"):
            continue                      # tables of that many queries do not fit the LDS
        ids_g, d_g, ids_o, d_o = _search_both(gidx, oidx, q, n_probes, k, dtype)
        assert_topk_matches(ids_g, d_g, ids_o, d_o, context=f"{share} pairs per workgroup")
        np.testing.assert_array_equal(d_g, d_one.cpu().numpy())
        np.testing.assert_array_equal(ids_g, ids_one.cpu().numpy())
    gidx.ivfpq_set_tuning(P.TUNE_SCAN_SHARE, 0)


def test_group_kernel_survivor_overflow_and_small_batches(P):
    # a bound that admits everything (nearest cluster smaller than k) makes every vector of the big cluster a
    # survivor: groups with more survivors than a wave stages are appended directly; also 1, 2 and 3 queries
    # (slots that are not full) and a workspace limit that cuts the batch into tiles
    n, d = 21000, 64
    cent, cb, _, codes, ids = si.random_index_arrays(n, d, 3, 32, 8, salt=811)
    offs = np.array([0, 40, 20040, 21000], dtype=np.int64)
    oidx = oracle.make_index(d, 3, 32, 8, cent, cb, offs, codes, ids)
    gidx = to_library(P, oidx)
    rng = np.random.default_rng(811)
    for nq in (1, 2, 3, 9):
        q = (cent[0] + 0.01 * rng.standard_normal((nq, d))).astype(np.float32)       # nearest cluster: the 40-vector one
        for share in (2, 4):
            gidx.ivfpq_set_tuning(P.TUNE_SCAN_SHARE, share)
            for dtype in (oracle.LUT_E5M3, oracle.LUT_FP16):
                _step(f"overflow nq={nq} share={share} dtype={dtype}")
                ids_g, d_g, ids_o, d_o = _search_both(gidx, oidx, q, 3, 1000, dtype)
                assert_topk_matches(ids_g, d_g, ids_o, d_o, context="group kernel, every vector survives")
    gidx.ivfpq_set_tuning(P.TUNE_SCAN_SHARE, 0)


@pytest.mark.parametrize("d,pq_dim,pq_bits,dtype", [
    (128, 64, 8, oracle.LUT_E5M3), (128, 64, 8, oracle.LUT_FP32),     # four 16-byte chunks
    (96, 48, 8, oracle.LUT_FP16),                                     # three
    (64, 64, 4, oracle.LUT_E5M3),                                     # 4-bit codes: 32 sub-spaces per chunk
    (64, 32, 6, oracle.LUT_E4M4),                                     # 6-bit codes in 4-byte chunks
    (128, 64, 6, oracle.LUT_E5M3),                                    # 6-bit codes, 48 bytes: 16-byte chunks
    (40, 40, 8, oracle.LUT_E5M3),                                     # 40-byte codes: 4-byte chunks
])
def test_early_exit_changes_nothing(P, d, pq_dim, pq_bits, dtype):
    # a group whose partial sums are all over the bound stops early: the survivors, hence the results, are the same
    oidx, gidx = random_pair(P, 12000, d, 9, pq_dim, pq_bits, salt=950 + d + pq_bits)
    q = np.random.default_rng(950 + d).standard_normal((130, d)).astype(np.float32)
    out = {}
    for mode in ("0", "1"):
        gidx.ivfpq_set_tuning(P.TUNE_EARLY_EXIT, 1 if mode == "1" else -1)
        _step(f"early exit {mode}: d={d} s={pq_dim} p={pq_bits} dtype={dtype}")
        ids, dist = gidx.ivfpq_search(q, 6, 10, dtype)
        out[mode] = (ids.cpu().numpy(), dist.cpu().numpy())
    np.testing.assert_array_equal(out["0"][0], out["1"][0])
    np.testing.assert_array_equal(out["0"][1], out["1"][1])
    gidx.ivfpq_set_tuning(P.TUNE_EARLY_EXIT, 0)
    ids_g, d_g, ids_o, d_o = _search_both(gidx, oidx, q, 6, 10, dtype)
    assert_topk_matches(ids_g, d_g, ids_o, d_o, context="early exit")


def test_split_scan_when_every_group_stays_in_the_race(P):
    # 64 sub-spaces of 8-bit codes: the filtered scan builds half the table first.  Here the nearest cluster
    # holds fewer than k vectors, so the bound admits everything: every group of the big cluster needs the
    # second half, more groups per wave than the first pass can note (it then takes them all again)
    n, d = 21000, 128
    cent, cb, _, codes, ids = si.random_index_arrays(n, d, 3, 64, 8, salt=810)
    offs = np.array([0, 40, 20040, 21000], dtype=np.int64)
    oidx = oracle.make_index(d, 3, 64, 8, cent, cb, offs, codes, ids)
    gidx = to_library(P, oidx)
    q = np.random.default_rng(810).standard_normal((6, d)).astype(np.float32)
    # (share: the one-pair kernel, the library's choice, and the group kernel with two and four pairs per workgroup)
    for share in (1, 0, 2, 4):
        gidx.ivfpq_set_tuning(P.TUNE_SCAN_SHARE, share)
        for probes_row, k in (([0, 1], 100), ([0, 1, 2], 1000), ([2, 1], 10), ([1, 2, 0], 10)):
            probes = np.tile(np.array([probes_row], dtype=np.uint32), (6, 1))
            for dtype in (oracle.LUT_FP32, oracle.LUT_E5M3):
                _step(f"split scan, everything in the race: share={share} probes={probes_row} k={k} dtype={dtype}: "
                      f"{gidx.ivfpq_scan_kernel_info(dtype)}")
                ids_g, d_g = gidx.ivfpq_search_with_probes(q, probes, k, dtype)
                ids_o, d_o = oracle.search(oidx, q, len(probes_row), k, dtype, probes=probes)
                assert_topk_matches(ids_g.cpu().numpy(), d_g.cpu().numpy(), ids_o, d_o, context=f"share={share} probes={probes_row} k={k}")
    gidx.ivfpq_set_tuning(P.TUNE_SCAN_SHARE, 0)


def test_search_nearest_cluster_smaller_than_k(P):
    # the cluster nearest to these queries holds 5 vectors, fewer than k: the search takes its bound from the
    # next probe that holds at least k (and scans that one unfiltered); the answer is the oracle's all the same
    n, d = 6000, 32
    cent, cb, _, codes, ids = si.random_index_arrays(n, d, 5, 16, 8, salt=820)
    offs = np.array([0, 5, 8, 3000, 3000, 6000], dtype=np.int64)          # 5, 3, 2992, 0 and 3000 vectors
    oidx = oracle.make_index(d, 5, 16, 8, cent, cb, offs, codes, ids)
    gidx = to_library(P, oidx)
    rng = np.random.default_rng(820)
    q = (cent[0] + 0.05 * rng.standard_normal((40, d))).astype(np.float32)
    q[20:] = (cent[1] + 0.05 * rng.standard_normal((20, d))).astype(np.float32)
    for n_probes, k in ((5, 10), (2, 10), (3, 4), (5, 1000), (1, 10)):
        for dtype in (oracle.LUT_FP32, oracle.LUT_E5M3):
            _step(f"nearest cluster smaller than k: P={n_probes} k={k} dtype={dtype}")
            ids_g, d_g, ids_o, d_o = _search_both(gidx, oidx, q, n_probes, k, dtype)
            assert_topk_matches(ids_g, d_g, ids_o, d_o, context=f"tiny nearest cluster P={n_probes} k={k}")


# ---------------------------------------------------------------- the search inside a HIP graph

def test_search_replays_correctly_from_a_hip_graph(P, tiny):
    # a serving loop may capture the search call once and replay it: the call only enqueues kernels
    # (no allocation, no synchronisation, no memset), so every replay must give the eager result
    w, data, oidx, gidx = tiny
    qs = si.queries(w, 192)
    q = torch.from_numpy(qs[:64]).cuda()
    out = (torch.empty((64, w.k), dtype=torch.int64, device="cuda"), torch.empty((64, w.k), dtype=torch.float32, device="cuda"))
    for dtype in (P.LUT_FP8_E5M3, P.LUT_FP32):
        _step(f"graph capture lut={dtype}")
        q.copy_(torch.from_numpy(qs[:64]))
        gidx.ivfpq_search(q, w.n_probes, w.k, dtype, out=out)          # eager: workspace and kernel attributes in place
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            gidx.ivfpq_search(q, w.n_probes, w.k, dtype, out=out)
        for rep in range(4):
            q.copy_(torch.from_numpy(qs[64 * (rep % 3):64 * (rep % 3) + 64]))      # new queries in the captured buffer
            want_i, want_d = gidx.ivfpq_search(q.clone(), w.n_probes, w.k, dtype)  # eager work between the replays
            torch.cuda.synchronize()
            out[0].fill_(-7)
            out[1].fill_(-1.0)
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(out[0], want_i) and torch.equal(out[1], want_d), f"replay {rep}"
        del g


def test_workspace_limit_changes_tiling_not_results(P, tiny):
    w, data, oidx, gidx = tiny
    q = torch.from_numpy(si.queries(w, 300)).cuda()
    big = gidx.ivfpq_search_workspace_bytes(300, w.n_probes, w.k, P.LUT_FP8_E5M3)
    want = gidx.ivfpq_search(q, w.n_probes, w.k, P.LUT_FP8_E5M3)
    torch.cuda.synchronize()
    try:
        gidx.ivfpq_set_workspace_limit(1 << 20)             # a few queries per tile
        small = gidx.ivfpq_search_workspace_bytes(300, w.n_probes, w.k, P.LUT_FP8_E5M3)
        assert small < big
        _step(f"workspace limit 1 MiB: {small} bytes instead of {big}")
        got = gidx.ivfpq_search(q, w.n_probes, w.k, P.LUT_FP8_E5M3)
        torch.cuda.synchronize()
        assert torch.equal(got[0], want[0]) and torch.equal(got[1], want[1])
        with pytest.raises(P.IvfpqError):
            gidx.ivfpq_set_workspace_limit(1000)
    finally:
        gidx.ivfpq_set_workspace_limit(32 << 30)


# ---------------------------------------------------------------- seeded random configurations

def test_search_seeded_random_configurations(P):
    # thirty configurations drawn from a seeded generator: code widths 4-8 bits, sub-vector lengths 1-6,
    # few or many clusters (some empty), any table dtype and encoding option, k and n_probes up to the
    # limits that the configuration allows
    rng = np.random.default_rng(20230106)
    for case in range(30):
        bits = int(rng.integers(4, 9))
        unit = {4: 8, 5: 32, 6: 16, 7: 32, 8: 4}[bits]             # sub-spaces per 32-bit boundary
        pq_dim = unit * int(rng.integers(1, 5 if unit < 32 else 3))
        m = int(rng.choice([1, 2, 3, 4, 6]))
        d = pq_dim * m
        n_lists = int(rng.choice([1, 2, 7, 33, 200, 1500]))
        n = int(rng.integers(max(n_lists, 50), 6000))
        empty = tuple(int(v) for v in rng.choice(n_lists, size=min(3, n_lists - 1), replace=False)) if n_lists > 3 else ()
        n_probes = int(rng.integers(1, min(n_lists, 40) + 1))
        k = int(rng.choice([1, 5, 10, 100, 1000]))
        dtype = int(rng.integers(0, 4))
        trunc, per_table = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
        scale = float(rng.choice([1e-3, 1.0, 30.0]))
        oidx, gidx = random_pair(P, n, d, n_lists, pq_dim, bits, salt=7000 + case, scale=scale, empty_lists=empty)
        q = (scale * rng.standard_normal((17, d))).astype(np.float32)
        kw = {}
        if dtype in FP8:
            bias = 15 if dtype == oracle.LUT_E5M3 else 7
            gidx.ivfpq_set_fp8_encoding(dtype, bias, int(trunc), per_table)
            kw = dict(truncate=trunc, bias=bias, per_table=per_table)
        _step(f"random case {case}: n={n} d={d} lists={n_lists} s={pq_dim} p={bits} P={n_probes} k={k} dtype={dtype} {kw}")
        ids_g, d_g = gidx.ivfpq_search(q, n_probes, k, dtype)
        probes, _ = gidx.ivfpq_select_probes(q, n_probes)
        probes = probes.cpu().numpy().view(np.uint32)
        assert_probes_match(probes, oidx.centroids, q, n_probes)
        ids_o, d_o = oracle.search(oidx, q, n_probes, k, dtype, probes=probes, **kw)
        assert_topk_matches(ids_g.cpu().numpy(), d_g.cpu().numpy(), ids_o, d_o, context=f"random case {case}")
        gidx.ivfpq_free()


def test_search_index_without_vectors(P):
    # every cluster empty: nothing faults, every result slot is padding
    d, n_lists, pq_dim = 32, 12, 16
    rng = np.random.default_rng(77)
    cent = rng.standard_normal((n_lists, d)).astype(np.float32)
    cb = rng.standard_normal((pq_dim, 256, 2)).astype(np.float32)
    gidx = P.Index.ivfpq_index_from_arrays(d, n_lists, pq_dim, 8, cent, cb, np.zeros(n_lists + 1, np.int64),
                                           np.zeros((0, pq_dim), np.uint8), np.zeros(0, np.int64)).ivfpq_upload()
    q = rng.standard_normal((9, d)).astype(np.float32)
    for n_probes in (1, 5, 12):
        _step(f"empty index P={n_probes}")
        ids, dist = gidx.ivfpq_search(q, n_probes, 7, P.LUT_FP8_E5M3)
        assert (ids.cpu().numpy() == -1).all() and np.isinf(dist.cpu().numpy()).all()
    probes, _ = gidx.ivfpq_select_probes(q, 12)
    assert_probes_match(probes.cpu().numpy().view(np.uint32), cent, q, 12)
