"""Pins for the oracle's IVFPQ build and search (Sec. I-B, I-C).  CPU only.

The oracle is checked against things other than itself:
  * exact k-NN against float64 numpy on a few hundred points;
  * k-means: nearest-centre assignment against brute-force numpy, the
    monotone objective of Lloyd's iteration, recovery of well-separated blobs,
    zero objective when every point is a centre;
  * probe selection against numpy's stable argsort of float64 distances;
  * Eq. (1) with the fp32 table: for a codebook with zero distortion
    (x = centroid + concatenated codebook entries) R equals |q - x|^2 -- the
    statement that closes search step 4 -- and the whole search with every
    cluster probed equals exact k-NN;
  * one cluster at the origin reduces IVFPQ to plain PQ asymmetric distance,
    typed out in float64 numpy;
  * top-k against numpy lexsort on the same R; padding when candidates < k;
  * 4-bit code packing round trip and a search on it;
  * recall behaviour on the tiny workload (sanity band, not a pin).
"""
import numpy as np
import pytest

import oracle
import synth_inputs as si


def _rng(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------ exact k-NN

def test_exact_knn_matches_numpy_float64():
    rng = _rng(10)
    data = rng.standard_normal((500, 12)).astype(np.float32)
    q = rng.standard_normal((20, 12)).astype(np.float32)
    ids, d2 = oracle.exact_knn(data, q, 7)
    full = ((q[:, None, :].astype(np.float64) - data[None, :, :].astype(np.float64)) ** 2).sum(-1)
    want = np.argsort(full, axis=1, kind="stable")[:, :7]
    np.testing.assert_array_equal(ids, want)
    np.testing.assert_allclose(d2, np.take_along_axis(full, want, 1), rtol=1e-14)


def test_exact_knn_ties_go_to_lower_id_and_padding():
    data = np.array([[0, 0], [1, 0], [1, 0], [0, 1], [-1, 0]], dtype=np.float32)
    ids, d2 = oracle.exact_knn(data, np.zeros((1, 2), np.float32), 7)
    np.testing.assert_array_equal(ids[0], [0, 1, 2, 3, 4, -1, -1])
    assert np.isinf(d2[0, 5:]).all()


def test_recall_definition():
    found = np.array([[1, 2, 3], [4, 5, -1]])
    truth = np.array([[3, 2, 9], [7, 8, 4]])
    assert oracle.recall(found, truth) == pytest.approx(3 / 6)


# ------------------------------------------------------------------ k-means

def test_assign_is_brute_force_argmin():
    rng = _rng(11)
    x = rng.standard_normal((700, 5)).astype(np.float32)
    c = rng.standard_normal((33, 5)).astype(np.float32)
    c[7] = c[3]                                        # exact duplicate: the lower index must win
    labels, total = oracle.assign(x, c)
    full = ((x[:, None, :].astype(np.float64) - c[None].astype(np.float64)) ** 2).sum(-1)
    np.testing.assert_array_equal(labels, full.argmin(1))
    assert total == pytest.approx(full.min(1).sum(), rel=1e-12)
    assert not np.any(labels == 7)


def test_kmeans_objective_never_increases_and_blobs_are_found():
    rng = _rng(12)
    true = np.array([[0, 0], [10, 0], [0, 10], [10, 10]], dtype=np.float32)
    x = (true[rng.integers(0, 4, 2000)] + 0.3 * rng.standard_normal((2000, 2))).astype(np.float32)
    # one start row from each blob (rows nearest to each true centre)
    init = np.array([np.argmin(((x - t) ** 2).sum(1)) for t in true], dtype=np.int64)
    c, inertia = oracle.kmeans(x, 4, 8, init)
    assert np.all(np.diff(inertia) <= 1e-9 * inertia[0])
    for t in true:
        assert np.min(np.abs(c - t).max(1)) < 0.1
    # centre = mean of its members (float64 mean, cast to fp32), members fixed after convergence
    labels, _ = oracle.assign(x, c)
    for j in range(4):
        np.testing.assert_allclose(c[j], x[labels == j].astype(np.float64).mean(0), rtol=0, atol=1e-5)


def test_kmeans_every_point_a_centre_gives_zero_objective_and_empty_keeps_centre():
    rng = _rng(13)
    x = rng.standard_normal((16, 3)).astype(np.float32)
    c, inertia = oracle.kmeans(x, 16, 3, np.arange(16, dtype=np.int64))
    assert np.all(inertia == 0)
    np.testing.assert_array_equal(c, x)
    # duplicate start rows: the second copy never wins a tie, stays empty, keeps its centre
    init = np.array([0, 0, 5], dtype=np.int64)
    c2, _ = oracle.kmeans(x, 3, 4, init)
    np.testing.assert_array_equal(c2[1], x[0])


def test_kmeans_random_start_objective_monotone():
    w = si.WORKLOADS["tiny"].with_(n=3000)
    x = si.dataset(w)
    init = si.kmeans_init_rows(si.STREAM_COARSE_INIT, 0, len(x), 32)
    _, inertia = oracle.kmeans(x, 32, 10, init)
    assert np.all(np.diff(inertia) <= 1e-9 * inertia[0])
    assert inertia[-1] < 0.8 * inertia[0]


# ------------------------------------------------------------------ build

def _tiny_index(n=3000, n_lists=16, pq_dim=16, pq_bits=8, iters=6, salt=0):
    w = si.WORKLOADS["tiny"].with_(n=n, salt=salt)
    data = si.dataset(w)
    coarse_init = si.kmeans_init_rows(si.STREAM_COARSE_INIT, 0, n, n_lists, salt)
    pq_init = np.stack([si.kmeans_init_rows(si.STREAM_PQ_INIT, j, n, 1 << pq_bits, salt) for j in range(pq_dim)])
    idx = oracle.build_index(data, n_lists, pq_dim, pq_bits, iters, coarse_init, pq_init)
    return w, data, idx


def test_build_structure_and_codes_are_argmin():
    w, data, idx = _tiny_index()
    n = len(data)
    assert idx.list_offsets[0] == 0 and idx.list_offsets[-1] == n
    assert np.all(np.diff(idx.list_offsets) >= 0)
    np.testing.assert_array_equal(np.sort(idx.ids), np.arange(n))
    m = idx.m
    # membership = nearest centroid; ids ascending inside a list; code = nearest codebook entry of the residual
    full = ((data[:, None, :].astype(np.float64) - idx.centroids[None].astype(np.float64)) ** 2).sum(-1)
    nearest = full.argmin(1)
    for l in range(idx.n_lists):
        lo, hi = idx.list_offsets[l], idx.list_offsets[l + 1]
        members = idx.ids[lo:hi]
        assert np.all(np.diff(members) > 0)
        assert np.all(nearest[members] == l)
    rows = _rng(1).choice(n, 200, replace=False)
    pos = {int(v): i for i, v in enumerate(idx.ids)}
    for r in rows:
        res = data[r] - idx.centroids[nearest[r]]
        for j in range(idx.pq_dim):
            sub = res[j * m:(j + 1) * m].astype(np.float64)
            dist = ((idx.codebooks[j].astype(np.float64) - sub) ** 2).sum(1)
            assert idx.codes[pos[int(r)], j] == dist.argmin()


def test_pack_unpack_4bit_round_trip():
    rng = _rng(14)
    c = rng.integers(0, 16, size=(100, 8), dtype=np.uint8)
    p = oracle.pack_codes(c, 4)
    assert p.shape == (100, 4)
    assert p[3, 1] == (c[3, 2] | (c[3, 3] << 4))
    np.testing.assert_array_equal(oracle.unpack_codes(p, 4), c)


@pytest.mark.parametrize("pq_bits,pq_dim", [(4, 8), (5, 32), (6, 16), (7, 32), (8, 12)])
def test_pack_codes_is_one_little_endian_bit_string(pq_bits, pq_dim):
    # independent statement of the layout: the row's codes form the integer sum_j c_j << (j*p), stored
    # little-endian
    rng = _rng(140 + pq_bits)
    c = rng.integers(0, 1 << pq_bits, size=(50, pq_dim), dtype=np.uint8)
    packed = oracle.pack_codes(c, pq_bits)
    nbytes = pq_dim * pq_bits // 8
    assert packed.shape == (50, nbytes)
    for r in range(50):
        value = sum(int(c[r, j]) << (j * pq_bits) for j in range(pq_dim))
        assert bytes(packed[r]) == value.to_bytes(nbytes, "little")
    np.testing.assert_array_equal(oracle.unpack_codes(packed, pq_bits), c)


# ------------------------------------------------------------------ probes

def test_select_probes_is_stable_argsort_of_float64_distances():
    rng = _rng(15)
    cent = rng.standard_normal((40, 6)).astype(np.float32)
    cent[11] = cent[4]
    idx = oracle.make_index(6, 40, 3, 8, cent, np.zeros((3, 256, 2)), np.zeros(41), np.zeros((0, 3)), np.zeros(0))
    q = rng.standard_normal((25, 6)).astype(np.float32)
    probes, d2 = oracle.select_probes(idx, q, 9)
    full = ((q[:, None].astype(np.float64) - cent[None].astype(np.float64)) ** 2).sum(-1)
    want = np.argsort(full, axis=1, kind="stable")[:, :9]
    np.testing.assert_array_equal(probes, want)
    np.testing.assert_allclose(d2, np.take_along_axis(full, want, 1), rtol=1e-14)


# ------------------------------------------------------------------ LUT + Eq. (1)

def _zero_distortion_case(seed, n=400, d=24, n_lists=5, pq_dim=6, pq_bits=8):
    """An index whose coded vectors are reproduced exactly by centroid + codebook entries."""
    cent, cb, offs, codes, ids = si.random_index_arrays(n, d, n_lists, pq_dim, pq_bits, salt=seed)
    # keep every coordinate on a coarse binary grid so that x = c + cb and q - x are exact in fp32
    cent = np.round(cent * 8) / 8
    cb = np.round(cb * 16) / 16
    idx = oracle.make_index(d, n_lists, pq_dim, pq_bits, cent, cb, offs, codes, ids)
    sub = oracle.unpack_codes(codes, pq_bits)
    labels = np.repeat(np.arange(n_lists), np.diff(offs))
    recon = cent[labels].astype(np.float64)
    m = d // pq_dim
    for j in range(pq_dim):
        recon[:, j * m:(j + 1) * m] += cb[j][sub[:, j]]
    x = np.empty_like(recon)
    x[ids] = recon                                     # row `id` of the data set
    return idx, x.astype(np.float32), labels


@pytest.mark.parametrize("pq_bits,pq_dim", [(8, 6), (4, 12)])
def test_zero_distortion_R_is_squared_distance(pq_bits, pq_dim):
    idx, x, labels = _zero_distortion_case(20 + pq_bits, pq_dim=pq_dim, pq_bits=pq_bits)
    assert np.array_equal(x.astype(np.float64), x)      # exact by construction
    q = (np.round(_rng(21).standard_normal((6, idx.d)) * 4) / 4).astype(np.float32)
    for qi in range(len(q)):
        for l in range(idx.n_lists):
            F = oracle.lut_f32(idx, q[qi], l)
            assert np.all(F >= 0)
            _, dec = oracle.lut_store(F, oracle.LUT_FP32)
            R, R64 = oracle.scan_list(idx, dec, l)
            lo, hi = idx.list_offsets[l], idx.list_offsets[l + 1]
            true = ((q[qi].astype(np.float64) - x[idx.ids[lo:hi]].astype(np.float64)) ** 2).sum(1)
            np.testing.assert_allclose(R, true, rtol=idx.pq_dim * 2.0 ** -23, atol=0)
            np.testing.assert_allclose(R64, true, rtol=1e-6)


def test_zero_distortion_full_probe_equals_exact_knn():
    idx, x, _ = _zero_distortion_case(30, n=600, n_lists=7)
    q = (np.round(_rng(31).standard_normal((40, idx.d)) * 4) / 4 + 1 / 64).astype(np.float32)
    ids, dist = oracle.search(idx, q, idx.n_lists, 10, oracle.LUT_FP32)
    gt_ids, gt_d2 = oracle.exact_knn(x, q, 10)
    np.testing.assert_allclose(dist, gt_d2, rtol=1e-5)
    # ids equal wherever the true distances around the rank are separated
    for r in range(len(q)):
        sep = np.abs(np.diff(np.concatenate([gt_d2[r], [np.inf]]))) > 1e-4 * gt_d2[r]
        sep[1:] &= sep[:-1].copy()
        assert np.array_equal(ids[r][sep], gt_ids[r][sep])
    assert oracle.recall(ids, gt_ids) > 0.99


def test_single_cluster_at_origin_is_plain_pq_distance():
    rng = _rng(32)
    n, d, pq_dim = 300, 16, 4
    m = d // pq_dim
    cb = rng.standard_normal((pq_dim, 256, m)).astype(np.float32)
    codes = rng.integers(0, 256, size=(n, pq_dim), dtype=np.uint8)
    idx = oracle.make_index(d, 1, pq_dim, 8, np.zeros((1, d)), cb, [0, n], codes, np.arange(n))
    q = rng.standard_normal(d).astype(np.float32)
    F = oracle.lut_f32(idx, q, 0)
    # the table itself, entry by entry, in float64: |codebook entry - query sub-vector|^2
    want_F = ((cb.astype(np.float64) - q.reshape(pq_dim, 1, m).astype(np.float64)) ** 2).sum(-1)
    np.testing.assert_allclose(F, want_F, rtol=3e-7)
    R, _ = oracle.scan_list(idx, F, 0)
    want = np.zeros(n)
    for j in range(pq_dim):
        want += ((cb[j][codes[:, j]].astype(np.float64) - q[j * m:(j + 1) * m].astype(np.float64)) ** 2).sum(1)
    np.testing.assert_allclose(R, want, rtol=1e-6)


def test_lut_uses_residual_of_the_probed_cluster():
    # F for cluster l must equal F of the shifted query q - c_l against a zero centroid
    cent, cb, offs, codes, ids = si.random_index_arrays(50, 8, 3, 4, 8, salt=33)
    idx = oracle.make_index(8, 3, 4, 8, cent, cb, offs, codes, ids)
    zero = oracle.make_index(8, 1, 4, 8, np.zeros((1, 8)), cb, [0, 50], codes, ids)
    q = _rng(33).standard_normal(8).astype(np.float32)
    for l in range(3):
        np.testing.assert_array_equal(oracle.lut_f32(idx, q, l), oracle.lut_f32(zero, q - cent[l], 0))


# ------------------------------------------------------------------ top-k

def test_search_topk_is_lexsort_of_all_candidates():
    cent, cb, offs, codes, ids = si.random_index_arrays(900, 16, 12, 8, 8, salt=34, empty_lists=(2,))
    codes[100:140] = codes[100]                       # exact duplicates -> equal R, order by id
    idx = oracle.make_index(16, 12, 8, 8, cent, cb, offs, codes, ids)
    q = _rng(34).standard_normal((15, 16)).astype(np.float32)
    probes, _ = oracle.select_probes(idx, q, 5)
    for dtype in (oracle.LUT_FP32, oracle.LUT_FP16, oracle.LUT_E5M3):
        got_ids, got_d = oracle.search(idx, q, 5, 20, dtype)
        for r in range(len(q)):
            Rs, Is = [], []
            for l in probes[r]:
                _, dec = oracle.lut_store(oracle.lut_f32(idx, q[r], int(l)), dtype)
                R, _ = oracle.scan_list(idx, dec, int(l))
                Rs.append(R)
                Is.append(idx.ids[idx.list_offsets[l]:idx.list_offsets[l + 1]])
            R, I = np.concatenate(Rs), np.concatenate(Is)
            order = np.lexsort((I, R))[:20]
            np.testing.assert_array_equal(got_ids[r], I[order])
            np.testing.assert_array_equal(got_d[r], R[order])


def test_search_pads_when_fewer_than_k_candidates_and_given_probes_are_used():
    cent, cb, offs, codes, ids = si.random_index_arrays(60, 8, 6, 4, 8, salt=35, empty_lists=(0, 1))
    idx = oracle.make_index(8, 6, 4, 8, cent, cb, offs, codes, ids)
    q = _rng(35).standard_normal((3, 8)).astype(np.float32)
    probes = np.array([[0, 1], [0, 2], [3, 1]], dtype=np.uint32)
    got_ids, got_d = oracle.search(idx, q, 2, 40, oracle.LUT_FP32, probes=probes)
    np.testing.assert_array_equal(got_ids[0], -1)
    assert np.isinf(got_d[0]).all()
    n2 = int(offs[3] - offs[2])
    assert np.all(got_ids[1, :min(n2, 40)] >= 0) and np.all(got_ids[1, n2:] == -1)
    assert set(got_ids[1, :n2]) <= set(ids[offs[2]:offs[3]])


@pytest.mark.parametrize("pq_bits,pq_dim", [(4, 8), (5, 32), (6, 16), (7, 32)])
def test_bit_packed_search_matches_unpacked_8bit_search(pq_bits, pq_dim):
    # a p-bit index is the same thing as an 8-bit index whose codebook has 2^p used entries
    d = 2 * pq_dim
    cent, cb4, offs, codes4, ids = si.random_index_arrays(500, d, 4, pq_dim, pq_bits, salt=36)
    idx4 = oracle.make_index(d, 4, pq_dim, pq_bits, cent, cb4, offs, codes4, ids)
    cb8 = np.zeros((pq_dim, 256, 2), dtype=np.float32)
    cb8[:, :1 << pq_bits] = cb4
    idx8 = oracle.make_index(d, 4, pq_dim, 8, cent, cb8, offs, oracle.unpack_codes(codes4, pq_bits), ids)
    q = _rng(36).standard_normal((10, d)).astype(np.float32)
    for dtype in (oracle.LUT_FP32, oracle.LUT_E5M3):
        a = oracle.search(idx4, q, 3, 10, dtype)
        b = oracle.search(idx8, q, 3, 10, dtype)
        np.testing.assert_array_equal(a[0], b[0])
        np.testing.assert_array_equal(a[1], b[1])


# ------------------------------------------------------------------ recall sanity on the tiny workload

def test_tiny_workload_recall_band():
    w, data, idx = _tiny_index(n=10_000, n_lists=64, iters=10)
    q = si.queries(w, 200)
    gt, _ = oracle.exact_knn(data, q, 10)
    rec = {}
    for P in (1, 8, 64):
        ids, _ = oracle.search(idx, q, P, 10, oracle.LUT_FP32)
        rec[P] = oracle.recall(ids, gt)
    assert rec[1] < rec[8] <= rec[64] + 1e-9
    assert rec[8] > 0.5
    ids16, _ = oracle.search(idx, q, 8, 10, oracle.LUT_FP16)
    ids8, _, stats = oracle.search(idx, q, 8, 10, oracle.LUT_E5M3, return_stats=True)
    ids8t, _ = oracle.search(idx, q, 8, 10, oracle.LUT_E5M3, truncate=True)
    assert abs(oracle.recall(ids16, gt) - rec[8]) < 0.01
    assert abs(oracle.recall(ids8, gt) - rec[8]) < 0.03
    assert oracle.recall(ids8t, gt) <= oracle.recall(ids8, gt) + 0.02
    assert stats["saturated"] == 0


@pytest.mark.parametrize("dt", [oracle.LUT_E5M3, oracle.LUT_E4M4])
def test_per_table_bias_makes_search_invariant_to_power_of_two_scaling(dt):
    # every step of the path is exact under a power-of-two scale of the inputs; a per-table bias makes
    # the 8-bit table follow the scale, so ids are unchanged and R scales by the square
    import dataclasses
    w, data, idx = _tiny_index(n=4000, n_lists=16, iters=5)
    q = si.queries(w, 40)
    s = np.float32(2.0 ** -9)
    idx_s = dataclasses.replace(idx, centroids=idx.centroids * s, codebooks=idx.codebooks * s)
    for trunc in (False, True):
        ids_a, d_a = oracle.search(idx, q, 6, 10, dt, truncate=trunc, per_table=True)
        ids_b, d_b = oracle.search(idx_s, q * s, 6, 10, dt, truncate=trunc, per_table=True)
        np.testing.assert_array_equal(ids_a, ids_b)
        np.testing.assert_array_equal(d_a.astype(np.float64) * float(s) ** 2, d_b.astype(np.float64))
    # with the fixed bias the scaled tables fall under the smallest code and the results change
    _, _, st_a = oracle.search(idx, q, 6, 10, dt, return_stats=True)
    ids_c, _, st_c = oracle.search(idx_s, q * s, 6, 10, dt, return_stats=True)
    assert st_c["floored"] > st_a["floored"]
    _, _, st_p = oracle.search(idx_s, q * s, 6, 10, dt, per_table=True, return_stats=True)
    assert st_p["floored"] < st_c["floored"]


def test_refine_is_exact_knn_restricted_to_the_candidates():
    rng = _rng(31)
    data = rng.standard_normal((500, 12)).astype(np.float32)
    q = rng.standard_normal((9, 12)).astype(np.float32)
    # all rows as candidates (in scrambled order): the exact k nearest neighbours
    cand = np.stack([rng.permutation(500) for _ in range(9)])
    ids, d2 = oracle.refine(data, q, cand, 7)
    gt_i, gt_d = oracle.exact_knn(data, q, 7)
    np.testing.assert_array_equal(ids, gt_i)
    np.testing.assert_array_equal(d2, gt_d)
    # a subset with padding entries: numpy float64 on the listed rows only; short rows are padded
    cand = rng.integers(0, 500, size=(9, 20)).astype(np.int64)
    cand[:, 15:] = -1
    cand[3, 2:] = -1
    ids, d2 = oracle.refine(data, q, cand, 5)
    for r in range(9):
        rows = cand[r][cand[r] >= 0]
        dist = ((data[rows].astype(np.float64) - q[r].astype(np.float64)) ** 2).sum(1)
        order = np.lexsort((rows, dist))[:5]
        want_i = np.full(5, -1, dtype=np.int64); want_d = np.full(5, np.inf)
        want_i[:len(order)] = rows[order]; want_d[:len(order)] = dist[order]
        np.testing.assert_array_equal(ids[r], want_i)
        np.testing.assert_allclose(d2[r], want_d, rtol=1e-12)
    assert ids[3, 2] == -1 and np.isinf(d2[3, 2])


def test_refine_raises_recall_of_a_pq_search():
    w, data, idx = _tiny_index(n=10_000, n_lists=64, iters=10)
    q = si.queries(w, 100)
    gt, _ = oracle.exact_knn(data, q, 10)
    ids10, _ = oracle.search(idx, q, 8, 10, oracle.LUT_E5M3)
    ids40, _ = oracle.search(idx, q, 8, 40, oracle.LUT_E5M3)
    ref, d2 = oracle.refine(data, q, ids40, 10)
    assert oracle.recall(ref, gt) > oracle.recall(ids10, gt) + 0.05
    assert np.all(np.diff(d2, axis=1) >= 0)
    # refining the k results themselves only reorders them
    same, _ = oracle.refine(data, q, ids10, 10)
    np.testing.assert_array_equal(np.sort(same, axis=1), np.sort(ids10, axis=1))
