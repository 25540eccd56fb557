"""Helpers shared by the GPU parity tests: build matching oracle/library indexes from the same
arrays and compare results where more than one answer is correct (ties)."""
import numpy as np

import oracle
import synth_inputs as si

RTOL = 1e-5   # relative tolerance on accumulated distances (the bar for the fp32 table)


def oracle_tiny_index(n=10_000, n_lists=64, pq_dim=16, pq_bits=8, iters=10, salt=0, name="tiny"):
    w = si.WORKLOADS[name].with_(n=n, salt=salt, n_lists=n_lists, pq_dim=pq_dim, pq_bits=pq_bits)
    data = si.dataset(w)
    coarse_init = si.kmeans_init_rows(si.STREAM_COARSE_INIT, 0, n, n_lists, salt)
    pq_init = np.stack([si.kmeans_init_rows(si.STREAM_PQ_INIT, j, n, 1 << pq_bits, salt) for j in range(pq_dim)])
    idx = oracle.build_index(data, n_lists, pq_dim, pq_bits, iters, coarse_init, pq_init)
    return w, data, idx


def to_library(P, oidx):
    """The same logical arrays imported into the HIP library and uploaded."""
    return P.Index.ivfpq_index_from_arrays(oidx.d, oidx.n_lists, oidx.pq_dim, oidx.pq_bits, oidx.centroids,
                                           oidx.codebooks, oidx.list_offsets, oidx.codes, oidx.ids).ivfpq_upload()


def random_pair(P, n, d, n_lists, pq_dim, pq_bits, salt, **kw):
    arrays = si.random_index_arrays(n, d, n_lists, pq_dim, pq_bits, salt=salt, **kw)
    oidx = oracle.make_index(d, n_lists, pq_dim, pq_bits, *arrays)
    return oidx, to_library(P, oidx)


def assert_topk_matches(ids_g, d_g, ids_o, d_o, rtol=RTOL, context=""):
    """Distances must agree to rtol position by position; ids must agree wherever the oracle's
    distance at that rank is separated by more than the tolerance from its neighbours and from the
    k-th distance (inside such a band any order / any member of the tie is a correct answer)."""
    ids_g, d_g, ids_o, d_o = map(np.asarray, (ids_g, d_g, ids_o, d_o))
    assert ids_g.shape == ids_o.shape and d_g.shape == d_o.shape, context
    fin = np.isfinite(d_o)
    assert np.array_equal(np.isfinite(d_g), fin), f"{context}: padding differs"
    np.testing.assert_allclose(d_g[fin], d_o[fin], rtol=rtol, atol=0, err_msg=context)
    assert np.array_equal(ids_g[~fin], ids_o[~fin]), f"{context}: padded ids differ"
    bad = np.argwhere((ids_g != ids_o) & fin)
    for r, j in bad:
        row = d_o[r].astype(np.float64)
        tol = rtol * max(row[j], np.finfo(np.float32).tiny)
        neighbours = np.abs(row - row[j]) <= tol
        neighbours[j] = False
        last_finite = row[np.isfinite(row)][-1]
        assert neighbours.any() or abs(last_finite - row[j]) <= tol, (
            f"{context}: query {r} rank {j}: id {ids_g[r, j]} vs oracle {ids_o[r, j]} at distance {row[j]} "
            f"with no tie inside the tolerance")
        # whatever was returned instead must sit at the same distance
        assert abs(float(d_g[r, j]) - row[j]) <= tol
    return len(bad)


def assert_probes_match(probes_g, cent, queries, n_probes, rtol=RTOL):
    """GPU probe lists against float64 distances: same clusters in the same order, except that
    clusters whose distances lie within rtol of each other may swap (or swap in/out at the end)."""
    probes_g = np.asarray(probes_g).astype(np.int64)
    full = ((queries[:, None, :].astype(np.float64) - cent[None].astype(np.float64)) ** 2).sum(-1)
    want = np.argsort(full, axis=1, kind="stable")[:, :n_probes]
    swaps = 0
    for r in range(len(queries)):
        assert len(set(probes_g[r])) == n_probes
        dg, dw = full[r, probes_g[r]], full[r, want[r]]
        np.testing.assert_allclose(dg, dw, rtol=rtol)          # rank by rank the same distance
        swaps += int((probes_g[r] != want[r]).sum())
    return swaps
