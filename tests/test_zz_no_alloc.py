"""The search entry point that allocates nothing (ivfpq_search_static: the library's fixed device scratch
instead of a caller workspace) against ivfpq_search, through the C ABI: identical ids and distances, on two
calls in a row, the second with a smaller input; both also agree with the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from util_parity import assert_topk_matches

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2301_06672_amd as pkg
    pkg.lib()
    return pkg


def _step(msg):
    print(f"[no-alloc] {msg}", flush=True)


def _index(P, n, d, n_lists, pq_dim, pq_bits, salt):
    arrays = si.random_index_arrays(n, d, n_lists, pq_dim, pq_bits, salt=salt)
    oidx = oracle.make_index(d, n_lists, pq_dim, pq_bits, *arrays)
    gidx = P.Index.ivfpq_index_from_arrays(d, n_lists, pq_dim, pq_bits, *arrays).ivfpq_upload()
    return oidx, gidx


@pytest.mark.parametrize("dtype", [oracle.LUT_E5M3, oracle.LUT_FP32])
def test_static_scratch_search_equals_workspace_search(P, dtype):
    # 60,000 vectors in 40 clusters, 12 probes: a query's share of the scratch is about 300 KB, so the
    # 1,500-query call runs in several tiles of the 64 MiB array and the 200-query call in one
    oidx, gidx = _index(P, 60000, 64, 40, 32, 8, salt=4242)
    rng = np.random.default_rng(4242)
    for nq, n_probes, k in ((1500, 12, 10), (200, 7, 100)):
        q = rng.standard_normal((nq, 64)).astype(np.float32)
        _step(f"dtype={dtype} nq={nq} P={n_probes} k={k}: workspace call")
        ids_w, d_w = gidx.ivfpq_search(q, n_probes, k, dtype)
        torch.cuda.synchronize()
        _step(f"dtype={dtype} nq={nq} P={n_probes} k={k}: static-scratch call")
        qd = torch.from_numpy(q).cuda()
        out = (torch.empty((nq, k), dtype=torch.int64, device="cuda"), torch.empty((nq, k), dtype=torch.float32, device="cuda"))
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        ids_s, d_s = gidx.ivfpq_search_static(qd, n_probes, k, dtype, out=out)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free_before          # the call took no device memory
        np.testing.assert_array_equal(ids_s.cpu().numpy(), ids_w.cpu().numpy())
        np.testing.assert_array_equal(d_s.cpu().numpy(), d_w.cpu().numpy())
        probes, _ = gidx.ivfpq_select_probes(qd[:64], n_probes)
        ids_o, d_o = oracle.search(oidx, q[:64], n_probes, k, dtype, probes=probes.cpu().numpy().view(np.uint32))
        assert_topk_matches(ids_s.cpu().numpy()[:64], d_s.cpu().numpy()[:64], ids_o, d_o, context="static scratch")
    gidx.ivfpq_free()


def test_static_scratch_search_edge_cases(P):
    oidx, gidx = _index(P, 3000, 32, 5, 16, 4, salt=77)
    # no queries: nothing happens; one query, one probe, k larger than the cluster
    gidx.ivfpq_search_static(np.zeros((0, 32), np.float32), 2, 5, oracle.LUT_FP16)
    q = np.random.default_rng(77).standard_normal((1, 32)).astype(np.float32)
    ids_w, d_w = gidx.ivfpq_search(q, 1, 1000, oracle.LUT_FP16)
    ids_s, d_s = gidx.ivfpq_search_static(q, 1, 1000, oracle.LUT_FP16)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(ids_s.cpu().numpy(), ids_w.cpu().numpy())
    np.testing.assert_array_equal(d_s.cpu().numpy(), d_w.cpu().numpy())
    gidx.ivfpq_free()
