"""ann_search_multi_static (the entry point that allocates nothing) against ann_search_multi.

Two calls in a row through the C ABI, the second with a smaller input: the library's own scratch
keeps the first call's contents, and the second call's result must not depend on them.  Integer
data, so ids, distances and counters are compared bit for bit."""
import ctypes as C

import numpy as np
import pytest
import torch

from conftest import sift_case, step
from parity import assert_bitwise

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def call(gpu, entry, g, b, q, k, t0, seed):
    """One call straight through the C ABI with outputs and counters allocated by the caller."""
    import paper_2204_00824_amd.api as api
    lib = gpu.load_library()
    nq = q.shape[0]
    ids = torch.full((nq, k), -7, dtype=torch.int32, device="cuda")
    s = torch.full((nq, k), -7.0, dtype=torch.float32, device="cuda")
    st = torch.zeros((nq, 3), dtype=torch.int32, device="cuda")
    prm = api._SearchParams()
    lib.ann_search_params_default(C.byref(prm))
    prm.seed = seed
    prm.stream = int(torch.cuda.current_stream().cuda_stream)
    if entry == "ann_search_multi":         # the existing entry point takes the caller's workspace
        ws = torch.empty(max(lib.ann_search_multi_workspace_bytes(nq, t0), 8), dtype=torch.uint8, device="cuda")
        rc = lib.ann_search_multi(g.ptr, b.data_ptr(), q.data_ptr(), nq, k, t0, C.byref(prm), ws.data_ptr(), ws.numel(),
                                  ids.data_ptr(), s.data_ptr(), st.data_ptr())
    else:
        rc = lib.ann_search_multi_static(g.ptr, b.data_ptr(), q.data_ptr(), nq, k, t0, C.byref(prm), ids.data_ptr(),
                                         s.data_ptr(), st.data_ptr())
    torch.cuda.synchronize()
    return rc, ids.cpu().numpy(), s.cpu().numpy(), st.cpu().numpy()


def test_static_scratch_matches_the_allocating_entry_point(gpu, orc):
    base, queries, adj, lam = sift_case(orc)[:4]
    g = gpu.ann_graph_import(dev(adj), dev(lam), base.shape[1])
    b = dev(base)
    # first call: 64 queries x 32 searches = 2,048, the whole scratch; second: 5 x 3
    for nq, k, t0, seed in ((64, 10, 32, 0), (5, 7, 3, 11)):
        step(f"ann_search_multi_static nq={nq} t0={t0}")
        q = dev(queries[:nq])
        rc1, ids1, s1, st1 = call(gpu, "ann_search_multi_static", g, b, q, k, t0, seed)
        assert rc1 == 0, gpu.ann_last_error()
        rc0, ids0, s0, st0 = call(gpu, "ann_search_multi", g, b, q, k, t0, seed)
        assert rc0 == 0, gpu.ann_last_error()
        assert_bitwise(ids1, ids0, f"ids nq={nq}")
        assert_bitwise(s1, s0, f"dists nq={nq}")
        assert_bitwise(st1, st0, f"counters nq={nq}")
        # and both equal the oracle's multi-search
        ref = orc.search_multi(adj, lam, base, queries[:nq], k, t0, want_stats=True, max_hops=16, lambda_visit=10,
                               seed=seed, qi_offset=0)
        assert_bitwise(ids1, ref[0], f"oracle ids nq={nq}")
        assert_bitwise(s1, ref[1], f"oracle dists nq={nq}")


def test_static_scratch_limit_is_an_error(gpu, orc):
    step("ann_search_multi_static over its limit")
    base, queries, adj, lam = sift_case(orc)[:4]
    g = gpu.ann_graph_import(dev(adj), dev(lam), base.shape[1])
    rc, ids, s, _ = call(gpu, "ann_search_multi_static", g, dev(base), dev(queries[:65]), 10, 32, 0)
    assert rc == 4 and "2048" in gpu.ann_last_error()          # ANN_EUNSUPPORTED, outputs untouched
    assert (ids == -7).all() and (s == -7.0).all()
