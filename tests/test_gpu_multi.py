"""Parity of the HIP small-batch multi-search (Alg. 1) with the CPU oracle."""
import numpy as np
import pytest
import torch

import workloads
from conftest import cached, sift_case, step, tiny_case
from parity import assert_bitwise, compare_topk

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run_both(gpu, orc, case, k, t0, **kw):
    base, queries, adj, lam = case[:4]
    g = gpu.ann_graph_import(dev(adj), dev(lam), base.shape[1])
    okw = dict(max_hops=kw.get("max_hops", 0) or 16, lambda_visit=kw.get("lambda_visit", 0) or 10,
               seed=kw.get("seed", 0), qi_offset=kw.get("qi_offset", 0))
    ref = orc.search_multi(adj, lam, base, queries, k, t0, want_stats=True, **okw)
    ids, s, st = gpu.ann_search_multi(g, dev(base), dev(queries), k, t0, want_stats=True, **kw)
    torch.cuda.synchronize()
    return (ids.cpu().numpy(), s.cpu().numpy(), st), ref


@pytest.mark.parametrize("t0,kw", [(1, {}), (4, {}), (16, dict(seed=7)), (3, dict(max_hops=1)), (8, dict(lambda_visit=5)),
                                   (2, dict(qi_offset=500, max_hops=3))])
def test_integer_data_matches_oracle_exactly(gpu, orc, t0, kw):
    step(f"multi-search sift20k t0={t0} {kw}")
    (ids, s, st), ref = run_both(gpu, orc, sift_case(orc), 10, t0, **kw)
    assert_bitwise(ids, ref[0], "ids")
    assert_bitwise(s, ref[1], "dists")
    assert np.array_equal(st.hops.cpu().numpy(), ref[2][:, 0])
    assert np.array_equal(st.dist_evals.cpu().numpy(), ref[2][:, 1])


@pytest.mark.parametrize("k,t0", [(1, 2), (32, 6)])
def test_tiny_matches_oracle(gpu, orc, k, t0):
    step(f"multi-search tiny k={k} t0={t0}")
    (ids, s, st), ref = run_both(gpu, orc, tiny_case(orc), k, t0)
    assert compare_topk(ids, s, ref[0], ref[1], "tiny") == 0
    assert_bitwise(s, ref[1], "tiny dists")
    assert np.array_equal(st.hops.cpu().numpy(), ref[2][:, 0])


@pytest.mark.parametrize("d,N", [(8, 3000), (96, 4000), (960, 2500)])
def test_row_shapes(gpu, orc, d, N):
    step(f"multi-search row shape d={d}")
    def make():
        base, queries = workloads.single_gaussian(N, d, seed=d, nq=64)
        adj, lam = orc.build_graph(base, 16)
        return base, queries, adj, lam
    (ids, s, st), ref = run_both(gpu, orc, cached(f"gauss{d}", make), 10, 4)
    assert compare_topk(ids, s, ref[0], ref[1], f"d={d}") == 0
    assert np.array_equal(st.hops.cpu().numpy(), ref[2][:, 0])


def test_uint8_rows_and_wide_rows(gpu, orc):
    step("multi-search uint8 / K=64 slot rule")
    def make():
        base, queries = workloads.sift_like(N=8000, nq=100, seed=5)
        b8 = base.astype(np.uint8)
        adj, lam = orc.build_graph(b8, 16)
        return b8, queries, adj, lam
    case8 = cached("u8", make)
    (ids, s, st), ref = run_both(gpu, orc, case8, 10, 4)
    assert_bitwise(ids, ref[0], "u8 ids")
    assert_bitwise(s, ref[1], "u8 dists")
    # queries that are not integers (and one outside the byte range) take the fp64 route on the same byte rows
    mixed = case8[1].copy()
    mixed[::2] += np.float32(0.375)
    mixed[1, 0] = 300.0
    (ids, s, st), ref = run_both(gpu, orc, (case8[0], mixed, case8[2], case8[3]), 10, 4)
    assert_bitwise(ids, ref[0], "u8 mixed ids")
    assert_bitwise(s, ref[1], "u8 mixed dists")
    # K = 64: positions p and p+32 of a row compete for one slot
    def make64():
        base, queries = workloads.single_gaussian(2000, 8, seed=64, nq=40)
        adj, lam = orc.build_graph(base, 64, lambda0=30, alpha=3.0)
        return base, queries, adj, lam
    case = cached("k64", make64)
    assert (case[2][:, 40] >= 0).mean() > 0.2          # rows longer than 32 do occur
    (ids, s, st), ref = run_both(gpu, orc, case, 16, 3, lambda_visit=31)
    assert compare_topk(ids, s, ref[0], ref[1], "K=64") == 0
    assert np.array_equal(st.dist_evals.cpu().numpy(), ref[2][:, 1])


def test_arguments(gpu, orc):
    step("multi-search arguments")
    base, queries, adj, lam = tiny_case(orc)[:4]
    g = gpu.ann_graph_import(dev(adj), dev(lam), 32)
    b, q = dev(base), dev(queries)
    for k, t0 in ((0, 1), (33, 1), (10, 0), (10, 2000)):
        with pytest.raises(gpu.AnnError):
            gpu.ann_search_multi(g, b, q, k, t0)
    ids, s = gpu.ann_search_multi(g, b, q[:0], 5, 2)
    assert ids.shape == (0, 5)
    # two calls in a row with a growing scratch need
    a1 = gpu.ann_search_multi(g, b, q[:10].contiguous(), 5, 2)[0].cpu().numpy()
    a2 = gpu.ann_search_multi(g, b, q, 5, 8)[0].cpu().numpy()
    a3 = gpu.ann_search_multi(g, b, q[:10].contiguous(), 5, 2)[0].cpu().numpy()
    assert np.array_equal(a1, a3) and a2.shape == (100, 5)


def test_merge_with_many_distinct_survivors(gpu, orc):
    """One hop gives rankings of 16 entries, so with k = 32 no ranking is full, nothing can be
    filtered and thousands of distinct keys reach the merge: the table-overflow path."""
    step("multi-search merge fallback")
    def make():
        g = np.random.default_rng(77)
        base, queries = workloads.single_gaussian(5000, 8, seed=78, nq=6)
        adj = np.stack([g.choice(np.delete(np.arange(5000), i), size=32, replace=False) for i in range(5000)])
        lam = np.zeros((5000, 32), np.uint8)
        return base, queries, adj.astype(np.int32), lam
    case = cached("randgraph", make)
    for t0, k, T in ((400, 32, 1), (300, 20, 2)):
        (ids, s, st), ref = run_both(gpu, orc, case, k, t0, max_hops=T, lambda_visit=1)
        assert compare_topk(ids, s, ref[0], ref[1], f"fallback t0={t0}") == 0
        assert np.array_equal(st.dist_evals.cpu().numpy(), ref[2][:, 1])
