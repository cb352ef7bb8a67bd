"""The other benchmark configurations at reduced N: the same generators, row shapes, K and k as the
large runs of bench_configs.py, built and searched end to end by the HIP path and compared with the
oracle's own build and search (graph: identical rows up to near-ties; search on the oracle's graph:
identical ids and distances)."""
import numpy as np
import pytest
import torch

import workloads
from conftest import cached, step
from parity import assert_bitwise, compare_topk
from test_gpu_build import check_graph

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def search_both(gpu, orc, base, queries, adj, lam, k, L, lv, mode):
    g = gpu.ann_graph_import(dev(adj), dev(lam), base.shape[1])
    ids, s = gpu.ann_search_ex(g, dev(base), dev(queries), k, L, mode=mode, lambda_visit=lv)
    ref = orc.search(adj, lam, base, queries, k, L, lv)
    return ids.cpu().numpy(), s.cpu().numpy(), ref


def test_gist_shape_build_and_search(gpu, orc):
    """d = 960 real-valued rows, K = 32, k = 10: the wide-row k-NN kernel, the 64-lane row shape of the
    diversification and of both search kernels."""
    step("config shape: gist-like 2,500 x 960")
    def make():
        base, queries = workloads.gist_like(N=2500, nq=40)
        adj, lam, st = orc.build_graph(base, 32, stages=True)
        return base, queries, adj, lam, st
    base, queries, adj, lam, st = cached("cfg_gist", make)
    assert check_graph(gpu, orc, base, 32, "gist shape", ref=(adj, lam, st)) == 0
    for mode, lv, L in ((1, 5, 64), (2, 10, 128)):
        ids, s, ref = search_both(gpu, orc, base, queries, adj, lam, 10, L, lv, mode)
        assert compare_topk(ids, s, ref[0], ref[1], f"gist shape mode {mode}") == 0
        assert_bitwise(s, ref[1], f"gist shape dists mode {mode}")


def test_deep_shape_build_and_search(gpu, orc):
    """d = 96 unit-norm rows, K = 32, k = 10 and k = 100 with lists up to 512 entries."""
    step("config shape: deep-like 6,000 x 96")
    def make():
        base, queries = workloads.deep_like(N=6000, nq=60)
        adj, lam, st = orc.build_graph(base, 32, stages=True)
        return base, queries, adj, lam, st
    base, queries, adj, lam, st = cached("cfg_deep", make)
    assert check_graph(gpu, orc, base, 32, "deep shape", ref=(adj, lam, st)) == 0
    for k, L, mode, lv in ((10, 64, 1, 5), (100, 128, 1, 5), (100, 512, 1, 5), (100, 256, 2, 10)):
        ids, s, ref = search_both(gpu, orc, base, queries, adj, lam, k, L, lv, mode)
        assert compare_topk(ids, s, ref[0], ref[1], f"deep shape k={k} L={L}") == 0
        assert_bitwise(s, ref[1], f"deep shape dists k={k} L={L}")


def test_scale_shape_uint8_build_and_search(gpu, orc):
    """uint8 rows of the 4,096-component generator, K = 32: build on the int8 matrix cores, search with
    the integer distance, both bit for bit."""
    step("config shape: 100M-style uint8 rows, 8,000 x 128")
    def make():
        chunk = next(iter(workloads.scale_u8_chunks(N=8000, chunk=8000)))
        base = np.ascontiguousarray(chunk[1] if isinstance(chunk, tuple) else chunk)
        queries = workloads.scale_u8_queries(nq=50)
        adj, lam, st = orc.build_graph(base, 32, stages=True)
        return base, queries, adj, lam, st
    base, queries, adj, lam, st = cached("cfg_u8", make)
    assert base.dtype == np.uint8
    g = gpu.ann_build_graph_ex(dev(base), 32)
    a2, l2 = gpu.ann_graph_export(g)
    assert_bitwise(a2.cpu().numpy(), adj, "u8 shape adjacency")
    assert_bitwise(l2.cpu().numpy(), lam, "u8 shape lambda")
    for L, mode, lv in ((32, 1, 5), (256, 1, 5), (32, 2, 10)):
        ids, s, ref = search_both(gpu, orc, base, queries, adj, lam, 10, L, lv, mode)
        assert_bitwise(ids, ref[0], f"u8 shape ids L={L}")
        assert_bitwise(s, ref[1], f"u8 shape dists L={L}")
