"""The documented limits of the boundary, each against the oracle: longest rows (2,048 fp32 / 1,024
uint8 elements), K = 64 with the longest reverse lists, L = 512, the smallest set a graph accepts."""
import numpy as np
import pytest
import torch

import workloads
from conftest import cached, step
from parity import assert_bitwise, compare_topk

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def test_longest_fp32_rows(gpu, orc):
    step("d=2048 fp32: k-NN, build, search (64 lanes x 8 chunks)")
    base, q = workloads.single_gaussian(700, 2048, seed=11, nq=16)
    adj_o, lam_o, st = orc.build_graph(base, 8, stages=True)
    ids, s = gpu.ann_knn(dev(base), 8)
    assert compare_topk(ids.cpu().numpy(), s.cpu().numpy(), st["knn_id"], st["knn_s"], "knn d=2048") == 0
    g = gpu.ann_build_graph_ex(dev(base), 8)
    adj, lam = gpu.ann_graph_export(g)
    assert_bitwise(adj.cpu().numpy(), adj_o, "adj d=2048")
    assert_bitwise(lam.cpu().numpy(), lam_o, "lam d=2048")
    for mode in (1, 2):
        ids, s = gpu.ann_search_ex(g, dev(base), dev(q), 5, 24, mode=mode, lambda_visit=10)
        ref = orc.search(adj_o, lam_o, base, q, 5, 24, 10)
        assert compare_topk(ids.cpu().numpy(), s.cpu().numpy(), ref[0], ref[1], f"search d=2048 mode {mode}") == 0
    ids, s = gpu.ann_search_multi(g, dev(base), dev(q), 5, 4, max_hops=4)
    ref = orc.search_multi(adj_o, lam_o, base, q, 5, 4, max_hops=4)
    assert compare_topk(ids.cpu().numpy(), s.cpu().numpy(), ref[0], ref[1], "multi d=2048") == 0


def test_longest_uint8_rows(gpu, orc):
    step("d=1024 uint8: build and search (16 lanes x 4 chunks)")
    g0 = np.random.default_rng(12)
    base = g0.integers(0, 256, size=(900, 1024), dtype=np.uint8)
    base[::3] //= 4                                    # some structure: a third of the rows are dark
    q = g0.integers(0, 256, size=(20, 1024)).astype(np.float32)
    adj_o, lam_o = orc.build_graph(base, 8)
    g = gpu.ann_build_graph_ex(dev(base), 8)
    adj, lam = gpu.ann_graph_export(g)
    assert_bitwise(adj.cpu().numpy(), adj_o, "adj u8 d=1024")
    assert_bitwise(lam.cpu().numpy(), lam_o, "lam u8 d=1024")
    ids, s = gpu.ann_search_ex(g, dev(base), dev(q), 10, 32, mode=1, lambda_visit=10)
    ref = orc.search(adj_o, lam_o, base, q, 10, 32, 10)
    assert_bitwise(ids.cpu().numpy(), ref[0], "ids u8 d=1024")
    assert_bitwise(s.cpu().numpy(), ref[1], "dists u8 d=1024")


def test_widest_graph_and_longest_list(gpu, orc):
    step("K=64 (reverse lists of 128), L=512, k=L")
    base, q = workloads.sift_like(N=3000, nq=30, seed=13)
    base, q = base[:, :32].copy(), q[:, :32].copy()
    adj_o, lam_o = orc.build_graph(base, 64, lambda0=30)
    g = gpu.ann_build_graph_ex(dev(base), 64, lambda0=30)
    adj, lam = gpu.ann_graph_export(g)
    assert_bitwise(adj.cpu().numpy(), adj_o, "adj K=64")
    assert_bitwise(lam.cpu().numpy(), lam_o, "lam K=64")
    for mode in (1, 2):
        ids, s = gpu.ann_search_ex(g, dev(base), dev(q), 512, 512, mode=mode, lambda_visit=32)
        ref = orc.search(adj_o, lam_o, base, q, 512, 512, 32)
        assert_bitwise(ids.cpu().numpy(), ref[0], f"ids L=512 mode {mode}")
        assert_bitwise(s.cpu().numpy(), ref[1], f"dists L=512 mode {mode}")


def test_smallest_set(gpu, orc):
    step("N = K + 1: every node lists every other node")
    base = workloads.single_gaussian(9, 4, seed=14)
    adj_o, lam_o = orc.build_graph(base, 8)
    g = gpu.ann_build_graph_ex(dev(base), 8)
    adj, lam = gpu.ann_graph_export(g)
    assert_bitwise(adj.cpu().numpy(), adj_o, "adj N=9")
    assert_bitwise(lam.cpu().numpy(), lam_o, "lam N=9")
    ids, s = gpu.ann_search_ex(g, dev(base), dev(base), 9, 9, mode=1, lambda_visit=32, n_seeds=1)
    ref = orc.search(adj_o, lam_o, base, base, 9, 9, 32, n_seeds=1)
    assert_bitwise(ids.cpu().numpy(), ref[0], "ids N=9")
    with pytest.raises(gpu.AnnError):
        gpu.ann_build_graph_ex(dev(base[:8]), 8)       # N must exceed K
    # empty batches are valid for every search entry point
    e = dev(base[:0])
    assert gpu.ann_search_ex(g, dev(base), e, 3, 8)[0].shape == (0, 3)
    assert gpu.ann_search_multi(g, dev(base), e, 3, 2)[0].shape == (0, 3)
    assert gpu.ann_search_alg2(g, dev(base), e, 3, 0.0)[0].shape == (0, 3)


def test_largest_batch(gpu, orc):
    """2^22 queries in one call (the grid is one workgroup per query); one more is refused.  Sampled
    queries of the big call against the oracle (the seeds depend on the query's index in the batch)."""
    step("2^22 queries in one search call")
    from conftest import tiny_case
    base, _, adj, lam, _ = tiny_case(orc)
    g = gpu.ann_graph_import(dev(adj), dev(lam), base.shape[1])
    nq = 1 << 22
    gen = torch.Generator(device="cuda").manual_seed(5)
    q = torch.randn((nq + 1, base.shape[1]), generator=gen, device="cuda") * 3.0
    b = dev(base)
    ids, s = gpu.ann_search_ex(g, b, q[:nq], 10, 16, mode=1, lambda_visit=5)
    torch.cuda.synchronize()
    for lo in (0, 123_457, nq - 40):
        qs = q[lo:lo + 40].cpu().numpy()
        ref = orc.search(adj, lam, base, qs, 10, 16, 5, qi_offset=lo)
        got_i, got_s = ids[lo:lo + 40].cpu().numpy(), s[lo:lo + 40].cpu().numpy()
        assert compare_topk(got_i, got_s, ref[0], ref[1], f"queries from {lo}") == 0
    with pytest.raises(gpu.AnnError) as e:
        gpu.ann_search_ex(g, b, q, 10, 16, mode=1)
    assert e.value.status == 4
