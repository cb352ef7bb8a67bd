"""Parity of the HIP neighbourhood-propagation k-NN builder with the oracle: the lists after every
number of iterations are identical (the method's result does not depend on execution order), for
each row type and list/sample size; then the graph built from them."""
import numpy as np
import pytest
import torch

import workloads
from conftest import step
from parity import assert_bitwise, compare_topk

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("iters", [0, 1, 2, 4])
def test_integer_rows_every_iteration(gpu, orc, iters):
    step(f"descent sift-like 4000 x 128, K=32 S=16, {iters} iterations")
    base, _ = workloads.sift_like(N=4000, nq=1, seed=41)
    ids_o, s_o, done_o, ch_o = orc.knn_descent(base, 32, S=16, max_iters=iters, delta=0.0, seed=5)
    ids, s, done, last = gpu.ann_knn_descent(dev(base), 32, S=16, max_iters=iters, delta=0.0, seed=5)
    assert done == done_o == iters
    assert_bitwise(ids.cpu().numpy(), ids_o, "descent ids")
    assert_bitwise(s.cpu().numpy(), s_o, "descent dists")
    if iters:
        assert last == ch_o[-1]


@pytest.mark.parametrize("K,S,d,u8", [(16, 8, 32, False), (8, 2, 8, False), (64, 16, 16, False), (32, 16, 128, True),
                                      (20, 4, 100, False), (48, 16, 960, False)])
def test_shapes_and_sample_sizes(gpu, orc, K, S, d, u8):
    step(f"descent K={K} S={S} d={d} u8={u8}")
    if u8:
        base = workloads.sift_like(N=3000, nq=1, d=d, seed=42)[0].astype(np.uint8)
    else:
        base = workloads.single_gaussian(2500, d, seed=43)
    ids_o, s_o, done_o, ch_o = orc.knn_descent(base, K, S=S, max_iters=3, delta=0.0, seed=11)
    ids, s, done, last = gpu.ann_knn_descent(dev(base), K, S=S, max_iters=3, delta=0.0, seed=11)
    assert done == done_o
    assert compare_topk(ids.cpu().numpy(), s.cpu().numpy(), ids_o, s_o, "descent") == 0
    assert last == ch_o[-1]


@pytest.mark.parametrize("which", ["A", "B"])
def test_hand_worked_example(gpu, orc, which):
    """tests/golden/knn_descent_line8.json: the lists derived by hand, not only the oracle's."""
    step(f"descent hand-worked line of 8 points, case {which}")
    from test_oracle_descent import line8_case
    doc, case, base, init = line8_case(which)
    for it in (1, 2):
        want = case[f"after_iteration_{it}"]
        ids, s, done, last = gpu.ann_knn_descent(dev(base), doc["K"], S=doc["S"], max_iters=it, delta=0.0,
                                                 init_ids=dev(init))
        assert done == it and ids.cpu().numpy().tolist() == want["ids"] and last == want["changed"]


def test_stops_by_delta_and_accepts_start_lists(gpu, orc):
    step("descent: delta stop, caller's start lists, exact graph as fixed point")
    base = workloads.single_gaussian(3000, 8, seed=44)
    ids_o, s_o, done_o, ch_o = orc.knn_descent(base, 16, S=8, max_iters=20, delta=0.002, seed=2)
    ids, s, done, last = gpu.ann_knn_descent(dev(base), 16, S=8, max_iters=20, delta=0.002, seed=2)
    assert done == done_o < 20 and last == ch_o[-1]
    assert_bitwise(ids.cpu().numpy(), ids_o, "ids at the delta stop")
    exact_ids, exact_s = orc.knn(base, 16)
    ids, s, done, last = gpu.ann_knn_descent(dev(base), 16, S=8, max_iters=3, delta=0.0, init_ids=dev(exact_ids))
    assert done == 1 and last == 0
    assert_bitwise(ids.cpu().numpy(), exact_ids, "fixed point ids")
    assert_bitwise(s.cpu().numpy(), exact_s, "fixed point dists")
    rec = np.mean([len(set(a) & set(b)) for a, b in zip(ids_o, exact_ids)]) / 16
    assert rec > 0.9


def test_graph_built_from_propagated_lists(gpu, orc):
    step("build with knn_mode=1 vs oracle diversification of the oracle's propagated lists")
    base, q = workloads.sift_like(N=5000, nq=50, seed=45)
    K = 16
    ids_o, s_o, _, _ = orc.knn_descent(base, K, S=8, max_iters=12, delta=0.001, seed=0)
    g1 = orc.stage1(base, ids_o, s_o, 1.2)
    g2 = orc.reverse(base, g1[0], g1[2], 2 * K)
    adj_o, lam_o = orc.stage2(base, g2[0], g2[1], g2[2], 9, K)
    g = gpu.ann_build_graph_ex(dev(base), K, knn_mode=1)
    adj, lam = gpu.ann_graph_export(g)
    assert_bitwise(adj.cpu().numpy(), adj_o, "adj from propagated lists")
    assert_bitwise(lam.cpu().numpy(), lam_o, "lam from propagated lists")
    with pytest.raises(gpu.AnnError):
        gpu.ann_knn_descent(dev(base), K, S=3)
