"""Parity at the headline size (N = 1,000,000, d = 128, K = 32, 10,000-query launch, the
configuration bench.py times), on sampled outputs the oracle can compute one by one."""
import numpy as np
import pytest
import torch

import workloads
from conftest import cached, step
from parity import assert_bitwise

pytestmark = pytest.mark.gpu

N, D, K, NQ = 1_000_000, 128, 32, 10_000


def full_case(gpu):
    def make():
        step("full size: generating 1M x 128")
        base, queries = workloads.sift_like(N=N, nq=NQ)
        b, q = torch.from_numpy(base).cuda(), torch.from_numpy(queries).cuda()
        step("full size: ann_knn")
        knn_id, knn_s = gpu.ann_knn(b, K)
        step("full size: ann_build_graph")
        g = gpu.ann_build_graph(b, K)
        adj, lam = gpu.ann_graph_export(g)
        return dict(base=base, queries=queries, b=b, q=q, g=g, knn_id=knn_id.cpu().numpy(),
                    knn_s=knn_s.cpu().numpy(), adj=adj.cpu().numpy(), lam=lam.cpu().numpy())
    return cached("full", make)


def test_knn_rows_sampled(gpu, orc):
    c = full_case(gpu)
    rows = np.random.default_rng(1).choice(N, size=48, replace=False)
    step("full size: oracle brute force on 48 sampled rows")
    ids, s = orc.bruteforce(c["base"], c["base"][rows], K + 1)
    for t, r in enumerate(rows):
        keep = ids[t] != r
        assert_bitwise(c["knn_id"][r], ids[t][keep][:K], f"knn ids row {r}")
        assert_bitwise(c["knn_s"][r], s[t][keep][:K], f"knn dists row {r}")


def test_graph_rows_sampled(gpu, orc):
    """Final adjacency of 150 sampled nodes, recomputed by the oracle's stage 1 / reverse /
    stage 2 from the k-NN lists.  Only the rows that can influence a sampled node are given to
    the oracle (the node itself and every y that lists it among its k-NN); all other rows are
    blanked, which does not change the sampled nodes' result."""
    c = full_case(gpu)
    knn_id, knn_s = c["knn_id"], c["knn_s"]
    sample = np.random.default_rng(2).choice(N, size=150, replace=False)
    step("full size: masked oracle chain for 150 sampled nodes")
    need = np.zeros(N, bool)
    need[sample] = True
    need[np.isin(knn_id, sample).any(axis=1)] = True
    m_id = np.where(need[:, None], knn_id, -1).astype(np.int32)
    m_s = np.where(need[:, None], knn_s, np.inf).astype(np.float32)
    g1_id, g1_s, g1_deg = orc.stage1(c["base"], m_id, m_s, 1.2)
    g2_id, g2_s, g2_deg = orc.reverse(c["base"], g1_id, g1_deg, 2 * K)
    keep = np.zeros(N, bool)
    keep[sample] = True
    g2_deg = np.where(keep, g2_deg, 0).astype(np.int32)
    adj_o, lam_o = orc.stage2(c["base"], g2_id, g2_s, g2_deg, 9, K)
    assert_bitwise(c["adj"][sample], adj_o[sample], "adjacency of sampled nodes")
    assert_bitwise(c["lam"][sample], lam_o[sample], "lambda of sampled nodes")


def test_graph_invariants_at_full_size(gpu):
    c = full_case(gpu)
    adj, lam = c["adj"], c["lam"]
    valid = adj >= 0
    assert adj.shape == (N, K) and adj.max() < N
    assert np.all(valid[:, 0]) and np.all(valid[:, :-1] >= valid[:, 1:])         # prefixes
    assert np.all(lam[valid] <= 9) and np.all(lam[~valid] == 255)
    lam_i = np.where(valid, lam, 255).astype(np.int16)
    assert np.all(np.diff(lam_i, axis=1) >= 0)                                    # sorted by lambda
    assert not np.any(adj == np.arange(N)[:, None])                               # no self loops
    srt = np.sort(np.where(valid, adj, -np.arange(1, K + 1)[None, :]), axis=1)
    assert np.all(np.diff(srt, axis=1) != 0)                                      # no repeats


@pytest.mark.parametrize("L", [32, 128])
def test_search_rows_sampled(gpu, orc, L):
    """The whole 10,000-query launch; 300 of its rows recomputed by the oracle on the exported graph."""
    c = full_case(gpu)
    step(f"full size: 10,000-query launch, L={L}")
    ids, s, st = gpu.ann_search_ex(c["g"], c["b"], c["q"], 10, L, mode=1, lambda_visit=5, want_stats=True)
    torch.cuda.synchronize()
    q0 = 4321
    ref = orc.search(c["adj"], c["lam"], c["base"], c["queries"][q0:q0 + 300], 10, L, 5, qi_offset=q0,
                     want_stats=True)
    assert_bitwise(ids.cpu().numpy()[q0:q0 + 300], ref[0], "ids")
    assert_bitwise(s.cpu().numpy()[q0:q0 + 300], ref[1], "dists")
    assert np.array_equal(st.hops.cpu().numpy()[q0:q0 + 300], ref[2][:, 0])
    # properties that hold for every row of the launch
    ids_h, s_h = ids.cpu().numpy(), s.cpu().numpy()
    assert np.all(np.diff(s_h, axis=1) >= 0) and ids_h.min() >= 0 and ids_h.max() < N
    assert np.all(np.diff(np.sort(ids_h, axis=1), axis=1) != 0)
    pick = np.random.default_rng(3).choice(NQ, size=200, replace=False)
    for r in pick:                                            # returned distances are the canonical ones
        t = c["queries"][r][None, :] - c["base"][ids_h[r]]
        assert np.array_equal(np.sum(t.astype(np.float64) ** 2, axis=1).astype(np.float32), s_h[r])


def test_small_batch_rows_sampled(gpu, orc):
    c = full_case(gpu)
    step("full size: small-batch calls (1, 16, 100 queries)")
    for bs, q0 in ((1, 7), (16, 100), (100, 2000)):
        q = c["q"][q0:q0 + bs].contiguous()
        ids, s = gpu.ann_search_ex(c["g"], c["b"], q, 10, 32, mode=2, lambda_visit=10, qi_offset=q0)
        ref = orc.search(c["adj"], c["lam"], c["base"], c["queries"][q0:q0 + bs], 10, 32, 10, qi_offset=q0)
        assert_bitwise(ids.cpu().numpy(), ref[0], f"small batch {bs} ids")
        assert_bitwise(s.cpu().numpy(), ref[1], f"small batch {bs} dists")
