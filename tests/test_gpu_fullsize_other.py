"""Sampled parity at the full size of the two real-valued configurations that bench.py does not time: 1,000,000 x 960
(gist-like) and 10,000,000 x 96 (deep-like, unit norm).  The two take about 75 s together, most of it generating the rows
on the host; TSDG_SKIP_FULLSIZE_OTHER=1 leaves them out (the same paths are covered at reduced N by
test_gpu_config_shapes.py).

What is compared: sampled rows of the exact k-NN lists with the oracle's brute force; sampled nodes of the graph with
the oracle's stage 1 / reverse / stage 2 run on a compacted copy of the rows that can influence them (ids renumbered
in order, which keeps every (s, id) comparison); sampled rows of a whole search launch with the oracle's search on the
exported graph."""
import os

import numpy as np
import pytest
import torch

import workloads
from conftest import step
from parity import assert_bitwise, compare_topk

pytestmark = [pytest.mark.gpu,
              pytest.mark.skipif(os.environ.get("TSDG_SKIP_FULLSIZE_OTHER") == "1",
                                 reason="left out by TSDG_SKIP_FULLSIZE_OTHER=1")]

K = 32


def sampled_graph_parity(gpu, orc, b, knn_id, knn_s, adj, lam, sample, what):
    """b, knn_id, knn_s, adj, lam: device tensors of the whole set; sample: sorted int64 numpy ids."""
    sample_t = torch.from_numpy(sample).cuda()
    lists_them = torch.isin(knn_id, sample_t.to(torch.int32)).any(dim=1)
    lists_them[sample_t] = True
    need = torch.nonzero(lists_them).flatten()
    need_ids, need_s = knn_id[need].cpu().numpy(), knn_s[need].cpu().numpy()
    need = need.cpu().numpy()
    rows = np.unique(np.concatenate([need, need_ids[need_ids >= 0].astype(np.int64)]))
    base_c = b[torch.from_numpy(rows).cuda()].cpu().numpy()
    m_id = np.full((len(rows), K), -1, np.int32)
    m_s = np.full((len(rows), K), np.inf, np.float32)
    at = np.searchsorted(rows, need)
    m_id[at] = np.where(need_ids >= 0, np.searchsorted(rows, np.maximum(need_ids, 0)), -1).astype(np.int32)
    m_s[at] = need_s
    g1_id, g1_s, g1_deg = orc.stage1(base_c, m_id, m_s, 1.2)
    g2_id, g2_s, g2_deg = orc.reverse(base_c, g1_id, g1_deg, 2 * K)
    sample_c = np.searchsorted(rows, sample)
    keep = np.zeros(len(rows), bool)
    keep[sample_c] = True
    adj_o, lam_o = orc.stage2(base_c, g2_id, g2_s, np.where(keep, g2_deg, 0).astype(np.int32), 9, K)
    adj_o = np.where(adj_o >= 0, rows[np.maximum(adj_o, 0)], -1).astype(np.int32)[sample_c]
    assert_bitwise(adj[sample_t].cpu().numpy(), adj_o, f"{what}: adjacency of sampled nodes")
    assert_bitwise(lam[sample_t].cpu().numpy(), lam_o[sample_c], f"{what}: lambda of sampled nodes")


def full_size_case(gpu, orc, what, base, queries, L):
    N, d = base.shape
    b, q = torch.from_numpy(base).cuda(), torch.from_numpy(queries).cuda()
    step(f"{what}: ann_knn")
    knn_id, knn_s = gpu.ann_knn(b, K)
    rows = np.random.default_rng(11).choice(N, size=24, replace=False)
    step(f"{what}: oracle brute force on 24 sampled rows")
    ids, s = orc.bruteforce(base, base[rows], K + 1)
    got_i, got_s = knn_id[torch.from_numpy(rows).cuda()].cpu().numpy(), knn_s[torch.from_numpy(rows).cuda()].cpu().numpy()
    ref_i = np.stack([ids[t][ids[t] != r][:K] for t, r in enumerate(rows)])
    ref_s = np.stack([s[t][ids[t] != r][:K] for t, r in enumerate(rows)])
    assert compare_topk(got_i, got_s, ref_i, ref_s, f"{what}: knn rows") == 0
    assert_bitwise(got_s, ref_s, f"{what}: knn distances")

    step(f"{what}: ann_build_graph_ex")
    g = gpu.ann_build_graph_ex(b, K)
    adj, lam = gpu.ann_graph_export(g)
    step(f"{what}: oracle stages for 100 sampled nodes")
    sample = np.sort(np.random.default_rng(12).choice(N, size=100, replace=False)).astype(np.int64)
    sampled_graph_parity(gpu, orc, b, knn_id, knn_s, adj, lam, sample, what)
    del knn_id, knn_s

    step(f"{what}: whole search launch, L = {L}; 200 of its rows against the oracle")
    ids, s, st = gpu.ann_search_ex(g, b, q, 10, L, mode=1, lambda_visit=5, want_stats=True)
    n = min(200, len(queries))
    ref = orc.search(adj.cpu().numpy(), lam.cpu().numpy(), base, queries[:n], 10, L, 5, want_stats=True)
    assert compare_topk(ids[:n].cpu().numpy(), s[:n].cpu().numpy(), ref[0], ref[1], f"{what}: search") == 0
    assert_bitwise(s[:n].cpu().numpy(), ref[1], f"{what}: search distances")
    assert np.array_equal(st.hops[:n].cpu().numpy(), ref[2][:, 0])


def test_gist_like_full_size(gpu, orc):
    step("full size: generating 1,000,000 x 960")
    base, queries = workloads.gist_like()
    full_size_case(gpu, orc, "gist-like 1M x 960", base, queries, 64)


def test_deep_like_full_size(gpu, orc):
    step("full size: generating 10,000,000 x 96")
    base, queries = workloads.deep_like()
    full_size_case(gpu, orc, "deep-like 10M x 96", base, queries, 64)
