"""More rows than a 1-D grid of one wavefront per row can hold (2^26 = 67,108,864): neighbourhood propagation,
diversification, export and search on 68,157,477 x 16 uint8 rows, checked on sampled rows the oracle can
recompute -- among them rows on both sides of 2^26 and the very last rows of the set.  The header's limit is
N < 2^27 (the id field of the packed adjacency word); this is the size class it is tested in."""
import numpy as np
import pytest
import torch

from conftest import step
from parity import assert_bitwise

pytestmark = pytest.mark.gpu

N = (1 << 26) + (1 << 20) + 37
D, K = 16, 8
FOLD = 1 << 26


def test_build_and_search_beyond_two_to_26_rows(gpu, orc):
    step(f"large N: generating {N} x {D} uint8")
    gen = torch.Generator(device="cuda")
    gen.manual_seed(2026)
    base = torch.randint(0, 256, (N, D), dtype=torch.uint8, device="cuda", generator=gen)
    step("large N: ann_knn_descent, 2 iterations")
    ids, s, done, _ = gpu.ann_knn_descent(base, K, S=4, max_iters=2, delta=0.0, seed=3)
    assert done == 2
    step("large N: ann_build_graph_ex (same propagation, then the diversification)")
    g = gpu.ann_build_graph_ex(base, K, knn_mode=1, descent_S=4, descent_iters=2, descent_delta=0.0, descent_seed=3)
    adj, lam = gpu.ann_graph_export(g)
    torch.cuda.synchronize()

    # ---- sampled nodes through the oracle's stage 1 / reverse / stage 2, on the rows that can influence them
    rng = np.random.default_rng(5)
    sample = np.unique(np.concatenate([rng.choice(N, 32, replace=False), np.arange(FOLD - 16, FOLD + 16),
                                       np.arange(N - 32, N)])).astype(np.int64)
    step(f"large N: masked oracle chain for {len(sample)} sampled nodes")
    sample_t = torch.from_numpy(sample).cuda()
    lists_them = torch.isin(ids, sample_t.to(torch.int32)).any(dim=1)       # rows y with a sampled node in knn(y)
    lists_them[sample_t] = True
    need = torch.nonzero(lists_them).flatten()
    need_ids, need_s = ids[need].cpu().numpy(), s[need].cpu().numpy()
    need = need.cpu().numpy()
    rows = np.unique(np.concatenate([need, need_ids[need_ids >= 0].astype(np.int64)]))   # sorted: the remap keeps id order
    base_c = base[torch.from_numpy(rows).cuda()].cpu().numpy()
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
    assert_bitwise(adj[sample_t].cpu().numpy(), adj_o, "adjacency of sampled nodes")
    assert_bitwise(lam[sample_t].cpu().numpy(), lam_o[sample_c], "lambda of sampled nodes")

    # ---- properties of every row, on the device
    valid = adj >= 0
    assert bool(valid[:, 0].all()), "a node without any edge"
    assert int(adj.max()) < N and not bool((adj == torch.arange(N, device="cuda", dtype=torch.int32)[:, None]).any())
    assert bool((valid[:, :-1] >= valid[:, 1:]).all())                      # prefixes
    assert int(adj[FOLD:].max()) >= FOLD                                    # the rows past 2^26 are part of the graph

    # ---- search: the whole launch against the oracle on the exported graph
    step("large N: search, 256 queries, L = 32")
    q = torch.randint(0, 256, (256, D), dtype=torch.uint8, device="cuda", generator=gen).to(torch.float32)
    got = gpu.ann_search_ex(g, base, q, 10, 32, mode=1, lambda_visit=10, want_stats=True)
    ref = orc.search(adj.cpu().numpy(), lam.cpu().numpy(), base.cpu().numpy(), q.cpu().numpy(), 10, 32, 10,
                     want_stats=True)
    assert_bitwise(got[0].cpu().numpy(), ref[0], "ids")
    assert_bitwise(got[1].cpu().numpy(), ref[1], "dists")
    assert np.array_equal(got[2].hops.cpu().numpy(), ref[2][:, 0])
    assert int(got[0].max()) >= FOLD                                         # some answers lie past 2^26
