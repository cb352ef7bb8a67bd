"""Pins for the oracle's best-first search.  CPU only."""
import numpy as np

import workloads


def np_canonical(base, q):
    t = (base.astype(np.float32) - q.astype(np.float32)[None, :]).astype(np.float32)
    return np.sum(t.astype(np.float64) ** 2, axis=1).astype(np.float32)


def np_topk(base, q, k):
    s = np_canonical(base, q)
    order = np.lexsort((np.arange(len(s)), s))[:k]
    return order.astype(np.int32), s[order]


def test_exhaustive_list_on_connected_graph_is_exact(orc):
    """L >= N on a connected graph: every node is reached and kept, so the
    first k entries are the exact top-k (recall 1.0)."""
    base, queries = workloads.single_gaussian(500, 8, seed=21, nq=20)
    adj, lam = orc.build_graph(base, 16)
    ids, s = orc.search(adj, lam, base, queries, 10, 500, 10)
    for i in range(20):
        e_ids, e_s = np_topk(base, queries[i], 10)
        assert np.array_equal(ids[i], e_ids)
        assert s[i].tobytes() == e_s.tobytes()
    gt, _ = orc.bruteforce(base, queries, 10)
    assert orc.recall(ids, gt) == 1.0


def test_all_nodes_as_seeds_is_exact_on_any_graph(orc):
    """With enough seeds to cover every node the graph does not matter."""
    base, queries = workloads.tiny(N=300, nq=10, d=8, components=6, seed=5)   # disconnected
    adj, lam = orc.build_graph(base, 6)
    ids, s = orc.search(adj, lam, base, queries, 5, 300, 10, n_seeds=20000)
    for i in range(10):
        e_ids, e_s = np_topk(base, queries[i], 5)
        assert np.array_equal(ids[i], e_ids) and s[i].tobytes() == e_s.tobytes()


def test_complete_graph_is_exact_after_expanding_once(orc):
    N, K = 13, 12
    base, queries = workloads.single_gaussian(N, 4, seed=22, nq=6)
    adj = np.array([[j for j in range(N) if j != i] for i in range(N)], np.int32)
    lam = np.zeros_like(adj, dtype=np.uint8)
    ids, s, st = orc.search(adj, lam, base, queries, 5, 5, 1, n_seeds=1, want_stats=True)
    for i in range(6):
        e_ids, e_s = np_topk(base, queries[i], 5)
        assert np.array_equal(ids[i], e_ids) and s[i].tobytes() == e_s.tobytes()
        assert st[i][1] == N                       # each node scored exactly once


def test_path_graph_walk_has_closed_form(orc):
    """Sorted points on a line, node i linked to i-1 and i+1, one seed, L = 1:
    the walk moves one node per hop towards the query and stops at the nearest
    point b.  From start a (interior, a != b): hops = |b-a|+1 and evaluations
    = 1 (seed) + 2 (both neighbours of a) + |b-a| (one new node per later hop)."""
    N = 200
    base = workloads.line_points(N, seed=3)
    adj = np.full((N, 2), -1, np.int32)
    lam = np.full((N, 2), 255, np.uint8)
    for i in range(N):
        nb = [j for j in (i - 1, i + 1) if 0 <= j < N]
        adj[i, :len(nb)] = nb
        lam[i, :len(nb)] = 0
    g = np.random.default_rng(4)
    checked = 0
    for qi in range(40):
        q = np.zeros((1, 4), np.float32)
        q[0, 0] = g.uniform(base[5, 0], base[N - 6, 0])
        b = int(np.argmin(np.abs(base[:, 0] - q[0, 0])))
        a = orc.seed_id(77, qi, 0, N)
        ids, s, st = orc.search(adj, lam, base, q, 1, 1, 1, n_seeds=1, seed=77, qi_offset=qi,
                                want_stats=True)
        assert ids[0][0] == b
        if 0 < a < N - 1 and 0 < b < N - 1 and a != b:
            assert st[0][0] == abs(b - a) + 1
            assert st[0][1] == 1 + 2 + abs(b - a)
            checked += 1
    assert checked > 20


def test_result_independent_of_visited_capacity_and_scoring_order(orc):
    base, queries = workloads.single_gaussian(3000, 10, seed=23, nq=40)
    adj, lam = orc.build_graph(base, 16)
    ref = orc.search(adj, lam, base, queries, 10, 48, 10, want_stats=True)
    for cap in (1, 7, 64, 1024):
        got = orc.search(adj, lam, base, queries, 10, 48, 10, visited_cap=cap, want_stats=True)
        assert np.array_equal(ref[0], got[0]) and np.array_equal(ref[1], got[1])
        assert np.array_equal(ref[2][:, 0], got[2][:, 0])          # same hops
        assert np.all(got[2][:, 1] >= ref[2][:, 1])                # lossy set only costs evaluations
    rev = orc.search(adj, lam, base, queries, 10, 48, 10, reverse_hop=True)
    assert np.array_equal(ref[0], rev[0]) and np.array_equal(ref[1], rev[1])


def test_lambda_prefix_and_hop_limit(orc):
    base, queries = workloads.single_gaussian(2000, 8, seed=24, nq=30)
    adj, lam = orc.build_graph(base, 16)
    # lambda_visit above every stored lambda == all edges; 1 == only lambda-0 edges
    all_e = orc.search(adj, lam, base, queries, 10, 32, 255, want_stats=True)
    ten = orc.search(adj, lam, base, queries, 10, 32, 10, want_stats=True)
    assert np.array_equal(all_e[0], ten[0])                        # lambda0 = 9 => identical
    one = orc.search(adj, lam, base, queries, 10, 32, 1, want_stats=True)
    assert one[2][:, 1].sum() < ten[2][:, 1].sum()                 # fewer evaluations
    adj0 = np.where(lam == 0, adj, -1)                             # graph cut to lambda == 0 ...
    lam0 = np.where(lam == 0, lam, 255).astype(np.uint8)
    cut = orc.search(adj0, lam0, base, queries, 10, 32, 255)
    assert np.array_equal(cut[0], one[0])                          # ... gives the same walk
    # hop limit T
    lim = orc.search(adj, lam, base, queries, 10, 32, 10, max_hops=3, want_stats=True)
    assert np.all(lim[2][:, 0] == 3)
    tr = orc.search(adj, lam, base, queries, 10, 32, 10, trace_cap=8)[2]
    tr3 = orc.search(adj, lam, base, queries, 10, 32, 10, max_hops=3, trace_cap=8)[2]
    assert np.array_equal(tr[:, :3], tr3[:, :3]) and np.all(tr3[:, 3:] == -1)


def test_list_properties(orc):
    """Returned entries are distinct, sorted by (s,id), carry the canonical
    distance of their id, and the first expansion is the closest seed."""
    base, queries = workloads.single_gaussian(2500, 12, seed=25, nq=25)
    adj, lam = orc.build_graph(base, 16)
    ids, s, tr = orc.search(adj, lam, base, queries, 20, 40, 10, seed=5, trace_cap=1)
    for i in range(25):
        assert len(set(ids[i])) == 20
        keys = list(zip(s[i], ids[i]))
        assert keys == sorted(keys)
        assert s[i].tobytes() == np_canonical(base[ids[i]], queries[i]).tobytes()
        seeds = sorted({orc.seed_id(5, i, j, 2500) for j in range(32)})
        ss = np_canonical(base[seeds], queries[i])
        best = seeds[int(np.lexsort((seeds, ss))[0])]
        assert tr[i][0] == best
    # fewer reachable nodes than k: padded with -1 / +inf
    small = workloads.single_gaussian(6, 4, seed=1)
    a = np.array([[(i + 1) % 6] for i in range(6)], np.int32)
    l0 = np.zeros_like(a, dtype=np.uint8)
    r_ids, r_s = orc.search(a, l0, small, small[:1], 8, 8, 1, n_seeds=1)
    assert np.all(r_ids[0][6:] == -1) and np.all(np.isinf(r_s[0][6:]))
    assert sorted(r_ids[0][:6]) == list(range(6))


def test_recall_grows_with_list_length_on_searchable_data(orc):
    """Sanity curve, not a parity pin: on a connected low-dimensional cloud
    recall@10 grows with L and reaches > 0.95."""
    base, queries = workloads.sift_like(N=6000, nq=60, seed=9)
    adj, lam = orc.build_graph(base, 16)
    gt, _ = orc.bruteforce(base, queries, 10)
    rec = [orc.recall(orc.search(adj, lam, base, queries, 10, L, 10)[0], gt) for L in (10, 40, 160)]
    assert rec[-1] > 0.95 and rec[0] < rec[-1]
