"""Pins for the oracle's small-batch multi-search (Alg. 1).  CPU only."""
import numpy as np

import workloads


def np_canonical(base, q):
    t = (base.astype(np.float32) - q.astype(np.float32)[None, :]).astype(np.float32)
    return np.sum(t.astype(np.float64) ** 2, axis=1).astype(np.float32)


def py_greedy(adj, lam, base, q, lv, seeds, T):
    """The greedy search of Alg. 1 written independently with Python sets and sorted()."""
    sc = lambda ids: sorted(zip(np_canonical(base[list(ids)], q).tolist(), list(ids)))
    u = sc(seeds)[0][1]
    R, hops, improved = [], 0, True
    while improved and hops < T:
        row = []
        for p in range(adj.shape[1]):
            if adj[u, p] < 0 or lam[u, p] >= lv:
                break
            row.append(int(adj[u, p]))
        hops += 1
        if not row:
            break
        scored = dict((i, s) for s, i in sc(row))
        slots = {}
        for p, v in enumerate(row):
            c = (scored[v], v)
            if p % 32 not in slots or c < slots[p % 32]:
                slots[p % 32] = c
        cand = sorted(slots.values())
        kept = R[:16]
        kept_ids = {i for _, i in kept}
        new = sorted(kept + [c for c in cand[:16] if c[1] not in kept_ids])[:32]
        improved = any(i not in kept_ids for _, i in new[:16])
        R, u = new, cand[0][1]
    return R


def test_matches_independent_python_version(orc):
    base, queries = workloads.single_gaussian(1500, 8, seed=41, nq=12)
    adj, lam = orc.build_graph(base, 16)
    for t0, T in ((1, 16), (3, 4), (5, 1)):
        ids, s = orc.search_multi(adj, lam, base, queries, 10, t0, max_hops=T, lambda_visit=10, seed=9)
        for qi in range(12):
            pool = {}
            for j in range(t0):
                seeds = [orc.seed_id(9, qi, 32 * j + t, 1500) for t in range(32)]
                for sc, i in py_greedy(adj, lam, base, queries[qi], 10, seeds, T):
                    pool[i] = sc
            want = sorted((sc, i) for i, sc in pool.items())[:10]
            want += [(np.inf, -1)] * (10 - len(want))
            assert [i for _, i in want] == list(ids[qi])
            assert np.array_equal(np.array([sc for sc, _ in want], np.float32), s[qi])


def test_complete_graph_is_exact_after_two_hops(orc):
    """17 nodes, everybody linked to everybody (K=16): hop 1 scores the 16 neighbours of the
    start node, hop 2 (from its best neighbour) scores the start node too; the kept half then
    holds the exact top-10."""
    N = 17
    base, queries = workloads.single_gaussian(N, 4, seed=42, nq=8)
    adj = np.array([[j for j in range(N) if j != i] for i in range(N)], np.int32)
    lam = np.zeros_like(adj, dtype=np.uint8)
    ids, s = orc.search_multi(adj, lam, base, queries, 10, 1, max_hops=4, lambda_visit=1)
    for qi in range(8):
        d = np_canonical(base, queries[qi])
        order = np.lexsort((np.arange(N), d))[:10]
        assert np.array_equal(ids[qi], order) and np.array_equal(s[qi], d[order])


def test_slot_rule_with_64_neighbours(orc):
    """A hub with 64 neighbours: position p and p+32 compete for one slot, so one hop keeps
    exactly the closer of each pair."""
    g = np.random.default_rng(43)
    N = 65
    base = np.zeros((N, 4), np.float32)
    base[1:, 0] = g.permutation(64) + 1.0            # neighbours at distinct distances from the origin
    adj = np.full((N, 64), -1, np.int32)
    lam = np.full((N, 64), 255, np.uint8)
    adj[0] = np.arange(1, 65)
    lam[0] = 0
    q = np.zeros((1, 4), np.float32)                 # the query sits on the hub
    # pick a seed value whose 32 start nodes include the hub; the hub (s = 0) is then the start
    seed = next(sd for sd in range(200) if 0 in [orc.seed_id(sd, 0, t, N) for t in range(32)])
    ids, s = orc.search_multi(adj, lam, base, q, 32, 1, max_hops=1, lambda_visit=1, seed=seed)
    d = np_canonical(base, q[0])
    want = sorted((min((d[p + 1], p + 1), (d[p + 33], p + 33))) for p in range(32))[:16]
    assert [i for _, i in want] == list(ids[0][:16])
    assert np.all(ids[0][16:] == -1)                 # only 16 of R_temp enter R


def test_more_searches_never_hurt_and_reach_high_recall(orc):
    base, queries = workloads.sift_like(N=5000, nq=60, seed=11)
    adj, lam = orc.build_graph(base, 16)
    gt, _ = orc.bruteforce(base, queries, 10)
    prev_s, rec = None, []
    for t0 in (1, 2, 4, 8, 16):
        ids, s, st = orc.search_multi(adj, lam, base, queries, 10, t0, want_stats=True)
        if prev_s is not None:
            assert np.all(s <= prev_s)               # search j does not depend on t0: the union only grows
        prev_s = s
        rec.append(orc.recall(ids, gt))
        for r in range(60):
            v = ids[r][ids[r] >= 0]
            assert len(set(v)) == len(v)
            assert list(zip(s[r][:len(v)], v)) == sorted(zip(s[r][:len(v)], v))
            assert np.array_equal(np_canonical(base[v], queries[r]), s[r][:len(v)])
        assert np.all(st[:, 0] <= 16 * t0)           # hop limit T = 16 per search
    assert rec[-1] > 0.9 and rec[0] < rec[-1]


def test_zero_hops_returns_nothing_and_limit_is_respected(orc):
    base, queries = workloads.single_gaussian(800, 8, seed=44, nq=5)
    adj, lam = orc.build_graph(base, 8)
    ids, s = orc.search_multi(adj, lam, base, queries, 5, 2, max_hops=0)
    assert np.all(ids == -1) and np.all(np.isinf(s))
    _, _, st = orc.search_multi(adj, lam, base, queries, 5, 3, max_hops=2, want_stats=True)
    assert np.all(st[:, 0] <= 6) and np.all(st[:, 1] >= 3 * 32)
