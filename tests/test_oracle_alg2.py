"""Pins for the oracle's search with the paper's own R / C / V structures (Alg. 2).  CPU only."""
import numpy as np

import workloads


def np_canonical(base, q):
    t = (base.astype(np.float32) - q.astype(np.float32)[None, :]).astype(np.float32)
    return np.sum(t.astype(np.float64) ** 2, axis=1).astype(np.float32)


def py_alg2(adj, lam, base, q, k, m_c, m_v, delta, T, lv, seeds):
    """Alg. 2 written independently: dicts of lists for the segments, sorted() for order."""
    s_of = lambda i: np_canonical(base[[i]], q)[0]
    u = min((s_of(i), i) for i in seeds)
    R, C = [u], {g: [] for g in range(m_c)}
    C[u[1] % m_c].append(u)
    V = {g: [None] * 32 for g in range(m_v)}
    vpos = {g: 0 for g in range(m_v)}
    hops, evals = 0, len(seeds)
    while True:
        if T and hops >= T:
            break
        heads = [C[g][0] for g in C if C[g]]
        if not heads:
            break
        u = min(heads)
        hops += 1
        C[u[1] % m_c].remove(u)
        if u[0] > np.float32(R[-1][0] + np.float32(delta)):
            break
        V[u[1] % m_v][vpos[u[1] % m_v]] = u[1]
        vpos[u[1] % m_v] = (vpos[u[1] % m_v] + 1) % 32
        fresh = []
        for p in range(adj.shape[1]):
            e = int(adj[u[1], p])
            if e < 0 or lam[u[1], p] >= lv:
                break
            if e in V[e % m_v] or any(i == e for _, i in C[e % m_c]):
                continue
            fresh.append((s_of(e), e))          # all look-ups of the hop precede its pushes
        evals += len(fresh)
        for c in fresh:
            e = c[1]
            if not (len(R) < k or c[0] < R[-1][0]):
                continue
            if any(i == e for _, i in R):
                continue
            R = sorted(R + [c])[:k]
            C[e % m_c] = sorted(C[e % m_c] + [c])[:32]
    return R, hops, evals


def test_matches_independent_python_version(orc):
    base, queries = workloads.single_gaussian(1500, 8, seed=51, nq=10)
    adj, lam = orc.build_graph(base, 16)
    typical = float(np.median(orc.bruteforce(base, queries, 10)[1][:, 9]))
    for k, m_c, m_v, delta, T in ((10, 4, 4, 0.0, 0), (20, 2, 1, 0.5 * typical, 0), (5, 1, 8, 10 * typical, 12)):
        ids, s, st = orc.search_alg2(adj, lam, base, queries, k, delta, m_c=m_c, m_v=m_v, max_hops=T,
                                     lambda_visit=10, seed=3, want_stats=True)
        for qi in range(10):
            seeds = [orc.seed_id(3, qi, t, 1500) for t in range(32)]
            R, hops, evals = py_alg2(adj, lam, base, queries[qi], k, m_c, m_v, delta, T, 10, seeds)
            R = R + [(np.inf, -1)] * (k - len(R))
            assert [i for _, i in R] == list(ids[qi])
            assert np.array_equal(np.array([v for v, _ in R], np.float32), s[qi])
            assert (hops, evals) == (st[qi][0], st[qi][1])


def test_everything_expanded_is_exact(orc):
    """k >= N, no segment ever full, Delta = +inf on a connected graph: every node is pushed and
    expanded, so R is the whole set in (s,id) order."""
    base, queries = workloads.single_gaussian(300, 6, seed=52, nq=6)
    adj, lam = orc.build_graph(base, 12)
    ids, s = orc.search_alg2(adj, lam, base, queries, 300, 3.0e38, m_c=64, m_v=64, lambda_visit=10)
    for qi in range(6):
        d = np_canonical(base, queries[qi])
        order = np.lexsort((np.arange(300), d))
        assert np.array_equal(ids[qi], order) and np.array_equal(s[qi], d[order])


def star(n_leaves):
    """Hub 0 linked to leaves 1..n (distinct distances from the hub); a leaf links back to the hub."""
    g = np.random.default_rng(53)
    N = n_leaves + 1
    base = np.zeros((N, 4), np.float32)
    base[1:, 0] = g.permutation(n_leaves) + 1.0
    adj = np.full((N, 64), -1, np.int32)
    lam = np.full((N, 64), 255, np.uint8)
    adj[0, :n_leaves] = np.arange(1, N)
    lam[0, :n_leaves] = 0
    adj[1:, 0] = 0
    lam[1:, 0] = 0
    return base, adj, lam


def test_queue_segment_drops_its_most_distant_entry(orc):
    """40 leaves pushed by one expansion.  One segment (m_c = 1) keeps the 32 nearest, so 1 + 32
    nodes get expanded; with two segments (20 entries each) all 41 do.  R (k = 64) holds all."""
    base, adj, lam = star(40)
    q = np.zeros((1, 4), np.float32)
    seed = next(sd for sd in range(300) if 0 in [orc.seed_id(sd, 0, t, 41) for t in range(32)])
    for m_c, hops in ((1, 33), (2, 41)):
        ids, s, st = orc.search_alg2(adj, lam, base, q, 64, 3.0e38, m_c=m_c, m_v=8, lambda_visit=1, seed=seed,
                                     want_stats=True)
        assert st[0][0] == hops
        assert sorted(ids[0][:41]) == list(range(41)) and np.all(ids[0][41:] == -1)
        assert st[0][1] == 32 + 40                       # leaves scored once; the hub is found in V afterwards


def test_delta_and_hop_limit(orc):
    base, queries = workloads.single_gaussian(2000, 8, seed=54, nq=30)
    adj, lam = orc.build_graph(base, 16)
    typical = float(np.median(orc.bruteforce(base, queries, 10)[1][:, 9]))
    prev = None
    for delta in (0.0, 0.2 * typical, typical, 5 * typical):
        ids, s, st = orc.search_alg2(adj, lam, base, queries, 10, delta, want_stats=True)
        if prev is not None:
            assert np.all(st[:, 0] >= prev)              # a larger Delta never stops earlier
        prev = st[:, 0].copy()
        for r in range(30):
            assert len(set(ids[r])) == 10 and list(zip(s[r], ids[r])) == sorted(zip(s[r], ids[r]))
            assert np.array_equal(np_canonical(base[ids[r]], queries[r]), s[r])
    _, _, st = orc.search_alg2(adj, lam, base, queries, 10, 5 * typical, max_hops=4, want_stats=True)
    assert np.all(st[:, 0] <= 4)
    gt = orc.bruteforce(base, queries, 10)[0]
    assert orc.recall(orc.search_alg2(adj, lam, base, queries, 32, typical)[0][:, :10].copy(), gt) > 0.9
