"""Pins for the oracle's search with the paper's own R / C / V structures (Alg. 2).  CPU only."""
import json
import os
from fractions import Fraction

import numpy as np

import workloads

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "alg2_segment_overflow.json")


def exact_stop_l2(s_u, s_f, delta):
    """sqrt(s_u) > sqrt(s_f) + delta decided in exact rational arithmetic (delta >= 0):
    s_u - s_f - delta^2 > 2 delta sqrt(s_f)  <=>  lhs > 0 and lhs^2 > 4 delta^2 s_f."""
    su, sf, dl = Fraction(float(s_u)), Fraction(float(s_f)), Fraction(float(delta))
    t = su - sf - dl * dl
    return t > 0 and t * t > 4 * dl * dl * sf


def overflow_case():
    """The hand-worked example of tests/golden/alg2_segment_overflow.json as arrays."""
    doc = json.load(open(GOLDEN))
    x = np.array(doc["x"], np.float32)
    N, K = len(x), 34                      # the longest row has 33 entries; an imported graph needs K < N
    base = np.zeros((N, 4), np.float32)
    base[:, 0] = x
    adj = np.full((N, K), -1, np.int32)
    lam = np.full((N, K), 255, np.uint8)
    for i in range(N):
        row = doc["rows"].get(str(i), doc["default_row"])
        adj[i, :len(row)] = row
        lam[i, :len(row)] = 0
    return doc, base, adj, lam, np.zeros((1, 4), np.float32)


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
        if exact_stop_l2(u[0], R[-1][0], delta):
            break
        V[u[1] % m_v][vpos[u[1] % m_v]] = u[1]
        vpos[u[1] % m_v] = (vpos[u[1] % m_v] + 1) % 32
        for p in range(adj.shape[1]):
            e = int(adj[u[1], p])
            if e < 0 or lam[u[1], p] >= lv:
                break
            if e in V[e % m_v] or any(i == e for _, i in C[e % m_c]):   # one neighbour at a time, as listed
                continue
            c = (s_of(e), e)
            evals += 1
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
    typical = float(np.sqrt(typical))                    # Delta is an L2 distance
    for k, m_c, m_v, delta, T in ((10, 4, 4, 0.0, 0), (20, 2, 1, 0.2 * typical, 0), (5, 1, 8, 3 * typical, 12)):
        ids, s, st = orc.search_alg2(adj, lam, base, queries, k, delta, m_c=m_c, m_v=m_v, max_hops=T,
                                     lambda_visit=10, seed=3, want_stats=True)
        for qi in range(10):
            seeds = [orc.seed_id(3, qi, t, 1500) for t in range(32)]
            R, hops, evals = py_alg2(adj, lam, base, queries[qi], k, m_c, m_v, delta, T, 10, seeds)
            R = R + [(np.inf, -1)] * (k - len(R))
            assert [i for _, i in R] == list(ids[qi])
            assert np.array_equal(np.array([v for v, _ in R], np.float32), s[qi])
            assert (hops, evals) == (st[qi][0], st[qi][1])


def test_hand_worked_segment_overflow(orc):
    """A push into the full segment of C drops a later neighbour of the same hop: in the
    listing's order that neighbour is scored once more (and pushed nowhere).  Expected counters
    and rankings are the hand-derived ones of the golden file."""
    doc, base, adj, lam, q = overflow_case()
    prm = doc["params"]
    seed = next(sd for sd in range(300) if 0 in [orc.seed_id(sd, 0, t, len(base)) for t in range(32)])
    for T in (1, 2, 3):
        want = doc["expected"][f"T={T}"]
        ids, s, st = orc.search_alg2(adj, lam, base, q, prm["k"], prm["delta"], m_c=prm["m_c"], m_v=prm["m_v"],
                                     max_hops=T, lambda_visit=prm["lambda_visit"], seed=seed, want_stats=True)
        assert [int(v) for v in st[0]] == [want["hops"], want["dist_evals"], want["skips"]], f"T={T}"
        n = len(want["ids"])
        assert list(ids[0][:n]) == want["ids"] and np.all(ids[0][n:] == -1)
        assert np.array_equal(s[0][:n], base[want["ids"], 0] ** 2)
    # what look-ups made before the hop's pushes would report: same ranking, one count moved
    other = doc["batched_lookups_would_give"]["T=2"]
    assert other["ids"] == doc["expected"]["T=2"]["ids"]
    assert (other["dist_evals"], other["skips"]) == (doc["expected"]["T=2"]["dist_evals"] - 1, 1)


def test_stop_rule_is_on_the_distance_itself(orc):
    """Alg. 2 compares m(u,q) > m(f,q) + Delta with m the L2 distance.  The oracle's square-root-free
    fp64 form against the same inequality in exact rational arithmetic, and closed cases."""
    assert not orc.alg2_stop(12.25, 9.0, 0.5)                      # 3.5 > 3 + 0.5 is false (equality)
    assert orc.alg2_stop(np.nextafter(np.float32(12.25), np.float32(20)), 9.0, 0.5)
    assert not orc.alg2_stop(16.0, 9.0, 1.0) and orc.alg2_stop(16.5, 9.0, 1.0)
    assert orc.alg2_stop(9.5, 9.0, 0.0) and not orc.alg2_stop(9.0, 9.0, 0.0)   # Delta = 0: plain comparison
    assert not orc.alg2_stop(1e30, 1.0, 3.0e38)
    # a test on squared distances with the same Delta would already stop at s_u = 12 (12 > 9 + 1);
    # on the distance itself sqrt(12) = 3.46 is not beyond 3 + 1
    assert not orc.alg2_stop(12.0, 9.0, 1.0)
    g = np.random.default_rng(5)
    n_stop = 0
    for _ in range(4000):
        s_f = np.float32(g.uniform(0.0, 100.0))
        delta = np.float32(g.choice([0.0, g.uniform(0, 3.0)]))
        s_u = np.float32((np.sqrt(float(s_f)) + float(delta)) ** 2 * g.choice([1.0, g.uniform(0.9, 1.1), 1 + 1e-6, 1 - 1e-6]))
        want = exact_stop_l2(s_u, s_f, delta)
        t = Fraction(float(s_u)) - Fraction(float(s_f)) - Fraction(float(delta)) ** 2
        knife = abs(t * t - 4 * Fraction(float(delta)) ** 2 * Fraction(float(s_f))) <= Fraction(1, 10 ** 9) * max(t * t, Fraction(1, 10 ** 30))
        if not knife:
            assert orc.alg2_stop(s_u, s_f, delta) == want
        n_stop += want
    assert 500 < n_stop < 3500
    # 1 - cos on unit rows: m = s/2
    assert orc.alg2_stop(1.01, 0.5, 0.25, "cosine") and not orc.alg2_stop(1.0, 0.5, 0.25, "cosine")


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
    typical = float(np.sqrt(np.median(orc.bruteforce(base, queries, 10)[1][:, 9])))
    prev = None
    for delta in (0.0, 0.1 * typical, 0.5 * typical, 2 * typical):
        ids, s, st = orc.search_alg2(adj, lam, base, queries, 10, delta, want_stats=True)
        if prev is not None:
            assert np.all(st[:, 0] >= prev)              # a larger Delta never stops earlier
        prev = st[:, 0].copy()
        for r in range(30):
            assert len(set(ids[r])) == 10 and list(zip(s[r], ids[r])) == sorted(zip(s[r], ids[r]))
            assert np.array_equal(np_canonical(base[ids[r]], queries[r]), s[r])
    _, _, st = orc.search_alg2(adj, lam, base, queries, 10, 2 * typical, max_hops=4, want_stats=True)
    assert np.all(st[:, 0] <= 4)
    gt = orc.bruteforce(base, queries, 10)[0]
    assert orc.recall(orc.search_alg2(adj, lam, base, queries, 32, 0.5 * typical)[0][:, :10].copy(), gt) > 0.9
