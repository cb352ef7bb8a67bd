"""Pins for the oracle's approximate k-NN builder (neighbourhood propagation in pull form), CPU only.

It is a heuristic, so what pins it: an independent re-statement of the same rules with Python sets
on a small input (ids must agree exactly), the invariants every iteration must keep, the exact k-NN
graph as a fixed point, and convergence towards the brute-force lists on a connected cloud."""
import json
import os

import numpy as np
import pytest

import workloads

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "knn_descent_line8.json")


def line8_case(which):
    """A hand-worked case of tests/golden/knn_descent_line8.json: rows of d = 4 (x, 0, 0, 0)."""
    doc = json.load(open(GOLDEN))
    base = np.zeros((len(doc["x"]), 4), np.float32)
    base[:, 0] = doc["x"]
    case = doc["cases"][which]
    return doc, case, base, np.array(case["init_ids"], np.int32)


@pytest.mark.parametrize("which", ["A", "B"])
def test_hand_worked_example(orc, which):
    """Eight points on a line, K = 3, S = 2: the lists after one and two iterations and the number of
    changed entries equal the values derived by hand in the golden file (its derivations walk through
    the sample cap, the slot of every reverse offer, the smallest-key rule, the new/old flags and the
    'old edge offers only its new part' rule; a mistake in any of them changes one of these lists)."""
    doc, case, base, init = line8_case(which)
    for it in (1, 2):
        want = case[f"after_iteration_{it}"]
        ids, s, done, changed = orc.knn_descent(base, doc["K"], S=doc["S"], max_iters=it, delta=0.0, init_ids=init)
        assert done == it and ids.tolist() == want["ids"] and int(changed[-1]) == want["changed"]
        x = np.array(doc["x"], np.float64)
        assert np.array_equal(s, ((x[:, None] - x[ids]) ** 2).astype(np.float32))


def test_reverse_table_slot(orc):
    """The cell a source takes in a reverse table, against products reduced by hand (golden file)."""
    doc = json.load(open(GOLDEN))
    assert [orc.descent_slot(u, 2) for u in range(8)] == doc["slot"]
    for c in doc["slot_examples_S16"]["cases"]:
        assert c["product"] - c["minus_multiples_of_2^32"] * 2 ** 32 == c["remainder"] < 2 ** 32
        assert orc.descent_slot(c["u"], 16) == c["slot"] == c["remainder"] >> 28
    assert len({c["slot"] for c in doc["slot_examples_S16"]["cases"]}) >= 5


def python_descent(orc, base, K, S, iters, seed):
    """The same rules written with dicts and sorts, sharing only the distance and the seed generator."""
    N = base.shape[0]
    log2s = S.bit_length() - 1
    dist = lambda a, b: float(orc.sqdist(base[a], base[b]))
    lists = []
    for v in range(N):
        picked = []
        for j in range(2 * K):
            c = orc.seed_id(seed, v, j, N)
            if c != v and c not in picked and len(picked) < K:
                picked.append(c)
        lists.append(sorted((dist(v, c), c, True) for c in picked))
    for _ in range(iters):
        newF = [[e[1] for e in l if e[2]][:S] for l in lists]
        oldF = [[e[1] for e in l if not e[2]][:S] for l in lists]
        sof = [{e[1]: e[0] for e in l} for l in lists]
        Rnew = [dict() for _ in range(N)]
        Rold = [dict() for _ in range(N)]
        for u in range(N):
            slot = ((u * 2654435761) & 0xFFFFFFFF) >> (32 - log2s)
            for tab, F in ((Rnew, newF), (Rold, oldF)):
                for w in F[u]:
                    key = (sof[u][w], u)
                    if slot not in tab[w] or key < tab[w][slot]:
                        tab[w][slot] = key
        rn = [[tab[t][1] for t in sorted(tab)] for tab in Rnew]
        ro = [[tab[t][1] for t in sorted(tab)] for tab in Rold]
        nxt = []
        for a in range(N):
            cur = {e[1]: (e[0], e[2] and e[1] not in newF[a]) for e in lists[a]}
            pool = dict(cur)
            for v, edge_new in [(v, True) for v in newF[a]] + [(v, False) for v in oldF[a]] + \
                               [(v, True) for v in rn[a]] + [(v, False) for v in ro[a]]:
                cands = newF[v] + rn[v] + ((oldF[v] + ro[v]) if edge_new else [])
                for b in cands:
                    if b != a and b not in pool:
                        pool[b] = (dist(a, b), True)
            best = sorted((s, b, fl) for b, (s, fl) in pool.items())[:K]
            nxt.append(best)
        lists = nxt
    ids = np.array([[e[1] for e in l] + [-1] * (K - len(l)) for l in lists], np.int32)
    return ids


@pytest.mark.parametrize("K,S,iters", [(4, 2, 3), (6, 4, 2)])
def test_agrees_with_a_restatement_in_python(orc, K, S, iters):
    base = workloads.single_gaussian(90, 5, seed=21)
    want = python_descent(orc, base, K, S, iters, seed=9)
    ids, s, done, changed = orc.knn_descent(base, K, S=S, max_iters=iters, delta=0.0, seed=9)
    assert done == iters
    assert np.array_equal(ids, want)


def test_invariants_every_iteration(orc):
    base = workloads.single_gaussian(1200, 8, seed=22)
    K = 12
    prev_kth = None
    for iters in range(0, 5):
        ids, s, done, changed = orc.knn_descent(base, K, S=8, max_iters=iters, delta=0.0, seed=1)
        assert done == iters and len(changed) == iters
        assert (ids >= 0).all() and (ids != np.arange(1200)[:, None]).all()
        assert all(len(set(r)) == K for r in ids)                             # distinct
        keys = s.astype(np.float64) * 2 ** 32 + ids                            # (s,id) order
        assert (np.diff(keys, axis=1) > 0).all()
        for v in range(0, 1200, 97):                                          # distances are the canonical ones
            for t in range(K):
                assert s[v, t] == orc.sqdist(base[v], base[ids[v, t]])
        if prev_kth is not None:
            assert (s[:, -1] <= prev_kth).all()                               # lists only improve
        prev_kth = s[:, -1].copy()


def test_exact_graph_is_a_fixed_point_and_the_cloud_converges(orc):
    base = workloads.single_gaussian(3000, 8, seed=23)
    K = 16
    exact_ids, exact_s = orc.knn(base, K)
    ids, s, done, changed = orc.knn_descent(base, K, S=8, max_iters=2, delta=0.0, init_ids=exact_ids)
    assert np.array_equal(ids, exact_ids) and np.array_equal(s, exact_s)
    assert done == 1 and list(changed) == [0]            # nothing to improve: it stops at once
    ids, s, done, changed = orc.knn_descent(base, K, S=8, max_iters=15, delta=0.001, seed=3)
    rec = np.mean([len(set(a) & set(b)) for a, b in zip(ids, exact_ids)]) / K
    assert rec > 0.9, rec
    assert done < 15 and changed[-1] <= 0.001 * 3000 * K and changed[0] > changed[-1]
