"""Pins for the oracle's graph build: stage 1 (relaxed occlusion, Eq. 2),
reverse edges, stage 2 (occlusion factor, Sec. 3.3).  CPU only."""
import json
import os

import numpy as np

import workloads

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def np_s(a, b):
    t = (a.astype(np.float32) - b.astype(np.float32)).astype(np.float32)
    return np.float32(np.sum(t.astype(np.float64) ** 2))


def pad4(pts):
    pts = np.asarray(pts, np.float32)
    out = np.zeros((pts.shape[0], 4), np.float32)
    out[:, :pts.shape[1]] = pts
    return out


def golden():
    g = json.load(open(os.path.join(GOLD, "occlusion_2d.json")))
    return g, pad4(g["points"])


# ---------------------------------------------------------------- hand example
def test_golden_distances(orc):
    """s(x0,.) of the hand example: x1 1; x2 1.44+.09; x3 1.21+.1225; x4 4+2.25;
    x5 5.29+2.89; x6 4; x7 .09+9."""
    g, pts = golden()
    for j, want in g["sq_dist_from_node"].items():
        assert abs(float(orc.sqdist(pts[0], pts[int(j)])) - want) < 1e-5


def test_golden_stage1(orc):
    """Order by s: x1(1) x3(1.3325) x2(1.53) x6(4) x4(6.25) x5(8.18) x7(9.09).
    alpha=1.2 (alpha^2=1.44): x3 kept (1.44 !< 1.3325); x2 dropped by x1
    (1.44<1.53, 1.44*.13<1.53); x6 kept (s(x1,x6)=9); x4 dropped by x1
    (1.44*3.25=4.68<6.25); x5 dropped by x1 (1.44*4.58=6.6<8.18); x7 kept
    (s(x1,x7)=9.49, s(x3,x7)=7.6625 -> 11.03, s(x6,x7)=14.29).
    alpha=1: x3 is dropped too (1<1.3325 and .1325<1.3325)."""
    g, pts = golden()
    kid, ks = orc.knn(pts, 7)
    assert list(kid[0]) == [1, 3, 2, 6, 4, 5, 7]
    for alpha, key in ((1.2, "stage1_kept_alpha_1.2"), (1.0, "stage1_kept_alpha_1.0")):
        g1_id, g1_s, g1_deg = orc.stage1(pts, kid, ks, alpha)
        want = g[key]
        assert g1_deg[0] == len(want)
        assert list(g1_id[0][:len(want)]) == want
        assert np.all(g1_id[0][len(want):] == -1)


def test_golden_stage2_lambda(orc):
    """lambda by Eq. 1 over the whole list of x0 (pairwise squared distances:
    s12 .13, s13 .1325, s23 .4325, s14 3.25, s24 2.08, s34 4.2325, s15 4.58,
    s25 3.17, s35 5.6425, s45 .13, s16 9, s37 7.6625, s17 9.49, s67 14.29):
    x1 0; x3 1 (x1); x2 2 (x1,x3); x4 3 (x1,x2,x3); x5 4; x6 0; x7 1 (x3)."""
    g, pts = golden()
    kid, ks = orc.knn(pts, 7)
    deg = np.full((8,), 7, np.int32)
    adj, lam = orc.stage2(pts, kid, ks, deg, lambda0=99, K=7)
    assert list(adj[0]) == g["order_by_lambda_then_distance"]
    assert [int(v) for v in lam[0]] == [g["lambda"][str(i)] for i in adj[0]]
    adj1, lam1 = orc.stage2(pts, kid, ks, deg, lambda0=1, K=7)
    assert list(adj1[0][:4]) == g["kept_with_lambda0_1"]
    assert np.all(adj1[0][4:] == -1) and np.all(lam1[0][4:] == 255)
    # degree cap K after the (lambda, s, id) sort
    adj2, lam2 = orc.stage2(pts, kid, ks, deg, lambda0=99, K=3)
    assert list(adj2[0]) == g["order_by_lambda_then_distance"][:3]


# ------------------------------------------------------------------ closed forms
def test_stage1_collinear_and_equilateral(orc):
    # 0,1,2 on a line: from node 0 the far edge (to 2) is occluded by the near one.
    line = pad4([[0, 0], [1, 0], [2, 0], [50, 50], [51, 50]])
    kid, ks = orc.knn(line, 2)
    g1_id, _, g1_deg = orc.stage1(line, kid, ks, 1.0)
    assert list(kid[0]) == [1, 2] and g1_deg[0] == 1 and g1_id[0][0] == 1
    # relaxed: alpha^2 * s(x1,x2) = 4 * 1 is not < s(x0,x2) = 4  -> kept at alpha = 2
    g1_id, _, g1_deg = orc.stage1(line, kid, ks, 2.0)
    assert g1_deg[0] == 2
    # equilateral triangle: all three distances equal, strict '<' drops nothing
    h = np.float32(np.sqrt(3.0) / 2)
    tri = pad4([[0, 0], [1, 0], [0.5, h], [40, 40]])
    kid, ks = orc.knn(tri, 2)
    if ks[0][0] == ks[0][1]:
        _, _, g1_deg = orc.stage1(tri, kid, ks, 1.0)
        assert g1_deg[0] == 2
    # exact integer isosceles version with equal squared sides: (0,0),(4,0),(0,4): s=16,16, s12=32
    iso = pad4([[0, 0], [4, 0], [0, 4], [90, 90]])
    kid, ks = orc.knn(iso, 2)
    _, _, g1_deg = orc.stage1(iso, kid, ks, 1.0)
    assert g1_deg[0] == 2


# -------------------------------------------------------------------- invariants
def _angles_ok(base, x0, kept):
    v = base[kept].astype(np.float64) - base[x0].astype(np.float64)
    v /= np.linalg.norm(v, axis=1, keepdims=True)
    c = v @ v.T
    iu = np.triu_indices(len(kept), 1)
    return np.all(c[iu] <= 0.5 + 1e-6)


def test_stage1_alpha1_keeps_edges_at_least_60_degrees_apart(orc):
    """Sec. 3.1: in l2 the rule guarantees >= 60 degrees between kept edges."""
    base = workloads.single_gaussian(600, 6, seed=11)
    kid, ks = orc.knn(base, 24)
    g1_id, g1_s, g1_deg = orc.stage1(base, kid, ks, 1.0)
    assert np.array_equal(g1_id[:, 0], kid[:, 0])            # closest always kept
    multi = 0
    for x0 in range(600):
        kept = g1_id[x0][:g1_deg[x0]]
        multi += len(kept) > 1
        assert _angles_ok(base, x0, kept)
    assert multi > 300


def test_stage1_rule_holds_for_every_edge(orc):
    """Any alpha: no kept pair satisfies Eq. 2 (later vs earlier), and every
    dropped edge has a kept, earlier witness that does."""
    base = workloads.single_gaussian(500, 5, seed=12)
    kid, ks = orc.knn(base, 20)
    for alpha in (1.0, 1.2, 1.5):
        a2 = np.float32(np.float32(alpha) * np.float32(alpha))
        g1_id, g1_s, g1_deg = orc.stage1(base, kid, ks, alpha)
        dropped_total = 0
        for x0 in range(0, 500, 3):
            kept = list(g1_id[x0][:g1_deg[x0]])
            kept_so_far = []
            for j in range(20):
                e, s0j = kid[x0][j], ks[x0][j]
                wit = any(a2 * ks[x0][list(kid[x0]).index(i)] < s0j and
                          a2 * np_s(base[i], base[e]) < s0j for i in kept_so_far)
                assert (e in kept) == (not wit)
                if e in kept:
                    kept_so_far.append(e)
                else:
                    dropped_total += 1
            assert kept_so_far == kept
            assert np.array_equal(g1_s[x0][:len(kept)], [ks[x0][list(kid[x0]).index(i)] for i in kept])
        assert dropped_total > 0


def test_reverse_edges_symmetric_and_counted(orc):
    base = workloads.single_gaussian(400, 6, seed=13)
    K = 10
    kid, ks = orc.knn(base, K)
    g1_id, g1_s, g1_deg = orc.stage1(base, kid, ks, 1.2)
    big = 400                                              # cap that never bites
    g2_id, g2_s, g2_deg = orc.reverse(base, g1_id, g1_deg, big)
    E = set()
    for x in range(400):
        for t in range(g1_deg[x]):
            E.add((x, int(g1_id[x][t])))
    und = E | {(b, a) for (a, b) in E}
    got = {(x, int(g2_id[x][t])) for x in range(400) for t in range(g2_deg[x])}
    assert got == und                                      # symmetric closure, no duplicates
    assert sum(g2_deg) == len(und)
    indeg = np.zeros(400, int)
    for (_, b) in E:
        indeg[b] += 1
    assert indeg.sum() == g1_deg.sum()                     # in-degree sum = out-degree sum
    for x in range(400):
        m = g2_deg[x]
        assert len(set(g2_id[x][:m])) == m
        keys = list(zip(g2_s[x][:m], g2_id[x][:m]))
        assert keys == sorted(keys)                        # (s, id) order
        for t in range(m):
            assert g2_s[x][t].tobytes() == np_s(base[x], base[g2_id[x][t]]).tobytes()
    # the cap keeps the (s,id)-smallest prefix
    c_id, c_s, c_deg = orc.reverse(base, g1_id, g1_deg, 2 * K)
    for x in range(400):
        m = min(g2_deg[x], 2 * K)
        assert c_deg[x] == m and np.array_equal(c_id[x][:m], g2_id[x][:m])
        assert np.all(c_id[x][m:] == -1)


def test_stage2_invariants(orc):
    base = workloads.single_gaussian(500, 6, seed=14)
    K = 12
    kid, ks = orc.knn(base, K)
    g1_id, g1_s, g1_deg = orc.stage1(base, kid, ks, 1.2)
    g2_id, g2_s, g2_deg = orc.reverse(base, g1_id, g1_deg, 2 * K)
    adj, lam = orc.stage2(base, g2_id, g2_s, g2_deg, lambda0=2 * K, K=2 * K)   # nothing dropped
    # GD (alpha = 1, sequential rule) applied to the same lists
    gd_id, _, gd_deg = orc.stage1(base, g2_id, g2_s, 1.0)
    for x in range(500):
        m = g2_deg[x]
        ids = list(adj[x][:m])
        assert sorted(ids) == sorted(g2_id[x][:m])                 # same edge set
        assert np.all(adj[x][m:] == -1) and np.all(lam[x][m:] == 255)
        lams = [int(v) for v in lam[x][:m]]
        rank = {int(e): r for r, e in enumerate(g2_id[x][:m])}     # rank by (s,id)
        s_of = {int(e): g2_s[x][r] for r, e in enumerate(g2_id[x][:m])}
        assert lam[x][ids.index(g2_id[x][0])] == 0                 # closest edge: lambda 0
        for e, l in zip(ids, lams):
            assert l <= rank[e]                                    # only closer edges can occlude
        keys = [(l, s_of[e], e) for e, l in zip(ids, lams)]
        assert keys == sorted(keys)                                # (lambda, s, id) order
        zero = {e for e, l in zip(ids, lams) if l == 0}
        assert zero <= set(gd_id[x][:gd_deg[x]])                   # lambda 0 => kept by GD
    # independent recount of lambda on a few nodes (Eq. 1, strict)
    for x in (0, 17, 333):
        m = g2_deg[x]
        for e, l in zip(adj[x][:m], lam[x][:m]):
            s0j = np_s(base[x], base[e])
            cnt = sum(1 for i in g2_id[x][:m] if i != e and np_s(base[x], base[i]) < s0j
                      and np_s(base[i], base[e]) < s0j)
            assert cnt == l


def test_build_degree_cap_and_threshold(orc):
    """Final lists hold at most K edges, all with lambda <= lambda0."""
    base = workloads.single_gaussian(600, 4, seed=15)
    for K, lam0 in ((8, 3), (16, 9)):
        adj, lam, st = orc.build_graph(base, K, alpha=1.2, lambda0=lam0, stages=True)
        assert adj.shape == (600, K)
        valid = adj >= 0
        assert np.all(lam[valid] <= lam0) and np.all(lam[~valid] == 255)
        assert np.all(valid[:, 0])                                  # closest edge survives
        # rows are prefixes: no valid entry after a pad
        assert np.all(valid[:, :-1] >= valid[:, 1:])
        # chain equals the stage-by-stage calls
        kid, ks = orc.knn(base, K)
        assert np.array_equal(st["knn_id"], kid)
        g1 = orc.stage1(base, kid, ks, 1.2)
        assert np.array_equal(st["g1_id"], g1[0])
        g2 = orc.reverse(base, g1[0], g1[2], 2 * K)
        assert np.array_equal(st["g2_id"], g2[0])
        a2, l2 = orc.stage2(base, g2[0], g2[1], g2[2], lam0, K)
        assert np.array_equal(a2, adj) and np.array_equal(l2, lam)


def test_duplicate_points_never_occlude_or_get_occluded(orc):
    """An exact duplicate of x0 has s = 0: nothing is < 0, and for i the
    duplicate s(xi,xj) = s(x0,xj), so the strict rule never fires through it."""
    pts = pad4([[0, 0], [0, 0], [1, 0], [0, 1], [7, 7]])
    kid, ks = orc.knn(pts, 3)
    assert kid[0][0] == 1 and ks[0][0] == 0
    g1_id, _, g1_deg = orc.stage1(pts, kid, ks, 1.0)
    assert list(g1_id[0][:g1_deg[0]]) == [1, 2, 3]
    deg = np.full((5,), 3, np.int32)
    adj, lam = orc.stage2(pts, kid, ks, deg, 9, 3)
    assert [int(v) for v in lam[0]] == [0, 0, 0]


def test_equal_length_edges_do_not_occlude_each_other(orc):
    """Eq. 1 / Eq. 2 need s(x0,xi) < s(x0,xj) strictly: two edges of equal
    length (17, 17) whose far ends are close (s = 4) keep lambda 0 and both
    survive stage 1, in id order."""
    pts = pad4([[0, 0], [4, 1], [4, -1], [60, 60], [61, 60]])
    kid, ks = orc.knn(pts, 2)
    assert list(kid[0]) == [1, 2] and list(ks[0]) == [17, 17]
    g1_id, _, g1_deg = orc.stage1(pts, kid, ks, 1.0)
    assert g1_deg[0] == 2
    deg = np.full((5,), 2, np.int32)
    adj, lam = orc.stage2(pts, kid, ks, deg, 9, 2)
    assert list(adj[0]) == [1, 2] and [int(v) for v in lam[0]] == [0, 0]
