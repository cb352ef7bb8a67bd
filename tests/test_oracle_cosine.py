"""Pins for the oracle's cosine metric (Sec. 5, Table 1: m = Cos), CPU only.

Cosine is taken as m(a,b) = 1 - cos(a,b) on rows normalised once in fp32; with unit rows m = s/2,
so the L2 machinery serves, with Eq. 2's factor alpha applied to m (alpha on s, not alpha^2).
Pinned here by closed forms, by invariance under row scaling (which only a cosine can have), by a
brute-force ranking computed in fp64 from the RAW rows, and by Eq. 2 re-evaluated in fp64 on 1 - cos.
"""
import numpy as np
import pytest

import workloads


def cosdist64(a, b):
    a = a.astype(np.float64)
    b = b.astype(np.float64)
    return 1.0 - (a @ b.T) / (np.linalg.norm(a, axis=1)[:, None] * np.linalg.norm(b, axis=1)[None, :])


def test_normalised_rows_are_unit_and_ignore_power_of_two_scaling(orc):
    g = np.random.default_rng(1)
    x = g.standard_normal((200, 36)).astype(np.float32)
    u = orc.normalize_rows(x)
    assert np.abs(np.linalg.norm(u.astype(np.float64), axis=1) - 1.0).max() < 2e-7
    scale = (2.0 ** g.integers(-20, 20, size=(200, 1))).astype(np.float32)
    assert np.array_equal(orc.normalize_rows(x * scale), u)          # exact: scaling by 2^k changes no mantissa
    z = np.zeros((1, 36), np.float32)
    assert np.array_equal(orc.normalize_rows(z), z)                  # a zero row stays zero


def test_closed_forms(orc):
    e = np.eye(4, dtype=np.float32)
    rows = orc.normalize_rows(np.stack([e[0], e[1], 3 * e[0], -2 * e[0], e[0] + e[1]]))
    half = lambda i, j: float(orc.sqdist(rows[i], rows[j])) * 0.5
    assert half(0, 1) == 1.0        # orthogonal
    assert half(0, 2) == 0.0        # same direction, other length
    assert half(0, 3) == 2.0        # opposite
    assert abs(half(0, 4) - (1.0 - 2 ** -0.5)) < 1e-7   # 45 degrees


def test_search_with_list_longer_than_the_set_ranks_by_one_minus_cos(orc):
    base_raw, q_raw = workloads.glove_like(N=600, nq=40, d=20, components=1, seed=5)
    base, q = orc.normalize_rows(base_raw), orc.normalize_rows(q_raw)
    adj, lam = orc.build_graph(base, 12, metric="cosine")
    ids, m = orc.search(adj, lam, base, q, 10, 600, 10, n_seeds=600, metric="cosine")
    truth = cosdist64(q_raw, base_raw)                 # from the raw rows: no normalisation shared with the oracle
    for i in range(q.shape[0]):
        order = np.argsort(truth[i], kind="stable")[:10]
        assert np.allclose(m[i], truth[i][ids[i]], rtol=0, atol=3e-7)
        if not np.array_equal(ids[i], order):          # only near-ties may swap
            assert np.abs(truth[i][ids[i]] - truth[i][order]).max() < 3e-7
    assert orc.recall(ids, np.argsort(truth, axis=1)[:, :10].astype(np.int32)) > 0.999


def test_row_lengths_do_not_change_the_graph(orc):
    base_raw, _ = workloads.glove_like(N=500, nq=1, d=16, components=4, seed=6)
    g = np.random.default_rng(2)
    scaled = base_raw * (2.0 ** g.integers(-8, 8, size=(500, 1))).astype(np.float32)
    a1, l1 = orc.build_graph(orc.normalize_rows(base_raw), 10, metric="cosine")
    a2, l2 = orc.build_graph(orc.normalize_rows(scaled), 10, metric="cosine")
    assert np.array_equal(a1, a2) and np.array_equal(l1, l2)


@pytest.mark.parametrize("alpha", [1.0, 1.2, 1.5])
def test_stage1_is_eq2_on_one_minus_cos(orc, alpha):
    """Every dropped edge has a kept, earlier witness under alpha*m < m (m = 1 - cos in fp64 from
    the raw rows), and no kept edge has one; pairs within 1e-5 of equality are not judged."""
    base_raw, _ = workloads.glove_like(N=400, nq=1, d=12, components=3, seed=7)
    base = orc.normalize_rows(base_raw)
    K = 16
    knn_id, knn_s = orc.knn(base, K)
    g1_id, _, g1_deg = orc.stage1(base, knn_id, knn_s, alpha, metric="cosine")
    M = cosdist64(base_raw, base_raw)
    eps = 1e-5
    judged = 0
    for x0 in range(base.shape[0]):
        kept = list(g1_id[x0, :g1_deg[x0]])
        assert kept[0] == knn_id[x0, 0]
        seen_kept = []
        for j in knn_id[x0]:
            m0j = M[x0, j]
            sure = [i for i in seen_kept if alpha * M[x0, i] < m0j * (1 - eps) and alpha * M[i, j] < m0j * (1 - eps)]
            maybe = [i for i in seen_kept if alpha * M[x0, i] < m0j * (1 + eps) and alpha * M[i, j] < m0j * (1 + eps)]
            if j in kept:
                assert not sure, (x0, j)
                seen_kept.append(j)
            else:
                assert maybe, (x0, j)
            judged += 1
    assert judged == base.shape[0] * K
    if alpha > 1.0:   # the factor is alpha, not alpha^2: the L2 rule on the same unit rows keeps more
        l2_deg = orc.stage1(base, knn_id, knn_s, alpha, metric="l2")[2]
        assert l2_deg.sum() > g1_deg.sum()


def test_inner_product_by_its_reduction_to_l2(orc):
    """Table 1's m = IP: on the augmented rows the L2 order of the base rows of a query is the order of
    -<q,x> computed in fp64 from the raw rows, and the inner product is recovered from the distance."""
    base, q = workloads.glove_like(N=700, nq=30, d=20, components=1, seed=8)
    M = np.float32(np.sqrt((base.astype(np.float64) ** 2).sum(1).max()) * 1.0001)
    ab, aq = orc.ip_augment_rows(base, M), orc.ip_augment_rows(q, is_query=True)
    assert ab.shape == (700, 24) and np.array_equal(ab[:, :20], base) and (ab[:, 21:] == 0).all() and (aq[:, 20:] == 0).all()
    assert np.abs((ab.astype(np.float64) ** 2).sum(1) - float(M) ** 2).max() < 1e-4 * float(M) ** 2   # all on the sphere of radius M
    ids, s = orc.bruteforce(ab, aq, 10)
    ip = q.astype(np.float64) @ base.astype(np.float64).T
    scale = np.abs(ip).max()
    for i in range(q.shape[0]):
        order = np.argsort(-ip[i], kind="stable")[:10]
        got_ip = ((q[i].astype(np.float64) ** 2).sum() + float(M) ** 2 - s[i].astype(np.float64)) / 2
        assert np.abs(got_ip - ip[i][ids[i]]).max() < 2e-6 * (float(M) ** 2 + scale)
        if not np.array_equal(ids[i], order):
            assert np.abs(ip[i][ids[i]] - ip[i][order]).max() < 2e-6 * (float(M) ** 2 + scale)
    # a row as long as M gets no extra coordinate; a longer one is clamped, not NaN
    two = np.array([[3.0, 4.0, 0.0, 0.0], [6.0, 8.0, 0.0, 0.0]], np.float32)
    out = orc.ip_augment_rows(two, 5.0)
    assert out[0, 4] == 0.0 and out[1, 4] == 0.0 and not np.isnan(out).any()
