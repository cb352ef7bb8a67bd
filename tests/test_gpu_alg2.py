"""Parity of the HIP search with the paper's own R / C / V structures (Alg. 2) with the CPU oracle."""
import numpy as np
import pytest
import torch

import workloads
from conftest import cached, sift_case, step, tiny_case
from parity import assert_bitwise, compare_topk

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run_both(gpu, orc, case, k, delta, **kw):
    base, queries, adj, lam = case[:4]
    g = gpu.ann_graph_import(dev(adj), dev(lam), base.shape[1])
    okw = dict(m_c=kw.get("m_c", 16), m_v=kw.get("m_v", 16), max_hops=kw.get("max_hops", 0),
               lambda_visit=kw.get("lambda_visit", 0) or 5, seed=kw.get("seed", 0), qi_offset=kw.get("qi_offset", 0))
    ref = orc.search_alg2(adj, lam, base, queries, k, delta, want_stats=True, **okw)
    ids, s, st = gpu.ann_search_alg2(g, dev(base), dev(queries), k, delta, want_stats=True, **kw)
    torch.cuda.synchronize()
    return (ids.cpu().numpy(), s.cpu().numpy(), st), ref


def check(got, ref, what, exact=True):
    ids, s, st = got
    if exact:
        assert_bitwise(ids, ref[0], what + " ids")
        assert_bitwise(s, ref[1], what + " dists")
    else:
        assert compare_topk(ids, s, ref[0], ref[1], what) == 0
    assert np.array_equal(st.hops.cpu().numpy(), ref[2][:, 0]), what + " hops"
    assert np.array_equal(st.dist_evals.cpu().numpy(), ref[2][:, 1]), what + " evals"
    assert np.array_equal(st.dedup_hits.cpu().numpy(), ref[2][:, 2]), what + " skips"


@pytest.mark.parametrize("k,frac,kw", [(10, 0.0, {}), (32, 0.1, {}), (64, 0.4, dict(m_c=4, m_v=2)),
                                       (1, 0.0, dict(m_c=1, m_v=1)), (20, 2.0, dict(max_hops=7, seed=9)),
                                       (16, 0.2, dict(m_c=64, m_v=64, lambda_visit=10, qi_offset=123)),
                                       (64, 0.3, dict(m_c=1, m_v=1, lambda_visit=32))])
def test_integer_data_matches_oracle_exactly(gpu, orc, k, frac, kw):
    step(f"alg2 sift20k k={k} delta={frac}x {kw}")
    case = sift_case(orc)
    typical = float(np.sqrt(np.median(orc.bruteforce(case[0], case[1][:50], 10)[1][:, 9])))   # an L2 distance
    got, ref = run_both(gpu, orc, case, k, frac * typical, **kw)
    check(got, ref, f"k={k}")


def test_tiny_and_shapes(gpu, orc):
    step("alg2 tiny / d=960 / uint8")
    got, ref = run_both(gpu, orc, tiny_case(orc), 10, 1.5, m_c=8, m_v=8, lambda_visit=10)
    check(got, ref, "tiny", exact=False)
    def make960():
        base, queries = workloads.single_gaussian(2500, 960, seed=960, nq=64)
        adj, lam = orc.build_graph(base, 16)
        return base, queries, adj, lam
    got, ref = run_both(gpu, orc, cached("gauss960", make960), 10, 3.0)
    check(got, ref, "d=960", exact=False)
    def make8():
        base, queries = workloads.sift_like(N=8000, nq=100, seed=5)
        b8 = base.astype(np.uint8)
        adj, lam = orc.build_graph(b8, 16)
        return b8, queries, adj, lam
    case8 = cached("u8", make8)
    got, ref = run_both(gpu, orc, case8, 10, 40.0)
    check(got, ref, "u8")
    # queries that are not integers (and one outside the byte range) take the fp64 route on the same byte rows
    mixed = case8[1].copy()
    mixed[::2] += np.float32(0.375)
    mixed[1, 0] = 300.0
    got, ref = run_both(gpu, orc, (case8[0], mixed, case8[2], case8[3]), 10, 40.0)
    check(got, ref, "u8 mixed")


def test_segment_overflow_star(gpu, orc):
    """Hub with 40 leaves: one queue segment keeps the 32 nearest (33 expansions), two keep all (41)."""
    step("alg2 star")
    g = np.random.default_rng(53)
    N = 41
    base = np.zeros((N, 4), np.float32)
    base[1:, 0] = g.permutation(40) + 1.0
    adj = np.full((N, 40), -1, np.int32)
    lam = np.full((N, 40), 255, np.uint8)
    adj[0, :40] = np.arange(1, N)
    lam[0, :40] = 0
    adj[1:, 0] = 0
    lam[1:, 0] = 0
    q = np.zeros((1, 4), np.float32)
    seed = next(sd for sd in range(300) if 0 in [orc.seed_id(sd, 0, t, N) for t in range(32)])
    for m_c, hops in ((1, 33), (2, 41)):
        got, ref = run_both(gpu, orc, (base, q, adj, lam), 64, 3.0e38, m_c=m_c, m_v=8, lambda_visit=1, seed=seed)
        check(got, ref, f"star m_c={m_c}")
        assert int(got[2].hops[0]) == hops


def test_push_that_drops_a_later_neighbour(gpu, orc):
    """The hand-worked hop of tests/golden/alg2_segment_overflow.json: counters and ranking equal the
    hand-derived ones (the listing's look-up order), not only the oracle's."""
    step("alg2 hand-worked segment overflow")
    from test_oracle_alg2 import overflow_case
    doc, base, adj, lam, q = overflow_case()
    prm = doc["params"]
    seed = next(sd for sd in range(300) if 0 in [orc.seed_id(sd, 0, t, len(base)) for t in range(32)])
    for T in (1, 2, 3):
        want = doc["expected"][f"T={T}"]
        got, ref = run_both(gpu, orc, (base, q, adj, lam), prm["k"], prm["delta"], m_c=prm["m_c"], m_v=prm["m_v"],
                            lambda_visit=prm["lambda_visit"], seed=seed, max_hops=T)
        check(got, ref, f"golden T={T}")
        st = got[2]
        assert [int(st.hops[0]), int(st.dist_evals[0]), int(st.dedup_hits[0])] == [want["hops"], want["dist_evals"], want["skips"]]
        assert list(got[0][0][:len(want["ids"])]) == want["ids"]


def test_arguments(gpu, orc):
    step("alg2 arguments")
    base, queries, adj, lam = tiny_case(orc)[:4]
    g = gpu.ann_graph_import(dev(adj), dev(lam), 32)
    b, q = dev(base), dev(queries)
    for k, m_c, m_v, delta in ((0, 4, 4, 0.0), (65, 4, 4, 0.0), (10, 0, 4, 0.0), (10, 4, 65, 0.0), (10, 4, 4, -1.0)):
        with pytest.raises(gpu.AnnError):
            gpu.ann_search_alg2(g, b, q, k, delta, m_c=m_c, m_v=m_v)
    ids, s = gpu.ann_search_alg2(g, b, q[:0], 5, 0.0)
    assert ids.shape == (0, 5)
