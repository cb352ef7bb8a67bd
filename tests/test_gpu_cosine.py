"""Parity of the HIP path under the cosine metric (Table 1: m = Cos) with the CPU oracle:
row normalisation, graph build (Eq. 2 with alpha on m = 1 - cos), and every search entry point."""
import numpy as np
import pytest
import torch

import workloads
from conftest import cached, step
from parity import assert_bitwise, compare_topk

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def cosine_case(orc, N=3000, nq=200, d=100, K=16):
    """Glove-like raw rows, the oracle's unit rows and the oracle's cosine graph."""
    def make():
        base_raw, q_raw = workloads.glove_like(N=N, nq=nq, d=d, components=24, seed=31)
        base, q = orc.normalize_rows(base_raw), orc.normalize_rows(q_raw)
        adj, lam, st = orc.build_graph(base, K, stages=True, metric="cosine")
        return dict(base_raw=base_raw, q_raw=q_raw, base=base, q=q, adj=adj, lam=lam, **st)
    return cached(f"cosine_{N}_{nq}_{d}_{K}", make)


def test_normalize_rows_matches_the_oracle(gpu, orc):
    step("ann_normalize_rows vs oracle")
    c = cosine_case(orc)
    for raw, want in ((c["base_raw"], c["base"]), (c["q_raw"], c["q"])):
        got = gpu.ann_normalize_rows(dev(raw)).cpu().numpy()
        # the fp64 sum of squares is formed in another order: a norm may round the other way once in ~1e9 rows
        bad = np.argwhere((got != want).any(axis=1))[:, 0]
        assert len(bad) <= 1, f"{len(bad)} rows differ"
        assert np.abs(got.astype(np.float64) - want).max() <= 1.2e-7
    x = dev(c["q_raw"].copy())
    assert gpu.ann_normalize_rows(x, out=x) is x and np.array_equal(x.cpu().numpy(), c["q"])   # in place
    z = torch.zeros((3, 8), device="cuda")
    assert torch.equal(gpu.ann_normalize_rows(z), z)


def test_cosine_graph_build(gpu, orc):
    step("cosine graph build (alpha on m) vs oracle")
    c = cosine_case(orc)
    g = gpu.ann_build_graph_ex(dev(c["base"]), 16, metric="cosine")
    adj, lam = gpu.ann_graph_export(g)
    adj, lam = adj.cpu().numpy(), lam.cpu().numpy()
    rows = np.unique(np.argwhere((adj != c["adj"]) | (lam != c["lam"]))[:, 0])
    for r in rows:                                   # excuse only near-ties inside the oracle's lists
        s = np.sort(c["g2_s"][r][:c["g2_deg"][r]].astype(np.float64))
        gaps = np.diff(s) / np.maximum(s[1:], 1e-30)
        assert gaps.size and gaps.min() < 1e-5, f"row {r} differs without a near-tie"
    assert len(rows) <= 0.01 * adj.shape[0]
    # and it is not the L2 graph of the same rows: alpha acts on m, not on the distance
    g_l2 = gpu.ann_build_graph_ex(dev(c["base"]), 16, metric="l2")
    assert not torch.equal(gpu.ann_graph_export(g_l2)[0].cpu(), torch.from_numpy(c["adj"]))


@pytest.mark.parametrize("mode,L,lv", [(1, 32, 5), (2, 32, 10), (1, 100, 32), (2, 16, 5)])
def test_cosine_search(gpu, orc, mode, L, lv):
    step(f"cosine search mode={mode} L={L} lambda_visit={lv}")
    c = cosine_case(orc)
    g = gpu.ann_graph_import(dev(c["adj"]), dev(c["lam"]), c["base"].shape[1])
    ids, m = gpu.ann_search_ex(g, dev(c["base"]), dev(c["q"]), 10, L, mode=mode, lambda_visit=lv, seed=7, metric="cosine")
    ids_o, m_o = orc.search(c["adj"], c["lam"], c["base"], c["q"], 10, L, lv, seed=7, metric="cosine")
    assert compare_topk(ids.cpu().numpy(), m.cpu().numpy(), ids_o, m_o, "cosine search") <= 2
    # the values are 1 - cos of the raw rows
    raw = 1.0 - np.einsum("qd,qkd->qk", c["q_raw"].astype(np.float64) / np.linalg.norm(c["q_raw"].astype(np.float64), axis=1)[:, None],
                          (c["base_raw"].astype(np.float64) / np.linalg.norm(c["base_raw"].astype(np.float64), axis=1)[:, None])[ids_o])
    assert np.abs(raw - m.cpu().numpy()).max() < 5e-7


def test_cosine_multi_search_and_alg2(gpu, orc):
    c = cosine_case(orc)
    g = gpu.ann_graph_import(dev(c["adj"]), dev(c["lam"]), c["base"].shape[1])
    b, q = dev(c["base"]), dev(c["q"][:64])
    step("cosine multi-search")
    ids, m = gpu.ann_search_multi(g, b, q, 10, 8, max_hops=6, seed=3, metric="cosine")
    ids_o, m_o = orc.search_multi(c["adj"], c["lam"], c["base"], c["q"][:64], 10, 8, max_hops=6, seed=3, metric="cosine")
    assert compare_topk(ids.cpu().numpy(), m.cpu().numpy(), ids_o, m_o, "cosine multi") <= 2
    step("cosine Alg. 2 structures, delta in units of 1 - cos")
    delta = 0.02
    ids, m, st = gpu.ann_search_alg2(g, b, q, 16, delta, seed=3, lambda_visit=5, want_stats=True, metric="cosine")
    ids_o, m_o, st_o = orc.search_alg2(c["adj"], c["lam"], c["base"], c["q"][:64], 16, delta, seed=3, lambda_visit=5,
                                       want_stats=True, metric="cosine")
    assert compare_topk(ids.cpu().numpy(), m.cpu().numpy(), ids_o, m_o, "cosine alg2") <= 2
    assert_bitwise(st.hops.cpu().numpy().astype(np.uint32), st_o[:, 0], "alg2 hops")
    # delta matters and is not read in squared-distance units: with 2*delta the walk is longer
    _, _, st2 = gpu.ann_search_alg2(g, b, q, 16, 2 * delta, seed=3, lambda_visit=5, want_stats=True, metric="cosine")
    assert int(st2.hops.sum()) > int(st.hops.sum())


def test_cosine_needs_fp32_rows(gpu):
    base = torch.randint(0, 255, (512, 32), dtype=torch.uint8, device="cuda")
    with pytest.raises(gpu.AnnError):
        gpu.ann_build_graph_ex(base, 8, metric="cosine")


def test_inner_product_by_reduction_to_l2(gpu, orc):
    step("inner product: augmented rows, build + search on them, ranking by <q,x>")
    base, q = workloads.glove_like(N=3000, nq=100, d=100, components=24, seed=32)
    M = gpu.ann_max_row_norm(dev(base))
    assert M == np.float32(np.sqrt((base.astype(np.float64) ** 2).sum(1).max()))
    ab = gpu.ann_ip_augment_rows(dev(base), M)
    aq = gpu.ann_ip_augment_rows(dev(q), is_query=True)
    ab_o, aq_o = orc.ip_augment_rows(base, M), orc.ip_augment_rows(q, is_query=True)
    assert np.array_equal(aq.cpu().numpy(), aq_o)
    assert np.abs(ab.cpu().numpy().astype(np.float64) - ab_o).max() <= 1e-6 * M      # the fp64 sum is formed in another order
    assert (ab.cpu().numpy() != ab_o).any(axis=1).sum() <= 3
    # from here on both sides work on the oracle's rows
    adj_o, lam_o = orc.build_graph(ab_o, 16)
    g = gpu.ann_build_graph_ex(dev(ab_o), 16)
    adj, lam = gpu.ann_graph_export(g)
    assert (adj.cpu().numpy() != adj_o).any(axis=1).sum() <= 0.01 * 3000
    g = gpu.ann_graph_import(dev(adj_o), dev(lam_o), 104)
    ids, s = gpu.ann_search_ex(g, dev(ab_o), dev(aq_o), 10, 64, mode=1, lambda_visit=10)
    ref = orc.search(adj_o, lam_o, ab_o, aq_o, 10, 64, 10)
    assert compare_topk(ids.cpu().numpy(), s.cpu().numpy(), ref[0], ref[1], "ip search") == 0
    ip = q.astype(np.float64) @ base.astype(np.float64).T
    truth = np.argsort(-ip, axis=1)[:, :10].astype(np.int32)
    assert orc.recall(ids.cpu().numpy(), truth) > 0.9
    got_ip = ((q.astype(np.float64) ** 2).sum(1)[:, None] + float(M) ** 2 - s.cpu().numpy().astype(np.float64)) / 2
    assert np.abs(got_ip - np.take_along_axis(ip, ids.cpu().numpy().astype(np.int64), 1)).max() < 1e-5 * float(M) ** 2
    with pytest.raises(gpu.AnnError):
        gpu.ann_ip_augment_rows(dev(base))            # base rows need M
