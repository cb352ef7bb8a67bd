"""Parity of the HIP graph build (exact k-NN contraction, two-stage diversification)
and of the brute-force top-k with the CPU oracle."""
import numpy as np
import pytest
import torch

import workloads
from conftest import cached, sift_case, step, tiny_case
from parity import assert_bitwise, compare_topk

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def check_graph(gpu, orc, base, K, what, ref=None, max_excused=0, **kw):
    """GPU build vs oracle build: adjacency and lambda identical.  A caller whose data holds
    constructed near-ties may allow `max_excused` rows to differ, and only rows in which the
    oracle's own competing distances are closer than 1e-5 relative; no caller needs it so far,
    so every call asserts that no row differs."""
    okw = dict(alpha=kw.get("alpha", 1.2), lambda0=kw.get("lambda0", 9))
    if kw.get("rev_cap"):
        okw["rev_cap"] = kw["rev_cap"]
    adj_o, lam_o, st = ref if ref is not None else orc.build_graph(base, K, stages=True, **okw)
    g = gpu.ann_build_graph_ex(dev(base), K, **kw)
    adj, lam = gpu.ann_graph_export(g)
    adj, lam = adj.cpu().numpy(), lam.cpu().numpy()
    assert gpu.ann_graph_info(g) == (base.shape[0], K, base.shape[1])
    rows = np.unique(np.argwhere((adj != adj_o) | (lam != lam_o))[:, 0])
    for r in rows:                                   # excuse only near-ties inside the oracle's lists
        s = np.sort(st["g2_s"][r][:st["g2_deg"][r]].astype(np.float64))
        gaps = np.diff(s) / np.maximum(s[1:], 1e-30)
        assert gaps.size and gaps.min() < 1e-5, (f"{what}: row {r} differs without a near-tie: "
                                                 f"{adj[r]} / {lam[r]} vs {adj_o[r]} / {lam_o[r]}")
    assert len(rows) <= max_excused, f"{what}: {len(rows)} rows differ at near-ties (allowed: {max_excused})"
    valid = adj >= 0
    assert np.all(lam[valid] <= okw["lambda0"]) and np.all(lam[~valid] == 255)
    return len(rows)


def test_knn_tiny_fp32(gpu, orc):
    step("ann_knn tiny (real-valued rows: bf16 split path)")
    base, _, _, _, st = tiny_case(orc)
    ref = (st["knn_id"], st["knn_s"])
    ids, s = gpu.ann_knn(dev(base), 16)
    assert compare_topk(ids.cpu().numpy(), s.cpu().numpy(), ref[0], ref[1], "knn tiny") == 0
    assert_bitwise(s.cpu().numpy(), ref[1], "knn tiny dists")


def test_knn_integer_bf16(gpu, orc):
    step("ann_knn sift-like 20k (integer rows: int8 MFMA path, exact)")
    base, _, _, _, st = sift_case(orc)
    ref = (st["knn_id"], st["knn_s"])
    ids, s = gpu.ann_knn(dev(base), 32)
    assert_bitwise(ids.cpu().numpy(), ref[0], "knn ids")
    assert_bitwise(s.cpu().numpy(), ref[1], "knn dists")


def test_knn_ragged_sizes_and_ties(gpu, orc):
    """N not a multiple of any tile; integer lattice (many equal distances, id tie rule);
    exact duplicates."""
    step("ann_knn ragged / lattice / duplicates")
    lat = workloads.integer_lattice(23)                        # 529 points
    b = np.zeros((529, 4), np.float32)
    b[:, :2] = lat
    ref = orc.knn(b, 12)
    ids, s = gpu.ann_knn(dev(b), 12)
    assert_bitwise(ids.cpu().numpy(), ref[0], "lattice ids")
    assert_bitwise(s.cpu().numpy(), ref[1], "lattice dists")
    g = np.random.default_rng(3)
    x = g.standard_normal((1237, 20)).astype(np.float32)
    x[100:110] = x[5]                                          # ten exact copies of row 5
    ref = orc.knn(x, 15)
    ids, s = gpu.ann_knn(dev(x), 15)
    assert compare_topk(ids.cpu().numpy(), s.cpu().numpy(), ref[0], ref[1], "dups") == 0
    tiny_n = g.standard_normal((9, 8)).astype(np.float32)      # N barely above K
    ref = orc.knn(tiny_n, 8)
    ids, s = gpu.ann_knn(dev(tiny_n), 8)
    assert_bitwise(ids.cpu().numpy(), ref[0], "N=9 ids")


def test_knn_uint8(gpu, orc):
    step("ann_knn uint8")
    base, _ = workloads.sift_like(N=6000, nq=1, seed=5)
    b8 = base.astype(np.uint8)
    ref = orc.knn(b8, 16)
    ids, s = gpu.ann_knn(dev(b8), 16)
    assert_bitwise(ids.cpu().numpy(), ref[0], "u8 knn ids")
    assert_bitwise(s.cpu().numpy(), ref[1], "u8 knn dists")


@pytest.mark.parametrize("precise", [False, True])
@pytest.mark.parametrize("d", [8, 96, 128, 960])
def test_knn_real_valued_shapes(gpu, orc, d, precise):
    """Real-valued rows pass the filter as one scaled binary16 part, or (knn_filter = 1, also the
    library's own fallback) as bf16 hi + lo parts: the lists equal the oracle's either way."""
    step(f"ann_knn gaussian d={d} precise={precise}")
    base = workloads.single_gaussian(3000 if d < 900 else 1500, d, seed=100 + d)
    ref = orc.knn(base, 16)
    ids, s, st = gpu.ann_knn(dev(base), 16, knn_filter=1 if precise else 0, want_stats=True)
    assert compare_topk(ids.cpu().numpy(), s.cpu().numpy(), ref[0], ref[1], f"knn d={d}") == 0
    assert st["knn_contraction"] == (2 if precise else 1) and st["knn_ms"] > 0   # the form asked for is the one that ran


@pytest.mark.parametrize("kind", ["int8", "real", "wide"])
def test_knn_in_several_row_blocks(gpu, orc, kind):
    """The sweep over all columns is repeated per block of query rows (2^21 rows by default); a small
    knn_row_block runs that loop several times on a small set, last block ragged."""
    step(f"ann_knn in row blocks of 512: {kind}")
    if kind == "int8":
        base = workloads.sift_like(N=1800, nq=1, seed=9)[0]
    else:
        base = workloads.single_gaussian(1800, 32 if kind == "real" else 160, seed=12)
    ref = orc.knn(base, 16)
    calls = []
    ids, s = gpu.ann_knn(dev(base), 16, knn_row_block=512, progress=lambda step_, done, total: calls.append((step_, done, total)))
    assert compare_topk(ids.cpu().numpy(), s.cpu().numpy(), ref[0], ref[1], f"row blocks {kind}") == 0
    assert [c[1] for c in calls if c[0] == "knn-rows"] == [512, 1024, 1536, 1800]
    assert all(c[1] <= c[2] == 1800 for c in calls if c[0] == "knn-sweep")
    with pytest.raises(gpu.AnnError):
        gpu.ann_knn(dev(base), 16, knn_row_block=100)


@pytest.mark.parametrize("d", [16, 200])
def test_knn_outlier_row_sends_every_row_to_the_fallbacks(gpu, orc, d):
    """One row 10^4 times longer than the rest makes the acceptance margin (a multiple of the largest norm)
    wider than every gap: the one-part filter gives up, the hi + lo filter runs, and its rejected rows are
    redone by the plain scan.  The lists still equal the oracle's."""
    step(f"ann_knn outlier d={d}")
    g = np.random.default_rng(77 + d)
    base = g.standard_normal((1500, d)).astype(np.float32)
    base[123] *= 1.0e4
    ref = orc.knn(base, 16)
    ids, s = gpu.ann_knn(dev(base), 16)
    assert compare_topk(ids.cpu().numpy(), s.cpu().numpy(), ref[0], ref[1], f"outlier d={d}") == 0


@pytest.mark.parametrize("d,N", [(132, 1237), (200, 2100), (516, 1500), (2048, 700)])
def test_knn_real_valued_wide_rows(gpu, orc, d, N):
    """Real-valued rows wider than 128 elements (operands staged through LDS in slabs): N not a multiple
    of the tile, d not a multiple of the slab, rows far from the origin, and separate query rows."""
    step(f"ann_knn wide rows d={d} N={N}")
    g = np.random.default_rng(500 + d)
    base = (g.standard_normal((N, d)) * g.uniform(0.2, 2.0, size=d) + 3.0).astype(np.float32)
    ref = orc.knn(base, 16)
    ids, s = gpu.ann_knn(dev(base), 16)
    assert compare_topk(ids.cpu().numpy(), s.cpu().numpy(), ref[0], ref[1], f"wide knn d={d}") == 0
    q = (base[:70] + g.standard_normal((70, d)) * 0.3).astype(np.float32)
    ref = orc.bruteforce(base, q, 10)
    ids, s = gpu.ann_bruteforce(dev(base), dev(q), 10)
    assert compare_topk(ids.cpu().numpy(), s.cpu().numpy(), ref[0], ref[1], f"wide bf d={d}") == 0


@pytest.mark.parametrize("kind", ["real", "real, hi + lo parts", "integer"])
def test_knn_wide_rows_over_several_spans(gpu, orc, kind):
    """Wide rows on a set large enough that one launch holds 25 query tiles of 256 rows (the last with 56; 49 of 128
    rows with hi + lo parts) and more than one candidate span (the last ending in a ragged tile): 6,200 x 264."""
    step(f"ann_knn wide rows over several spans, {kind}")
    N, d = 6200, 264
    g = np.random.default_rng(77)
    protos = g.normal(0, 1, size=(40, d))
    base = protos[g.integers(0, 40, size=N)] + 0.4 * g.standard_normal((N, d))
    if kind == "integer":
        base = np.clip(np.rint(base * 30 + 128), 0, 255)
    base = base.astype(np.float32)
    ref = orc.knn(base, 24)
    ids, s = gpu.ann_knn(dev(base), 24, knn_filter=1 if "hi + lo" in kind else 0)
    if kind == "integer":
        assert_bitwise(ids.cpu().numpy(), ref[0], "ids")
        assert_bitwise(s.cpu().numpy(), ref[1], "dists")
    else:
        assert compare_topk(ids.cpu().numpy(), s.cpu().numpy(), ref[0], ref[1], "several spans") == 0
        assert_bitwise(s.cpu().numpy(), ref[1], "dists")


@pytest.mark.parametrize("d", [208, 320, 1024, 1100])
def test_knn_integer_wide_rows(gpu, orc, d):
    """Integer rows in [0,255] wider than 128 elements: centred they are exact in bf16 and, up to d = 1024,
    so is every partial sum of the fp32 accumulators (the filter then runs in int32); wider ones go the
    way of real-valued rows.  fp32 and uint8 storage, and separate query rows (integer and not)."""
    step(f"ann_knn integer rows d={d}")
    g = np.random.default_rng(700 + d)
    protos = g.integers(0, 256, size=(24, d))
    base = np.clip(protos[g.integers(0, 24, size=900)] + np.rint(g.normal(0, 25, size=(900, d))), 0, 255).astype(np.float32)
    base[:3] = 255.0                                        # rows of the largest norm, exact copies of each other
    base[3:6] = 0.0
    ref = orc.knn(base, 16)
    ids, s = gpu.ann_knn(dev(base), 16)
    assert_bitwise(ids.cpu().numpy(), ref[0], f"integer wide ids d={d}")
    assert_bitwise(s.cpu().numpy(), ref[1], f"integer wide dists d={d}")
    if d <= 1024:
        b8 = base.astype(np.uint8)
        ids, s = gpu.ann_knn(dev(b8), 16)
        assert_bitwise(ids.cpu().numpy(), ref[0], f"integer wide ids u8 d={d}")
        q = base[100:140].copy()
        q[::2] = np.clip(q[::2] + 3.0, 0, 255)
        refb = orc.bruteforce(b8, q, 10)
        ids, s = gpu.ann_bruteforce(dev(b8), dev(q), 10)
        assert_bitwise(ids.cpu().numpy(), refb[0], f"integer wide bf ids d={d}")
        assert_bitwise(s.cpu().numpy(), refb[1], f"integer wide bf dists d={d}")
        qr = (q + 0.25).astype(np.float32)                  # queries that are not integers: the split path on uint8 rows
        refb = orc.bruteforce(b8, qr, 10)
        ids, s = gpu.ann_bruteforce(dev(b8), dev(qr), 10)
        assert compare_topk(ids.cpu().numpy(), s.cpu().numpy(), refb[0], refb[1], f"integer wide bf real q d={d}") == 0


@pytest.mark.parametrize("d", [32, 160])
def test_bruteforce_queries_far_longer_than_the_base_rows(gpu, orc, d):
    """The scale of the one-part filter is set by the longest row of EITHER operand: queries 300 times longer
    than the base rows must neither overflow binary16 nor lose the base rows' digits."""
    step(f"ann_bruteforce long queries d={d}")
    g = np.random.default_rng(31 + d)
    base = g.standard_normal((2500, d)).astype(np.float32)
    q = (g.standard_normal((70, d)) * 300.0).astype(np.float32)
    q[::2] = base[:35] + (g.standard_normal((35, d)) * 0.05).astype(np.float32)   # and some queries among the rows
    ref = orc.bruteforce(base, q, 10)
    ids, s = gpu.ann_bruteforce(dev(base), dev(q), 10)
    assert compare_topk(ids.cpu().numpy(), s.cpu().numpy(), ref[0], ref[1], f"long queries d={d}") == 0


def test_bruteforce(gpu, orc):
    step("ann_bruteforce")
    base, queries = workloads.tiny()
    ref = orc.bruteforce(base, queries, 10)
    ids, s = gpu.ann_bruteforce(dev(base), dev(queries), 10)
    assert compare_topk(ids.cpu().numpy(), s.cpu().numpy(), ref[0], ref[1], "bf tiny") == 0
    base, queries = sift_case(orc)[:2]
    ref = orc.bruteforce(base, queries, 100)
    ids, s = gpu.ann_bruteforce(dev(base), dev(queries), 100)
    assert_bitwise(ids.cpu().numpy(), ref[0], "bf sift ids")
    assert_bitwise(s.cpu().numpy(), ref[1], "bf sift dists")
    b8 = base[:5000].astype(np.uint8)
    ref = orc.bruteforce(b8, queries[:50], 10)
    ids, s = gpu.ann_bruteforce(dev(b8), dev(queries[:50]), 10)
    assert_bitwise(ids.cpu().numpy(), ref[0], "bf u8 ids")
    real_q = (queries[:50] + 0.25).astype(np.float32)          # non-integer queries on uint8 rows
    ref = orc.bruteforce(b8, real_q, 10)
    ids, s = gpu.ann_bruteforce(dev(b8), dev(real_q), 10)
    assert compare_topk(ids.cpu().numpy(), s.cpu().numpy(), ref[0], ref[1], "bf u8 real q") == 0


def test_build_tiny(gpu, orc):
    step("ann_build_graph tiny")
    base, _, adj, lam, st = tiny_case(orc)
    assert check_graph(gpu, orc, base, 16, "tiny", ref=(adj, lam, st)) == 0


def test_build_integer_data(gpu, orc):
    step("ann_build_graph sift-like 20k")
    base, _, adj, lam, st = sift_case(orc)
    assert check_graph(gpu, orc, base, 32, "sift20k", ref=(adj, lam, st)) == 0


@pytest.mark.parametrize("kw", [dict(alpha=1.0, lambda0=2), dict(alpha=1.5, lambda0=30), dict(rev_cap=20),
                                dict(alpha=1.2, lambda0=0)])
def test_build_parameters(gpu, orc, kw):
    step(f"ann_build_graph params {kw}")
    base = workloads.single_gaussian(3000, 6, seed=31)
    base = np.concatenate([base, np.zeros((3000, 2), np.float32)], axis=1)       # d = 8
    assert check_graph(gpu, orc, base, 16, str(kw), **kw) == 0


@pytest.mark.parametrize("K,scale", [(16, 0.37), (40, 1.0 / 3.0)])
def test_build_real_valued_near_ties(gpu, orc, K, scale):
    """Real-valued rows take their pairwise distances from the matrix cores with an error band and decide a
    comparison of Eq. 2 / Eq. 1 exactly only inside it.  A scaled integer lattice is all near-ties: equal lattice
    offsets give distances that differ in the last bits (the scaled coordinates are rounded), so most comparisons
    fall inside the band and are settled by the canonical distance; K = 40 runs the three-block (lists up to 64) form.
    Exact copies of a row (distance 0) ride along."""
    step(f"ann_build_graph real-valued lattice K={K}")
    lat = workloads.integer_lattice(25).astype(np.float32)          # 625 points
    pts = np.zeros((625 + 6, 4), np.float32)
    pts[:625, :2] = lat * np.float32(scale)
    pts[625:] = pts[[7, 7, 300, 300, 300, 624]]
    assert not np.array_equal(pts, np.rint(pts))                     # not the integer-row path
    assert check_graph(gpu, orc, pts, K, f"lattice x {scale}", lambda0=30 if K > 32 else 9) == 0


def test_build_hub_node(gpu, orc):
    """A star: one centre that is the nearest neighbour of everybody gets an in-degree far
    above rev_cap; the cut must keep its (s,id)-smallest reverse edges."""
    step("ann_build_graph hub")
    g = np.random.default_rng(8)
    pts = g.standard_normal((2000, 8)).astype(np.float32)
    pts /= np.linalg.norm(pts, axis=1, keepdims=True)
    pts *= g.uniform(5.0, 6.0, size=(2000, 1)).astype(np.float32)
    pts[0] = 0
    assert check_graph(gpu, orc, pts, 8, "hub") == 0


def test_build_then_search_end_to_end(gpu, orc):
    """The default entry points: GPU-built graph searched on the GPU equals the oracle
    searching the oracle-built graph."""
    step("build + search end to end")
    base, queries, adj_o, lam_o, _ = sift_case(orc)
    g = gpu.ann_build_graph(dev(base), 32)
    ids, s = gpu.ann_search_ex(g, dev(base), dev(queries), 10, 64, mode=1, lambda_visit=5)
    ref = orc.search(adj_o, lam_o, base, queries, 10, 64, 5)
    assert_bitwise(ids.cpu().numpy(), ref[0], "e2e ids")
    assert_bitwise(s.cpu().numpy(), ref[1], "e2e dists")
    gt = orc.bruteforce(base, queries, 10)[0]
    assert orc.recall(ids.cpu().numpy(), gt) > 0.9


def test_knn_real_valued_with_large_offset_and_near_ties(gpu, orc):
    """The contraction only selects candidates; exactness must survive (a) rows far from the
    origin (norms much larger than distances) and (b) many almost-equal distances, where the
    acceptance test of the re-scoring pass fails and rows are redone by the plain scan."""
    step("ann_knn offset / near ties")
    g = np.random.default_rng(12)
    x = (g.standard_normal((3000, 16)) + 1000.0).astype(np.float32)
    ref = orc.knn(x, 16)
    ids, s = gpu.ann_knn(dev(x), 16)
    assert compare_topk(ids.cpu().numpy(), s.cpu().numpy(), ref[0], ref[1], "offset") == 0
    lat = workloads.integer_lattice(40)                                  # 1,600 points, massive ties ...
    y = np.zeros((1600, 4), np.float32)
    y[:, :2] = lat + g.uniform(-1e-4, 1e-4, size=lat.shape)              # ... broken by tiny real jitter
    ref = orc.knn(y, 12)
    ids, s = gpu.ann_knn(dev(y), 12)
    assert compare_topk(ids.cpu().numpy(), s.cpu().numpy(), ref[0], ref[1], "near ties") == 0
    q = (y[:50] + 0.3).astype(np.float32)
    ref = orc.bruteforce(y, q, 10)
    ids, s = gpu.ann_bruteforce(dev(y), dev(q), 10)
    assert compare_topk(ids.cpu().numpy(), s.cpu().numpy(), ref[0], ref[1], "near ties bf") == 0


def test_knn_rows_that_differ_in_their_last_bits(gpu, orc):
    """Rows near 1000 that differ by a few units in the last place: centred, they fall below binary16's normal
    range at the scale the row lengths dictate (the filter's absolute error term), distances are multiples of
    2^-28 with ties everywhere, and whatever the filters reject the plain scan redoes."""
    step("ann_knn last-bit differences")
    g = np.random.default_rng(5150)
    x = (1000.0 + 1.0e-4 * g.standard_normal((2000, 16))).astype(np.float32)
    ref = orc.knn(x, 12)
    ids, s = gpu.ann_knn(dev(x), 12)
    assert compare_topk(ids.cpu().numpy(), s.cpu().numpy(), ref[0], ref[1], "last bits") == 0


@pytest.mark.parametrize("scale", [1e-12, 1e12])
@pytest.mark.parametrize("d", [16, 200])
def test_knn_extreme_magnitudes(gpu, orc, scale, d):
    """Rows whose squares sit far from 1 in fp32 (1e-24 and 1e24 per element): the hi + lo split, the
    norms and the acceptance margin scale with the data, so the lists still equal the oracle's."""
    step(f"ann_knn magnitudes scale={scale:g} d={d}")
    g = np.random.default_rng(900 + d)
    base = (g.standard_normal((1500, d)) * scale).astype(np.float32)
    ref = orc.knn(base, 16)
    ids, s = gpu.ann_knn(dev(base), 16)
    assert compare_topk(ids.cpu().numpy(), s.cpu().numpy(), ref[0], ref[1], f"scale {scale:g} d={d}") == 0
