"""Pins for the oracle's canonical distance, exact k-NN / brute force, seed
generator and recall.  None of these use a GPU."""
import json
import os

import numpy as np

import workloads

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def np_canonical(a, b):
    """fl32( sum (double)(fl32(a-b))^2 ), written with numpy array ops."""
    t = (a.astype(np.float32) - b.astype(np.float32)).astype(np.float32)
    return np.float32(np.sum(t.astype(np.float64) ** 2, axis=-1))


# ------------------------------------------------------------------ distance
def test_sqdist_integer_data_is_exact(orc):
    g = np.random.default_rng(0)
    for d in (4, 32, 128):
        a = g.integers(0, 256, size=d)
        b = g.integers(0, 256, size=d)
        exact = int(np.sum((a - b) ** 2))          # integer arithmetic
        assert exact < 2 ** 24
        got = orc.sqdist(a.astype(np.float32), b.astype(np.float32))
        assert float(got) == float(exact)


def test_sqdist_closed_forms(orc):
    # 3-4-5 triangle, zero distance, one-hot difference
    assert orc.sqdist(np.array([0, 0, 0, 0], np.float32), np.array([3, 4, 0, 0], np.float32)) == 25.0
    x = np.arange(8, dtype=np.float32) * 0.37
    assert orc.sqdist(x, x) == 0.0
    y = x.copy()
    y[5] += np.float32(2.0)
    assert orc.sqdist(x, y) == np.float32((np.float32(x[5] + np.float32(2.0)) - x[5]) ** 2)


def test_sqdist_against_fp64_within_bound_and_symmetric(orc):
    g = np.random.default_rng(1)
    for d in (32, 96, 128, 960):
        for _ in range(20):
            a = g.standard_normal(d).astype(np.float32) * 3
            b = g.standard_normal(d).astype(np.float32) * 3
            truth = np.sum((a.astype(np.float64) - b.astype(np.float64)) ** 2)
            got = orc.sqdist(a, b)
            # one rounding of each difference (rel 2^-24 on t => 2^-23 on t^2) plus the final one
            assert abs(float(got) - truth) <= 1.9e-7 * truth
            assert got.tobytes() == orc.sqdist(b, a).tobytes()      # bitwise symmetric
            assert got.tobytes() == np_canonical(a, b).tobytes()


def test_sqdist_rounds_difference_in_fp32_not_fp64(orc):
    """1 - 2^-25 is halfway between two fp32 numbers and rounds (to even) to 1,
    so the canonical value is 1; squaring the unrounded difference would give
    1 - 2^-24 + 2^-50, which rounds to the fp32 number below 1."""
    a = np.array([1.0, 0, 0, 0], np.float32)
    b = np.array([2.0 ** -25, 0, 0, 0], np.float32)
    assert orc.sqdist(a, b) == np.float32(1.0)
    assert np.float32((1.0 - 2.0 ** -25) ** 2) == np.float32(1.0 - 2.0 ** -24)


# ---------------------------------------------------------------- brute force
def np_topk(base, q, k, exclude=None):
    s = np_canonical(base, q[None, :])
    ids = np.arange(base.shape[0])
    if exclude is not None:
        keep = ids != exclude
        s, ids = s[keep], ids[keep]
    order = np.lexsort((ids, s))[:k]
    return ids[order].astype(np.int32), s[order]


def test_bruteforce_matches_numpy_definition(orc):
    base, queries = workloads.single_gaussian(700, 12, seed=3, nq=25)
    ids, s = orc.bruteforce(base, queries, 10)
    for i in range(queries.shape[0]):
        e_ids, e_s = np_topk(base, queries[i], 10)
        assert np.array_equal(ids[i], e_ids)
        assert s[i].tobytes() == e_s.astype(np.float32).tobytes()


def test_bruteforce_uint8_base(orc):
    g = np.random.default_rng(5)
    base = g.integers(0, 256, size=(300, 16), dtype=np.uint8)
    queries = g.integers(0, 256, size=(7, 16)).astype(np.float32)
    ids, s = orc.bruteforce(base, queries, 5)
    ids2, s2 = orc.bruteforce(base.astype(np.float32), queries, 5)
    assert np.array_equal(ids, ids2) and np.array_equal(s, s2)
    # exact integers
    for i in range(7):
        ex = np.sum((base[ids[i]].astype(np.int64) - queries[i].astype(np.int64)) ** 2, axis=1)
        assert np.array_equal(ex.astype(np.float32), s[i])


def test_bruteforce_pads_when_k_exceeds_n(orc):
    base = np.eye(4, dtype=np.float32)[:3]
    ids, s = orc.bruteforce(base, base[:1], 5)
    assert list(ids[0][3:]) == [-1, -1] and np.all(np.isinf(s[0][3:]))
    assert ids[0][0] == 0 and s[0][0] == 0.0


def test_knn_excludes_self_and_matches_numpy(orc):
    base = workloads.single_gaussian(400, 8, seed=7)
    ids, s = orc.knn(base, 12)
    for i in range(0, 400, 13):
        e_ids, e_s = np_topk(base, base[i], 12, exclude=i)
        assert np.array_equal(ids[i], e_ids)
        assert s[i].tobytes() == e_s.astype(np.float32).tobytes()
    assert not np.any(ids == np.arange(400)[:, None])


def test_knn_lattice_ties_break_by_smaller_id(orc):
    """7x7 integer grid, id = 7*r + c.  For the centre point (3,3), id 24: the
    four neighbours at s=1 are ids 17,23,25,31, then the four at s=2 are
    16,18,30,32, then the four at s=4 are 10,22,26,38 (closed form)."""
    base = workloads.integer_lattice(7)
    base4 = np.zeros((49, 4), np.float32)
    base4[:, :2] = base
    ids, s = orc.knn(base4, 12)
    assert list(ids[24]) == [17, 23, 25, 31, 16, 18, 30, 32, 10, 22, 26, 38]
    assert list(s[24]) == [1, 1, 1, 1, 2, 2, 2, 2, 4, 4, 4, 4]
    # corner (0,0): s=1 -> ids 1,7 ; s=2 -> 8 ; s=4 -> 2,14 ; s=5 -> 9,15
    assert list(ids[0][:7]) == [1, 7, 8, 2, 14, 9, 15]


def test_knn_exact_duplicates_are_ordinary_neighbours(orc):
    base = np.zeros((6, 4), np.float32)
    base[:, 0] = [0, 0, 1, 2, 3, 0]          # ids 0,1,5 coincide
    ids, s = orc.knn(base, 3)
    assert list(ids[0]) == [1, 5, 2] and list(s[0]) == [0, 0, 1]
    assert list(ids[5]) == [0, 1, 2]


# --------------------------------------------------------------------- seeds
def test_seed_generator_matches_published_splitmix64_vector(orc):
    ref = json.load(open(os.path.join(GOLD, "splitmix64_seed1234567.json")))
    for j, word in enumerate(ref["outputs"]):
        assert orc.seed_id(ref["state"], 0, j, 2 ** 62) == word >> 2


def test_seed_generator_range_and_query_dependence(orc):
    N = 1000
    a = [orc.seed_id(9, 0, j, N) for j in range(64)]
    b = [orc.seed_id(9, 1, j, N) for j in range(64)]
    assert all(0 <= v < N for v in a + b)
    assert a != b and len(set(a)) > 48
    # counter layout: query index occupies the high 32 bits of the counter
    assert orc.seed_id(9, 1, 0, 2 ** 62) != orc.seed_id(9, 0, 1, 2 ** 62)
    big = [orc.seed_id(77, 3, j, 10 ** 8) for j in range(2000)]
    assert abs(np.mean(big) / 10 ** 8 - 0.5) < 0.03           # roughly uniform


# -------------------------------------------------------------------- recall
def test_recall_definition(orc):
    truth = np.array([[1, 2, 3, 4], [5, 6, 7, 8]], np.int32)
    found = np.array([[4, 3, 9, -1], [8, 7, 6, 5]], np.int32)
    assert orc.recall(found, truth) == (2 + 4) / 8.0          # Eq. 3
    assert orc.recall(truth, truth) == 1.0


def test_binary16_rows_convert_exactly_and_serve_as_base(orc):
    """Rows stored as IEEE binary16: all 65,536 bit patterns convert like numpy's routine, and a base
    set given in binary16 behaves exactly like the same values given in fp32."""
    import ctypes as C
    lib = orc.lib()
    lib.orc_half_to_float.restype = C.c_float
    lib.orc_half_to_float.argtypes = [C.c_uint16]
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float32)
    got = np.array([lib.orc_half_to_float(int(b)) for b in bits], np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan) and np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))
    base = workloads.single_gaussian(400, 16, seed=77).astype(np.float16)
    q = workloads.single_gaussian(20, 16, seed=78)
    a16 = orc.bruteforce(base, q, 7)
    a32 = orc.bruteforce(base.astype(np.float32), q, 7)
    assert np.array_equal(a16[0], a32[0]) and np.array_equal(a16[1], a32[1])
    assert np.array_equal(orc.build_graph(base, 8)[0], orc.build_graph(base.astype(np.float32), 8)[0])
