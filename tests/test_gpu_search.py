"""Parity of the HIP search kernels with the CPU oracle (same graph, same seeds).

Graphs here are built by the ORACLE and imported, so these tests isolate the
search path; tests/test_gpu_build.py covers the build."""
import numpy as np
import pytest
import torch

import workloads
from conftest import cached, sift_case, step, tiny_case
from parity import assert_bitwise, compare_topk

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run_both(gpu, orc, case, k, L, lv, mode, **kw):
    base, queries, adj, lam = case[:4]
    g = gpu.ann_graph_import(dev(adj), dev(lam), base.shape[1])
    okw = {a: kw[a] for a in ("n_seeds", "seed", "max_hops", "qi_offset") if a in kw}
    ref = orc.search(adj, lam, base, queries, k, L, lv, want_stats=True, **okw)
    ids, s, st = gpu.ann_search_ex(g, dev(base), dev(queries), k, L, mode=mode, lambda_visit=lv,
                                   want_stats=True, **kw)
    torch.cuda.synchronize()
    return (ids.cpu().numpy(), s.cpu().numpy(), st), ref


@pytest.mark.parametrize("mode,waves", [(1, 0), (2, 2), (2, 4), (2, 8)])
@pytest.mark.parametrize("lv", [10, 5])
def test_tiny_matches_oracle(gpu, orc, mode, waves, lv):
    step(f"tiny search mode={mode} waves={waves} lambda_visit={lv}")
    (ids, s, st), ref = run_both(gpu, orc, tiny_case(orc), 10, 32, lv, mode, waves_per_query=waves)
    excused = compare_topk(ids, s, ref[0], ref[1], "tiny")
    assert excused == 0
    assert_bitwise(s, ref[1], "tiny distances")
    assert np.array_equal(st.hops.cpu().numpy(), ref[2][:, 0])
    assert np.all(st.dist_evals.cpu().numpy() >= ref[2][:, 1])


@pytest.mark.parametrize("L,k,mode", [(16, 10, 1), (64, 10, 1), (65, 10, 1), (100, 10, 1), (128, 100, 1), (128, 10, 2),
                                      (129, 10, 1), (200, 100, 1), (257, 10, 2), (512, 10, 1), (512, 100, 2), (64, 10, 2),
                                      (1, 1, 1), (64, 64, 1), (65, 65, 2), (127, 127, 1), (128, 128, 2), (63, 63, 2)])
def test_integer_data_matches_oracle_exactly(gpu, orc, L, k, mode):
    """d=128 integer-valued rows: every distance is an exact integer, so parity is zero-tolerance."""
    step(f"sift20k search L={L} k={k} mode={mode}")
    (ids, s, st), ref = run_both(gpu, orc, sift_case(orc), k, L, 5 if mode == 1 else 10, mode)
    assert_bitwise(ids, ref[0], f"ids L={L}")
    assert_bitwise(s, ref[1], f"dists L={L}")
    assert np.array_equal(st.hops.cpu().numpy(), ref[2][:, 0])


def test_result_independent_of_visited_capacity(gpu, orc):
    step("visited capacity invariance")
    case = sift_case(orc)
    outs = []
    for slots in (64, 1024, 16384):
        (ids, s, st), ref = run_both(gpu, orc, case, 10, 48, 10, 1, visited_slots=slots)
        assert_bitwise(ids, ref[0], f"slots={slots}")
        outs.append(int(st.dist_evals.sum()))
    assert outs[0] >= outs[1] >= outs[2] >= int(ref[2][:, 1].sum())   # a smaller set only costs evaluations
    for slots in (192, 1280, 16320):   # table sizes that are no powers of two: probing wraps at the end
        (ids, s, st), ref = run_both(gpu, orc, case, 10, 48, 10, 1, visited_slots=slots)
        assert_bitwise(ids, ref[0], f"slots={slots}")
        assert_bitwise(s, ref[1], f"slots={slots} dists")
    # a list of two entries per lane with a set that forgets: re-scored ids meet their copies in the list
    (ids, s, st), ref = run_both(gpu, orc, case, 10, 100, 10, 1, visited_slots=64)
    assert_bitwise(ids, ref[0], "L=100 slots=64")
    assert int(st.dist_evals.sum()) > int(ref[2][:, 1].sum())
    # and a list searched in LDS (more than 128 entries)
    (ids, s, st), ref = run_both(gpu, orc, case, 100, 300, 10, 1, visited_slots=64)
    assert_bitwise(ids, ref[0], "L=300 slots=64")
    assert_bitwise(s, ref[1], "L=300 slots=64 dists")


@pytest.mark.parametrize("kw", [dict(n_seeds=1), dict(n_seeds=100), dict(n_seeds=32, seed=12345),
                                dict(max_hops=3), dict(qi_offset=1000)])
def test_seed_and_limit_parameters(gpu, orc, kw):
    step(f"search params {kw}")
    (ids, s, st), ref = run_both(gpu, orc, sift_case(orc), 10, 32, 10, 1, **kw)
    assert_bitwise(ids, ref[0], str(kw))
    assert_bitwise(s, ref[1], str(kw))
    assert np.array_equal(st.hops.cpu().numpy(), ref[2][:, 0])


@pytest.mark.parametrize("d,N", [(4, 3000), (8, 3000), (96, 4000), (100, 4000), (200, 3000), (960, 2500)])
def test_row_shapes(gpu, orc, d, N):
    """Real-valued rows of every supported chunking (d=960: 64 lanes x 4 chunks)."""
    step(f"row shape d={d}")
    def make():
        base, queries = workloads.single_gaussian(N, d, seed=d, nq=64)
        adj, lam = orc.build_graph(base, 16)
        return base, queries, adj, lam
    case = cached(f"gauss{d}", make)
    for mode in (1, 2):
        (ids, s, st), ref = run_both(gpu, orc, case, 10, 40, 10, mode)
        assert compare_topk(ids, s, ref[0], ref[1], f"d={d} mode={mode}") == 0
        assert_bitwise(s, ref[1], f"d={d} mode={mode}")


def test_uint8_rows(gpu, orc):
    step("uint8 rows")
    def make():
        base, queries = workloads.sift_like(N=8000, nq=100, seed=5)
        b8 = base.astype(np.uint8)
        adj, lam = orc.build_graph(b8, 16)
        return b8, queries, adj, lam
    case = cached("u8", make)
    for mode in (1, 2):
        (ids, s, st), ref = run_both(gpu, orc, case, 10, 32, 10, mode)
        assert_bitwise(ids, ref[0], "u8 ids")
        assert_bitwise(s, ref[1], "u8 dists")
    # queries that are not integers take the general path on the same uint8 rows; a batch that mixes
    # both kinds exercises the per-query choice
    mixed = case[1].copy()
    mixed[::2] += np.float32(0.375)
    mixed[1, 0] = 300.0                                   # integer but outside the byte range
    for L, mode in ((32, 1), (32, 2), (100, 1), (200, 1), (100, 2)):   # list in one register, two, in LDS
        (ids, s, st), ref = run_both(gpu, orc, (case[0], mixed, case[2], case[3]), 10, L, 10, mode)
        assert_bitwise(ids, ref[0], f"u8 mixed ids L={L} mode={mode}")
        assert_bitwise(s, ref[1], f"u8 mixed dists L={L} mode={mode}")
    # rows that do not fill the lanes' chunks (d = 48: three 16-byte chunks for eight lanes), both kinds of query
    def make48():
        base, queries = workloads.sift_like(N=6000, nq=60, d=48, seed=6)
        b8 = base.astype(np.uint8)
        adj, lam = orc.build_graph(b8, 16)
        q = queries.copy()
        q[::3] += np.float32(0.25)
        return b8, q, adj, lam
    case48 = cached("u8d48", make48)
    for mode in (1, 2):
        (ids, s, st), ref = run_both(gpu, orc, case48, 10, 40, 10, mode)
        assert_bitwise(ids, ref[0], f"u8 d=48 ids mode={mode}")
        assert_bitwise(s, ref[1], f"u8 d=48 dists mode={mode}")


def test_degenerate_graphs_and_padding(gpu, orc):
    step("degenerate graphs")
    # ring of 40 nodes, degree 1: fewer reachable nodes than k from one seed -> padded tail
    base = workloads.single_gaussian(40, 8, seed=2)
    adj = np.full((40, 4), -1, np.int32)
    lam = np.full((40, 4), 255, np.uint8)
    adj[:, 0] = (np.arange(40) + 1) % 40
    lam[:, 0] = 0
    q = base[:5].copy()
    ref = orc.search(adj, lam, base, q, 50, 64, 1, n_seeds=1)
    g = gpu.ann_graph_import(dev(adj), dev(lam), 8)
    ids, s = gpu.ann_search_ex(g, dev(base), dev(q), 50, 64, mode=1, lambda_visit=1, n_seeds=1)
    assert_bitwise(ids.cpu().numpy(), ref[0], "ring ids")
    assert_bitwise(s.cpu().numpy(), ref[1], "ring dists")
    assert (ref[0][:, 40:] == -1).all()
    # empty batch is valid
    e_ids, e_s = gpu.ann_search_ex(g, dev(base), dev(q[:0]), 5, 8)
    assert e_ids.shape == (0, 5)
    # export returns what was imported
    a2, l2 = gpu.ann_graph_export(g)
    assert_bitwise(a2.cpu().numpy(), adj, "export adj")
    assert_bitwise(l2.cpu().numpy(), lam, "export lam")
    assert gpu.ann_graph_info(g) == (40, 4, 8)


def test_argument_errors(gpu, orc):
    step("argument errors")
    base, queries, adj, lam = tiny_case(orc)[:4]
    g = gpu.ann_graph_import(dev(adj), dev(lam), 32)
    b, q = dev(base), dev(queries)
    for k, L in ((11, 10), (0, 10), (10, 513)):
        with pytest.raises(gpu.AnnError) as e:
            gpu.ann_search_ex(g, b, q, k, L)
        assert e.value.status == 1
    with pytest.raises(gpu.AnnError):
        gpu.ann_search_ex(g, b, q, 10, 32, visited_slots=100)        # not a multiple of 64
    with pytest.raises(gpu.AnnError):
        gpu.ann_search_ex(g, b, q, 10, 32, waves_per_query=3, mode=2)
    bad = adj.copy()
    bad[5, 0] = bad[5, 1]                                            # repeated id in a row
    with pytest.raises(gpu.AnnError):
        gpu.ann_graph_import(dev(bad), dev(lam), 32)
    bad = adj.copy()
    bad[7, 2] = 7                                                    # self loop
    with pytest.raises(gpu.AnnError):
        gpu.ann_graph_import(dev(bad), dev(lam), 32)
    badl = lam.copy()
    badl[3, 0] = 31                                                  # lambda above 30 on a used slot
    with pytest.raises(gpu.AnnError):
        gpu.ann_graph_import(dev(adj), dev(badl), 32)
    # defaults entry point: mode by batch size, lambda_visit by mode
    ids, s = gpu.ann_search(g, b, q, 10, 32)
    ref = orc.search(adj, lam, base, queries, 10, 32, 10)            # 100 queries -> small batch -> lambda < 10
    assert_bitwise(ids.cpu().numpy(), ref[0], "defaults")


@pytest.mark.gpu
@pytest.mark.parametrize("row_bytes", [16, 128, 384, 512, 1040, 3840, 8192])
def test_probe_gather_reads_the_rows_it_is_given(gpu, row_bytes):
    """The gather probe's one word per row is the xor of the row's 32-bit words (ids past the end read the last row)."""
    import torch
    P = gpu
    g = torch.Generator().manual_seed(row_bytes)
    N, n = 3001, 10_007
    tab = torch.randint(0, 256, (N, row_bytes), generator=g, dtype=torch.uint8)
    ids = torch.randint(0, N, (n,), generator=g, dtype=torch.int32)
    ids[5] = N + 17
    step(f"probe gather row_bytes={row_bytes}")
    got = P.ann_probe_gather(tab.cuda(), ids.cuda()).cpu().numpy().view(np.uint32)
    words = tab.numpy().view(np.uint32)
    want = np.bitwise_xor.reduce(words[np.minimum(ids.numpy(), N - 1)], axis=1)
    assert np.array_equal(got, want)


@pytest.mark.gpu
@pytest.mark.parametrize("kind,per_mfma", [(0, 32), (1, 16)])
def test_probe_mfma_counts_every_instruction(gpu, kind, per_mfma):
    """The matrix-core probe's operands are all ones, so each wavefront's word is 4 blocks x iters x k."""
    step(f"probe mfma kind={kind}")
    out = gpu.ann_probe_mfma(kind, 37, 1000).cpu().numpy()
    assert out.shape == (4 * 37,) and np.all(out == 4 * 1000 * per_mfma)
    with pytest.raises(gpu.AnnError):
        gpu.ann_probe_mfma(4, 1, 1)


def _probe_fragments(kind):
    """The probe's pseudo-random register fragments, recomputed: [thread 0..255][block 0..3][A|B][4 words]."""
    def mix(x):
        x = x.astype(np.uint64)
        x ^= x >> 16; x = (x * 0x7FEB352D) & 0xFFFFFFFF
        x ^= x >> 15; x = (x * 0x846CA68B) & 0xFFFFFFFF
        x ^= x >> 16
        return x.astype(np.uint32)
    t = np.arange(256, dtype=np.uint64)[:, None] * 64 + np.arange(32, dtype=np.uint64)[None, :] + 1
    h = mix(t & 0xFFFFFFFF)
    if kind == 3:
        h = (h & np.uint32(0x807F807F)) | np.uint32(0x3F803F80)
    return h.reshape(256, 4, 2, 4)


@pytest.mark.gpu
@pytest.mark.parametrize("kind", [2, 3])
def test_probe_mfma_random_fragments(gpu, kind):
    """Kinds 2 and 3 multiply pseudo-random fragments: the word each wavefront writes is iters x the
    sum of four entries of A_b B_b^T, recomputed here from the fragments (rows of A and B sit in lanes
    l % 32, the two halves of the k range in lanes < 32 and >= 32)."""
    step(f"probe mfma kind={kind}")
    iters = 3
    out = gpu.ann_probe_mfma(kind, 5, iters).cpu().numpy().reshape(5, 4)
    w = _probe_fragments(kind)
    if kind == 2:
        v = w.view(np.int8).reshape(256, 4, 2, 16).astype(np.int64)
    else:
        v = (w.view(np.uint16).astype(np.uint32) << 16).view(np.float32).reshape(256, 4, 2, 8).astype(np.float64)
    want = np.zeros(4)
    for wave in range(4):
        for b, m in enumerate((0, 9, 18, 27)):      # registers 0, 5, 10, 15 of lane 0: rows 0, 9, 18, 27, column 0
            for kh in range(2):
                want[wave] += np.dot(v[wave * 64 + m + 32 * kh, b, 0], v[wave * 64 + 0 + 32 * kh, b, 1])
    want *= iters
    for blk in range(5):
        if kind == 2:
            assert np.array_equal(out[blk], want.astype(np.float32)), (out[blk], want)
        else:
            assert np.allclose(out[blk], want, rtol=1e-5, atol=1e-4), (out[blk], want)


@pytest.mark.gpu
@pytest.mark.parametrize("d", [8, 96, 128, 960])
def test_binary16_storage(gpu, orc, d):
    """Rows stored as binary16 (a storage type of the search calls): distances are the canonical ones
    of the stored values, so every search agrees with the oracle run on the same binary16 rows."""
    step(f"binary16 rows d={d}")
    def make():
        base, queries = workloads.single_gaussian(3000, d, seed=300 + d, nq=64)
        h = base.astype(np.float16)
        adj, lam = orc.build_graph(h, 16)
        return h, queries, adj, lam
    h, queries, adj, lam = cached(f"f16_{d}", make)
    g = gpu.ann_graph_import(dev(adj), dev(lam), d)
    hb = torch.from_numpy(h).cuda()
    for mode in (1, 2):
        ids, s = gpu.ann_search_ex(g, hb, dev(queries), 10, 40, mode=mode, lambda_visit=10)
        ref = orc.search(adj, lam, h, queries, 10, 40, 10)
        assert compare_topk(ids.cpu().numpy(), s.cpu().numpy(), ref[0], ref[1], f"f16 d={d} mode={mode}") == 0
        assert_bitwise(s.cpu().numpy(), ref[1], f"f16 dists d={d}")
    ids, s = gpu.ann_search_multi(g, hb, dev(queries[:16]), 10, 4, max_hops=5)
    ref = orc.search_multi(adj, lam, h, queries[:16], 10, 4, max_hops=5)
    assert compare_topk(ids.cpu().numpy(), s.cpu().numpy(), ref[0], ref[1], "f16 multi") == 0
    ids, s = gpu.ann_search_alg2(g, hb, dev(queries[:16]), 16, 0.0)
    ref = orc.search_alg2(adj, lam, h, queries[:16], 16, 0.0)
    assert compare_topk(ids.cpu().numpy(), s.cpu().numpy(), ref[0], ref[1], "f16 alg2") == 0
    with pytest.raises(gpu.AnnError):      # not a type the build takes
        gpu.ann_build_graph_ex(hb, 8)


def test_automatic_mode_by_row_length(gpu, orc):
    """mode 0 picks the kernel from the batch size and the row length (thresholds measured per row length); whichever
    it picks, with the visited prefix given the ids are those of either explicit mode."""
    step("search: automatic batch regime")
    base, queries, adj, lam, _ = sift_case(orc)
    g = gpu.ann_graph_import(dev(adj), dev(lam), base.shape[1])
    b = dev(base)
    q = dev(np.tile(queries, (20, 1))[:5000])          # 5,000 queries: above the 4,096 of 512-byte rows
    ref = gpu.ann_search_ex(g, b, q, 10, 32, mode=1, lambda_visit=5)
    for nq in (5000, 4095, 300):
        ids, s = gpu.ann_search_ex(g, b, q[:nq].contiguous(), 10, 32, mode=0, lambda_visit=5)
        assert_bitwise(ids.cpu().numpy(), ref[0][:nq].cpu().numpy(), f"auto nq={nq}")
    b8 = dev(base.astype(np.uint8))                    # 128-byte rows: the change-over is at 1,024 queries
    ref8 = gpu.ann_search_ex(g, b8, q[:1500].contiguous(), 10, 32, mode=2, lambda_visit=5)
    ids, s = gpu.ann_search_ex(g, b8, q[:1500].contiguous(), 10, 32, mode=0, lambda_visit=5)
    assert_bitwise(ids.cpu().numpy(), ref8[0].cpu().numpy(), "auto uint8")
