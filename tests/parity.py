"""Comparison rules between the HIP path and the CPU oracle.

(b) result ids identical under the (distance, id) order, except where the
    competing distances differ by less than 1e-5 relative;
(c) returned fp32 distances within 1e-5 relative.
The HIP path accumulates in fp64 like the oracle, so in practice everything is
bit-identical; the excuse rule exists for the one-ulp case where two fp64 sums
taken in different orders round to different fp32 neighbours.
"""
import numpy as np

REL = 1e-5


def _close(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    both_inf = np.isinf(a) & np.isinf(b)
    with np.errstate(invalid="ignore"):
        ok = np.abs(a - b) <= REL * np.maximum(np.abs(a), np.abs(b))
    return ok | both_inf


def compare_topk(got_ids, got_s, ref_ids, ref_s, what=""):
    """Returns the number of excused positions; raises AssertionError on a real mismatch."""
    got_ids, ref_ids = np.asarray(got_ids), np.asarray(ref_ids)
    got_s, ref_s = np.asarray(got_s), np.asarray(ref_s)
    assert got_ids.shape == ref_ids.shape, f"{what}: shape {got_ids.shape} vs {ref_ids.shape}"
    close = _close(got_s, ref_s)
    assert close.all(), (f"{what}: distance mismatch at {np.argwhere(~close)[:5].tolist()} "
                         f"got {got_s[~close][:5]} want {ref_s[~close][:5]}")
    diff = got_ids != ref_ids
    if not diff.any():
        return 0
    # an id may differ only inside a run of near-equal distances, and the run must hold the same id set
    excused = 0
    for r in np.unique(np.argwhere(diff)[:, 0]):
        s = ref_s[r].astype(np.float64)
        for c in np.argwhere(diff[r])[:, 0]:
            lo = c
            while lo > 0 and _close(s[lo - 1], s[c]):
                lo -= 1
            hi = c
            while hi + 1 < len(s) and _close(s[hi + 1], s[c]):
                hi += 1
            same_set = sorted(got_ids[r, lo:hi + 1]) == sorted(ref_ids[r, lo:hi + 1])
            at_tail = hi == len(s) - 1          # a near-tie with the first entry that fell off the list
            assert hi > lo or at_tail, (f"{what}: row {r} col {c}: id {got_ids[r, c]} vs {ref_ids[r, c]} with a "
                                        f"clear distance gap ({got_s[r, c]} vs {ref_s[r, c]})")
            assert same_set or at_tail, f"{what}: row {r}: different ids in a near-tie run {lo}..{hi}"
            excused += 1
    return excused


def assert_bitwise(got, ref, what=""):
    got, ref = np.ascontiguousarray(got), np.ascontiguousarray(ref)
    assert got.shape == ref.shape and got.dtype == ref.dtype, f"{what}: {got.shape}/{got.dtype} vs {ref.shape}/{ref.dtype}"
    if got.tobytes() != ref.tobytes():
        bad = np.argwhere(got != ref)
        raise AssertionError(f"{what}: {len(bad)} entries differ, first at {bad[:5].tolist()}: "
                             f"{got[tuple(bad[0])]} vs {ref[tuple(bad[0])]}")
