"""Host-side checks of the benchmark's command line (no GPU needed)."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          timeout=120)


def test_more_than_one_gpu_is_refused_with_a_message():
    """Everything here runs on one GPU: --gpus above 1 must end with a message, not a number."""
    for n in ("2", "8"):
        r = _run("--gpus", n)
        assert r.returncode == 2
        assert "ONE GPU" in r.stderr + r.stdout
        assert not r.stdout.strip().startswith("{")      # no JSON line that could be taken for a result


def test_counter_summaries_name_what_they_were_taken_on():
    """bench.py takes `traffic` from a committed counter summary only when that summary was taken on the same
    workload, at the list length it times, and with the search kernel's present sources: each file must carry
    those lines in the form the parser reads."""
    for name in ("search_large_sift1m_pmc.txt", "search_large_sift4m_pmc.txt"):
        path = os.path.join(ROOT, "profiles", name)
        if not os.path.exists(path):
            continue
        text = open(path).read()
        for key in ("L", "N", "nq"):
            assert re.search(rf"^{key}: \d+$", text, re.M), (name, key)
        assert re.search(r"^kernel_source_sha256: [0-9a-f]{16}$", text, re.M), name
        m = re.search(r"^hbm_bytes_per_launch: (\d+)$", text, re.M)
        assert m and 1e9 < int(m.group(1)) < 1e10


def test_a_stale_counter_summary_is_not_quoted(tmp_path, monkeypatch):
    """A summary taken at another list length, on another workload, or before the kernel's sources changed
    yields no traffic figure, and the reason is said."""
    sys.path.insert(0, ROOT)
    import bench
    prof = tmp_path / "profiles"
    prof.mkdir()
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    monkeypatch.setattr(bench, "kernel_source_sha256", lambda: "0123456789abcdef")
    body = "L: 29\nN: 1000000\nnq: 10000\nhbm_bytes_per_launch: 4200000000\nkernel_source_sha256: {}\n"
    (prof / "x.txt").write_text(body.format("0123456789abcdef"))
    assert bench.profile_traffic("x.txt", 29, 1_000_000, 10_000)[0] == 4_200_000_000
    assert bench.profile_traffic("x.txt", 30, 1_000_000, 10_000)[0] is None
    assert bench.profile_traffic("x.txt", 29, 2_000_000, 10_000)[0] is None
    (prof / "x.txt").write_text(body.format("ffffffffffffffff"))
    got, why = bench.profile_traffic("x.txt", 29, 1_000_000, 10_000)
    assert got is None and "stale" in why
    assert bench.profile_traffic("missing.txt", 29, 1_000_000, 10_000)[0] is None
