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


def test_profile_of_the_timed_launch_names_its_list_length():
    """bench.py takes `traffic` from the committed counter summary only when that summary was taken at the list
    length it times: the file must carry both lines in the form the parser reads."""
    text = open(os.path.join(ROOT, "profiles", "search_large_sift1m_pmc.txt")).read()
    assert re.search(r"^L: \d+$", text, re.M)
    m = re.search(r"^hbm_bytes_per_launch: (\d+)$", text, re.M)
    assert m and 1e9 < int(m.group(1)) < 1e10
