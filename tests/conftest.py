import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def orc():
    """The CPU oracle (compiled on first use)."""
    import oracle
    oracle.lib()
    return oracle


def step(msg: str) -> None:
    """Names the GPU case about to run: printed unbuffered and, when TSDG_STEP_LOG names a
    file, appended to it, so that a run that dies still says where it was."""
    line = f"[step] {msg}"
    print(line, file=sys.stderr, flush=True)
    path = os.environ.get("TSDG_STEP_LOG")
    if not path:
        return
    try:
        os.makedirs(os.path.dirname(os.path.abspath(path)), exist_ok=True)
        with open(path, "a") as f:
            f.write(line + "\n")
            f.flush()
            os.fsync(f.fileno())
    except OSError:
        pass


@pytest.fixture(scope="session")
def gpu():
    """torch + the HIP library on cuda:0; fails loudly when either is missing."""
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2204_00824_amd as P
    P.load_library()
    return P


_cache = {}


def cached(key, fn):
    if key not in _cache:
        _cache[key] = fn()
    return _cache[key]


def tiny_case(orc):
    """Tiny workload + oracle graph (K=16) with the intermediate stages."""
    def make():
        import workloads
        base, queries = workloads.tiny()
        adj, lam, st = orc.build_graph(base, 16, stages=True)
        return base, queries, adj, lam, st
    return cached("tiny", make)


def sift_case(orc):
    """20,000 integer-valued rows of d=128 + oracle graph (K=32) with the intermediate stages."""
    def make():
        import workloads
        base, queries = workloads.sift_like(N=20000, nq=300, seed=77)
        adj, lam, st = orc.build_graph(base, 32, stages=True)
        return base, queries, adj, lam, st
    return cached("sift20k", make)
