"""The search calls allocate nothing and enqueue only kernels, so a caller may record them into a HIP graph:
the replays, with new queries written into the same input buffer between them and eager work in between,
must equal the eager calls."""
import numpy as np
import pytest
import torch

from conftest import sift_case, step
from parity import assert_bitwise

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("entry", ["best_first_small", "best_first_large", "multi", "multi_static", "alg2"])
def test_replays_equal_eager_calls(gpu, orc, entry):
    step(f"graph capture: {entry}")
    base, queries, adj, lam, _ = sift_case(orc)
    b = dev(base)
    g = gpu.ann_graph_import(dev(adj), dev(lam), base.shape[1])
    nq = {"best_first_small": 4, "best_first_large": 64, "multi": 4, "multi_static": 4, "alg2": 64}[entry]
    q_all = dev(queries)
    ws = torch.empty(gpu.ann_search_multi_workspace_bytes(nq, 8), dtype=torch.uint8, device="cuda")   # outside the capture

    def call(qbuf, out):
        if entry == "best_first_small":
            gpu.ann_search_ex(g, b, qbuf, 10, 32, mode=2, lambda_visit=10, out=out)
        elif entry == "best_first_large":
            gpu.ann_search_ex(g, b, qbuf, 10, 48, mode=1, lambda_visit=5, out=out)
        elif entry == "multi":
            gpu.ann_search_multi(g, b, qbuf, 10, 8, out=out, workspace=ws)
        elif entry == "multi_static":
            gpu.ann_search_multi_static(g, b, qbuf, 10, 8, out=out)
        else:
            gpu.ann_search_alg2(g, b, qbuf, 16, 0.0, out=out)

    k = 16 if entry == "alg2" else 10
    qbuf = q_all[:nq].clone()
    out = (torch.empty((nq, k), dtype=torch.int32, device="cuda"), torch.empty((nq, k), dtype=torch.float32, device="cuda"))
    call(qbuf, out)                               # eager warm-up (the static scratch's address is looked up here)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call(qbuf, out)
    for rep in range(4):
        lo = (rep * nq) % (q_all.shape[0] - nq)
        qbuf.copy_(q_all[lo:lo + nq])
        graph.replay()
        torch.cuda.synchronize()
        got = (out[0].cpu().numpy().copy(), out[1].cpu().numpy().copy())
        ref = (torch.empty_like(out[0]), torch.empty_like(out[1]))
        call(q_all[lo:lo + nq].contiguous(), ref)     # eager, between the replays
        torch.cuda.synchronize()
        assert_bitwise(got[0], ref[0].cpu().numpy(), f"{entry} replay {rep} ids")
        assert_bitwise(got[1], ref[1].cpu().numpy(), f"{entry} replay {rep} dists")
