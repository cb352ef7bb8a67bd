"""Every kernel of a call goes to the stream the caller names: the calls are issued on a side stream
while the default stream is kept busy, only the side stream is waited for, and the results must equal
those of the same calls on the default stream.  A kernel launched on the wrong stream would still be
queued behind the busy work when the results are read."""
import numpy as np
import pytest
import torch

from conftest import sift_case, step
from parity import assert_bitwise

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def test_calls_run_on_the_given_stream(gpu, orc):
    step("side stream: build, export, every search entry point")
    base, queries, adj, lam, _ = sift_case(orc)
    b, q = dev(base), dev(queries)
    # reference results on the default stream
    g0 = gpu.ann_build_graph_ex(b, 32)
    ref_graph = [t.cpu().numpy() for t in gpu.ann_graph_export(g0)]
    ref = {
        "large": gpu.ann_search_ex(g0, b, q, 10, 32, mode=1, lambda_visit=5),
        "small": gpu.ann_search_ex(g0, b, q[:16], 10, 64, mode=2, lambda_visit=10),
        "multi": gpu.ann_search_multi(g0, b, q[:16], 10, 8),
        "alg2": gpu.ann_search_alg2(g0, b, q, 16, 0.0),
        "knn": gpu.ann_knn(b[:5000].contiguous(), 16),
        "bf": gpu.ann_bruteforce(b, q[:64], 10),
    }
    ref = {k: [t.cpu().numpy() for t in v] for k, v in ref.items()}
    torch.cuda.synchronize()

    side = torch.cuda.Stream()
    # the calls that allocate and free temporaries (build, k-NN, brute force: freeing device memory waits for
    # the whole device) first, on the side stream with an idle default stream
    g1 = gpu.ann_build_graph_ex(b, 32, stream=side)
    got_graph = gpu.ann_graph_export(g1, stream=side)
    got = {
        "knn": gpu.ann_knn(b[:5000].contiguous(), 16, stream=side),
        "bf": gpu.ann_bruteforce(b, q[:64], 10, stream=side),
    }
    ws = torch.empty(gpu.ann_search_multi_workspace_bytes(16, 8), dtype=torch.uint8, device="cuda")  # the caller's workspace
    side.synchronize()
    # the search calls allocate nothing: they must run beside a busy default stream and finish before it
    outs = {k: [torch.empty(t.shape, dtype=torch.from_numpy(t).dtype, device="cuda") for t in ref[k]]
            for k in ("large", "small", "multi", "alg2")}
    q16 = q[:16].contiguous()
    busy = torch.randn(4096, 4096, device="cuda")
    torch.cuda.synchronize()
    for _ in range(1500):                      # a second or two of work queued on the default stream
        busy = torch.tanh(busy @ busy * 1e-3)
    gpu.ann_search_ex(g1, b, q, 10, 32, mode=1, lambda_visit=5, stream=side, out=tuple(outs["large"]))
    gpu.ann_search_ex(g1, b, q16, 10, 64, mode=2, lambda_visit=10, stream=side, out=tuple(outs["small"]))
    gpu.ann_search_multi(g1, b, q16, 10, 8, stream=side, out=tuple(outs["multi"]), workspace=ws)
    gpu.ann_search_alg2(g1, b, q, 16, 0.0, stream=side, out=tuple(outs["alg2"]))
    side.synchronize()                          # the default stream is NOT waited for
    default_still_busy = not torch.cuda.default_stream().query()
    got.update(outs)
    for a_, r_ in zip(got_graph, ref_graph):
        assert_bitwise(a_.cpu().numpy(), r_, "graph on the side stream")
    for k, v in got.items():
        for a_, r_ in zip(v, ref[k]):
            assert_bitwise(a_.cpu().numpy(), r_, f"{k} on the side stream")
    torch.cuda.synchronize()
    assert busy.isfinite().all()
    assert default_still_busy, "the default stream drained too early for this test to mean anything"
