#!/usr/bin/env python3
"""Measurements on the other workload shapes (one MI355X): gist-like 1M x 960,
deep-like 10M x 96, glove-like 1M x 100 under the cosine metric, and the 100M x 128 uint8 set.  bench.py stays the headline
(sift-like 1M x 128); this script prints one JSON line per run with the same
kind of fields.  Long builds print progress (the build calls get a progress callback).

The 100M set cannot get an exact k-NN graph in one session (2.6e18 flop), so it
is built as 25 independent blocks of 4M rows, each an exact TSDG of its block,
and a query is answered by searching every block and merging the per-block
top-k by (distance, id): the form a base set split over several devices would
also take.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def log(msg):
    print(f"[bench_configs] {msg}", file=sys.stderr, flush=True)


def progress(step, done, total):
    """Progress callback of the long builds: one line per finished chunk / iteration."""
    print(f"[tsdg] {step}: {done} / {total}", file=sys.stderr, flush=True)


def recall(found, gt):
    return float((found[:, :, None] == gt[:, None, :]).any(axis=2).sum()) / gt.size


def timed_search(fn, reps=3):
    import torch
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def run_single_graph(args, name, base_h, queries_h, ks, Ls, metric="l2"):
    import torch
    import paper_2204_00824_amd as P
    K = 32
    base = torch.from_numpy(base_h).cuda()
    queries = torch.from_numpy(queries_h).cuda()
    N, d = base.shape
    nq = queries.shape[0]
    if metric == "cosine":      # unit rows, once; ground truth by squared L2 of unit rows = the 1 - cos order
        P.ann_normalize_rows(base, out=base)
        P.ann_normalize_rows(queries, out=queries)
    t0 = time.time()
    graph = P.ann_build_graph_ex(base, K, metric=metric, progress=progress)
    torch.cuda.synchronize()
    build_s = time.time() - t0
    log(f"{name}: build {build_s:.1f}s")
    adj, _ = P.ann_graph_export(graph)
    deg = (adj >= 0).sum(dim=1).float().mean().item()
    del adj
    out = {"workload": name, "metric": metric, "N": N, "d": d, "nq": nq, "K": K, "build_seconds": round(build_s, 2),
           "knn_tflops": round(2.0 * N * N * d / build_s / 1e12, 1), "avg_degree": round(deg, 2), "curves": {}}
    for k in ks:
        gt, _ = P.ann_bruteforce(base, queries, k)
        gt_h = gt.cpu().numpy()
        for mode, lv in ((1, 5), (2, 10)):
            rows = []
            for L in Ls:
                if L < k:
                    continue
                ids, s, st = P.ann_search_ex(graph, base, queries, k, L, mode=mode, lambda_visit=lv, want_stats=True, metric=metric)
                ms = timed_search(lambda: P.ann_search_ex(graph, base, queries, k, L, mode=mode, lambda_visit=lv, out=(ids, s), metric=metric))
                ev = st.dist_evals.double().mean().item()
                hp = st.hops.double().mean().item()
                alg = (ev * d * base.element_size() + hp * K * 4) * nq
                rows.append({"L": L, f"recall@{k}": round(recall(ids.cpu().numpy(), gt_h), 4), "qps": round(nq / ms * 1e3),
                             "ms": round(ms, 3), "dist_evals": round(ev, 1), "alg_TBps": round(alg / ms / 1e9, 2)})
                log(f"{name} k={k} mode={mode}: {rows[-1]}")
            out["curves"][f"k{k}_mode{mode}_lambda{lv}"] = rows
    if base.dtype == torch.float32 and metric == "l2":
        # the same graph searched over rows stored as binary16 (half the bytes per evaluation); recall
        # still against the fp32 ground truth
        k = ks[0]
        gt_h = P.ann_bruteforce(base, queries, k)[0].cpu().numpy()
        half = base.to(torch.float16)
        rows = []
        for L in Ls:
            if L < k:
                continue
            ids, s, st = P.ann_search_ex(graph, half, queries, k, L, mode=1, lambda_visit=5, want_stats=True)
            ms = timed_search(lambda: P.ann_search_ex(graph, half, queries, k, L, mode=1, lambda_visit=5, out=(ids, s)))
            ev, hp = st.dist_evals.double().mean().item(), st.hops.double().mean().item()
            rows.append({"L": L, f"recall@{k}": round(recall(ids.cpu().numpy(), gt_h), 4), "qps": round(nq / ms * 1e3),
                         "ms": round(ms, 3), "alg_TBps": round((ev * d * 2 + hp * K * 4) * nq / ms / 1e9, 2)})
            log(f"{name} binary16 storage k={k}: {rows[-1]}")
        out["curves"][f"k{k}_mode1_lambda5_binary16_storage"] = rows
    print(json.dumps(out), flush=True)


def run_sharded_u8(args):
    import torch
    import workloads
    import paper_2204_00824_amd as P
    N, d, K, k, block = args.n or 100_000_000, 128, 32, 10, 4_000_000
    nq = 10_000
    _, queries = next(workloads.scale_u8_torch(N=N, nq=nq))
    shards = []
    t_build = 0.0
    t0 = time.time()
    for lo, x in workloads.scale_u8_torch(N=N, chunk=block):
        torch.cuda.synchronize()
        t1 = time.time()
        g = P.ann_build_graph_ex(x, K, progress=progress)
        torch.cuda.synchronize()
        t_build += time.time() - t1
        shards.append((lo, x, g))
        log(f"block at {lo}: {x.shape[0]} rows, build total {t_build:.1f}s, wall {time.time() - t0:.1f}s")
    # ground truth: exact top-k per block (ann_bruteforce), merged by (distance, id)
    def merge(parts_ids, parts_s):
        ids = torch.cat(parts_ids, dim=1).long()
        s = torch.cat(parts_s, dim=1)
        key = (s.view(torch.int32).long() << 32) | ids.clamp(min=0)
        key = torch.where(ids < 0, torch.full_like(key, 2 ** 62), key)
        order = torch.sort(key, dim=1).indices[:, :k]
        return torch.gather(ids, 1, order), torch.gather(s, 1, order)
    gi, gs = [], []
    for lo, x, g in shards:
        i, s = P.ann_bruteforce(x, queries, k)
        gi.append(i + lo)
        gs.append(s)
    gt_h = merge(gi, gs)[0].cpu().numpy()
    log("ground truth done")
    out = {"workload": f"scale N={N} d={d} uint8, {len(shards)} blocks of {block}, sharded search", "nq": nq, "K": K,
           "build_seconds": round(t_build, 1),
           "knn_tflops": round(sum(2.0 * x.shape[0] ** 2 * d for _, x, _ in shards) / t_build / 1e12, 1), "curves": {}}

    def search_all(q, L, mode, lv, qi_offset=0):
        pi, ps = [], []
        for lo, x, g in shards:
            i, s = P.ann_search_ex(g, x, q, k, L, mode=mode, lambda_visit=lv, qi_offset=qi_offset)
            pi.append(torch.where(i >= 0, i + lo, i))
            ps.append(s)
        return merge(pi, ps)

    rows = []
    for L in (16, 32, 64, 128, 256):
        ids, _ = search_all(queries, L, 1, 5)
        ms = timed_search(lambda: search_all(queries, L, 1, 5), reps=2)
        rows.append({"L": L, "recall@10": round(recall(ids.cpu().numpy(), gt_h), 4), "qps": round(nq / ms * 1e3), "ms": round(ms, 2)})
        log(f"sharded large batch: {rows[-1]}")
    out["curves"]["large_batch_lambda5"] = rows
    for bs in (1, 16):
        rows = []
        for L in (32, 64):
            lat, hit = [], 0
            for c in range(30):
                q = queries[c * bs:(c + 1) * bs].contiguous()
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                ids, _ = search_all(q, L, 2, 10, qi_offset=c * bs)
                torch.cuda.synchronize()
                lat.append(time.perf_counter() - t1)
                hit += recall(ids.cpu().numpy(), gt_h[c * bs:(c + 1) * bs]) * bs
            rows.append({"L": L, "recall@10": round(hit / (30 * bs), 4), "median_latency_ms": round(float(np.median(lat)) * 1e3, 3)})
            log(f"sharded batch {bs}: {rows[-1]}")
        out["curves"][f"batch{bs}_lambda10"] = rows
    print(json.dumps(out), flush=True)


def run_whole_u8(args):
    """The 100M x 128 uint8 set as ONE graph: k-NN lists by neighbourhood propagation (O(N) work per
    iteration instead of the exact build's N^2), then the same two-stage diversification."""
    import torch
    import workloads
    import paper_2204_00824_amd as P
    N, d, K, k = args.n or 100_000_000, 128, 32, 10
    nq = 10_000
    _, queries = next(workloads.scale_u8_torch(N=N, nq=nq))
    base = torch.empty((N, d), dtype=torch.uint8, device="cuda")
    for lo, x in workloads.scale_u8_torch(N=N, chunk=4_000_000):
        base[lo:lo + x.shape[0]] = x
    torch.cuda.synchronize()
    log(f"generated {N} rows")
    t0 = time.time()
    ids, _, done, last = P.ann_knn_descent(base, K, S=16, max_iters=args.iters, delta=0.001, seed=0)
    torch.cuda.synchronize()
    knn_s = time.time() - t0
    log(f"neighbourhood propagation alone: {done} iterations, {last} entries changed in the last, {knn_s:.1f}s")
    # quality of the lists on a sample of rows against the exact lists
    sample = torch.arange(0, N, max(1, N // 2000), device="cuda")[:2000]
    ex, _ = P.ann_bruteforce(base, base[sample].to(torch.float32), K + 1)
    ex = ex[:, 1:]                                            # the row itself comes first
    list_recall = (ids[sample.long()].unsqueeze(2) == ex.unsqueeze(1)).any(dim=2).float().mean().item()
    del ids, ex
    torch.cuda.empty_cache()                                  # the library allocates outside torch's cache
    t0 = time.time()
    graph = P.ann_build_graph_ex(base, K, knn_mode=1, descent_iters=args.iters, progress=progress)
    torch.cuda.synchronize()
    build_s = time.time() - t0
    log(f"whole build (propagation + diversification): {build_s:.1f}s; list recall on 2000 rows {list_recall:.4f}")
    gt, _ = P.ann_bruteforce(base, queries, k)
    gt_h = gt.cpu().numpy()
    log("ground truth done")
    out = {"workload": f"scale N={N} d={d} uint8, one graph from neighbourhood propagation (S=16)", "nq": nq, "K": K,
           "knn_seconds": round(knn_s, 1), "knn_iterations": done, "knn_list_recall_on_2000_rows": round(list_recall, 4),
           "build_seconds": round(build_s, 1), "curves": {}}
    rows = []
    for L in (16, 32, 64, 128, 256):
        ids, s, st = P.ann_search_ex(graph, base, queries, k, L, mode=1, lambda_visit=5, want_stats=True)
        ms = timed_search(lambda: P.ann_search_ex(graph, base, queries, k, L, mode=1, lambda_visit=5, out=(ids, s)))
        ev, hp = st.dist_evals.double().mean().item(), st.hops.double().mean().item()
        rows.append({"L": L, "recall@10": round(recall(ids.cpu().numpy(), gt_h), 4), "qps": round(nq / ms * 1e3),
                     "ms": round(ms, 3), "dist_evals": round(ev, 1), "alg_TBps": round((ev * d + hp * K * 4) * nq / ms / 1e9, 2)})
        log(f"large batch: {rows[-1]}")
    out["curves"]["large_batch_lambda5"] = rows
    # small batches (1 and 16 queries per call): Alg. 1's multi-search and the best-first search
    for bs in (1, 16):
        rows = []
        ws = torch.empty(P.ann_search_multi_workspace_bytes(bs, 128), dtype=torch.uint8, device="cuda")
        for t0_ in (32, 64, 128):
            lat, hit = [], 0
            for c in range(50):
                q = queries[c * bs:(c + 1) * bs].contiguous()
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                ids, _ = P.ann_search_multi(graph, base, q, k, t0_, max_hops=8, qi_offset=c * bs, workspace=ws)
                torch.cuda.synchronize()
                lat.append(time.perf_counter() - t1)
                hit += recall(ids.cpu().numpy(), gt_h[c * bs:(c + 1) * bs])
            rows.append({"t0": t0_, "T": 8, "recall@10": round(hit / 50, 4), "median_latency_ms": round(float(np.median(lat)) * 1e3, 3)})
            log(f"batch {bs} multi-search: {rows[-1]}")
        out["curves"][f"batch{bs}_multi_search"] = rows
        rows = []
        for L in (64, 128, 256):
            lat, hit = [], 0
            for c in range(50):
                q = queries[c * bs:(c + 1) * bs].contiguous()
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                ids, _ = P.ann_search_ex(graph, base, q, k, L, mode=2, lambda_visit=10, qi_offset=c * bs)
                torch.cuda.synchronize()
                lat.append(time.perf_counter() - t1)
                hit += recall(ids.cpu().numpy(), gt_h[c * bs:(c + 1) * bs])
            rows.append({"L": L, "recall@10": round(hit / 50, 4), "median_latency_ms": round(float(np.median(lat)) * 1e3, 3)})
            log(f"batch {bs} best-first: {rows[-1]}")
        out["curves"][f"batch{bs}_best_first"] = rows
    print(json.dumps(out), flush=True)


def run_descent_1m(args):
    """The neighbourhood-propagation builder alone on the headline set (fp32 rows and the same rows as uint8)."""
    import torch
    import workloads
    import paper_2204_00824_amd as P
    N, K = args.n or 1_000_000, 32
    base = torch.from_numpy(workloads.sift_like(N=N, nq=16)[0]).cuda()
    exact = P.ann_knn(base, K)[0][:20000]
    out = {"workload": f"sift-like N={N} d=128, K={K}, S=16, delta=0.001", "runs": []}
    for x, name in ((base, "fp32"), (base.to(torch.uint8), "uint8")):
        for rep in range(2):
            torch.cuda.synchronize()
            t0 = time.time()
            ids, _, done, last = P.ann_knn_descent(x, K, S=16, max_iters=12, delta=0.001, seed=1)
            torch.cuda.synchronize()
            dt = time.time() - t0
        rec = (ids[:20000].unsqueeze(2) == exact.unsqueeze(1)).any(dim=2).float().mean().item()
        out["runs"].append({"rows": name, "seconds": round(dt, 3), "iterations": done, "last_changed": last,
                            "list_recall_on_20000_rows": round(rec, 4)})
        log(str(out["runs"][-1]))
    print(json.dumps(out), flush=True)


def run_crossover(args):
    """Where the workgroup-per-query kernel (mode 2) stops paying and the wave-per-query kernel (mode 1) takes over, by
    row shape: queries/s of both at the same L and lambda prefix (so both return the same ids) over batch sizes 1..8192.
    Sec. 4 says the division depends on the device and on d; api.hip's automatic mode takes its thresholds from this."""
    import torch
    import workloads
    import paper_2204_00824_amd as P
    K, k, L = 32, 10, 64
    out = {"workload": "small/large batch crossover", "K": K, "k": k, "L": L, "lambda_visit": 5, "shapes": []}
    shapes = (("deep-like d=96 fp32 (384 B rows)", lambda: workloads.deep_like(N=args.n or 1_000_000, nq=8192), None),
              ("sift-like d=128 fp32 (512 B rows)", lambda: workloads.sift_like(N=args.n or 1_000_000, nq=8192), None),
              ("sift-like d=128 uint8 (128 B rows)", lambda: workloads.sift_like(N=args.n or 1_000_000, nq=8192), "u8"),
              ("gist-like d=960 fp32 (3840 B rows)", lambda: workloads.gist_like(N=args.n or 250_000, nq=8192), None))
    for name, make, cast in shapes:
        base_h, q_h = make()
        base = torch.from_numpy(base_h).cuda()
        if cast == "u8":
            base = base.to(torch.uint8)
        queries = torch.from_numpy(q_h).cuda()
        graph = P.ann_build_graph_ex(base, K, progress=progress)
        rows = []
        for bs in (1, 16, 64, 128, 256, 512, 1024, 2048, 4096, 8192):
            q = queries[:bs].contiguous()
            o = (torch.empty((bs, k), dtype=torch.int32, device="cuda"), torch.empty((bs, k), dtype=torch.float32, device="cuda"))
            row = {"batch": bs}
            for label, kw in (("wave_per_query", dict(mode=1)), ("workgroup_2_waves", dict(mode=2, waves_per_query=2)),
                              ("workgroup_4_waves", dict(mode=2, waves_per_query=4)), ("workgroup_8_waves", dict(mode=2, waves_per_query=8))):
                ms = timed_search(lambda: P.ann_search_ex(graph, base, q, k, L, lambda_visit=5, out=o, **kw), reps=10)
                row[label + "_qps"] = round(bs / ms * 1e3)
            best = max((v, n) for n, v in row.items() if n.endswith("_qps"))
            row["fastest"] = best[1][:-4]
            rows.append(row)
            log(f"{name}: {row}")
        out["shapes"].append({"rows": name, "N": base.shape[0], "table": rows})
        del base, queries, graph
        torch.cuda.empty_cache()
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", required=True, choices=["gist1m", "gist1m_latent", "deep10m", "scale100m", "scale100m_one_graph", "glove1m", "descent1m", "crossover"])
    ap.add_argument("--n", type=int, default=0, help="override the number of base rows")
    ap.add_argument("--iters", type=int, default=20, help="scale100m_one_graph: most iterations of the propagation")
    args = ap.parse_args()
    import workloads
    if args.workload == "gist1m":
        base, q = workloads.gist_like(N=args.n or 1_000_000)
        run_single_graph(args, "gist-like", base, q, (10,), (32, 64, 128, 256, 512))
    elif args.workload == "gist1m_latent":
        base, q = workloads.gist_like_latent(N=args.n or 1_000_000)
        run_single_graph(args, "gist-shaped, latent-factor recipe (ours)", base, q, (10,), (32, 64, 128, 256, 512))
    elif args.workload == "deep10m":
        base, q = workloads.deep_like(N=args.n or 10_000_000)
        run_single_graph(args, "deep-like", base, q, (10, 100), (64, 128, 256, 512))
    elif args.workload == "glove1m":
        base, q = workloads.glove_like(N=args.n or 1_000_000)
        run_single_graph(args, "glove-like, cosine", base, q, (10,), (32, 64, 128, 256, 512), metric="cosine")
    elif args.workload == "scale100m_one_graph":
        run_whole_u8(args)
    elif args.workload == "descent1m":
        run_descent_1m(args)
    elif args.workload == "crossover":
        run_crossover(args)
    else:
        run_sharded_u8(args)


if __name__ == "__main__":
    main()
