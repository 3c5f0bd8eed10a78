#!/usr/bin/env python3
"""Benchmark of the whole kNN-graph construction path on one MI355X.

One step = efanna_build_trees + efanna_init_graph + efanna_nndescent(I) +
efanna_get_graph on a synthetic workload already resident in HBM.  Prints ONE JSON
line: build seconds per step, distance evaluations per second, recall@K, the roofline
of the dominant kernel (the NN-descent local join) and the CPU oracle timed on a
bounded prefix of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))

HBM_PEAK_GBS = 8000.0

# HBM bytes per launch of the dominant kernel, from two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE)
# scaled by what the same counters read for a plain 256 MiB copy (factors 2.0 and 1.0); summary and
# commands in profiles/join_kernels_sift1m_like_hbm_traffic.txt.  Only measured for the headline workload.
MEASURED_TRAFFIC_BYTES = {"sift1m_like": {"calibrated": 4.85e9, "raw_counters": 2.53e9}}


def exact_knn_torch(Xd, rows, K):
    """Ground truth for recall on the sampled rows: float64 brute force with torch
    (measurement infrastructure, outside the timed region and outside the library)."""
    import torch
    X64 = Xd.double()
    norms = (X64 * X64).sum(1)
    out = []
    for r0 in range(0, rows.shape[0], 250):
        rr = rows[r0:r0 + 250]
        G = X64[rr] @ X64.T
        G.mul_(-2.0).add_(norms[None, :]).add_(norms[rr][:, None])
        G[torch.arange(rr.shape[0], device=G.device), rr] = float("inf")
        out.append(torch.topk(G, K, dim=1, largest=False).indices)
    return torch.cat(out).cpu().numpy()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="sift1m_like")
    ap.add_argument("--n", type=int, default=None, help="use only the first n rows of the workload")
    ap.add_argument("--cpu-rows", type=int, default=1_000_000,
                    help="rows of the workload the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--recall-rows", type=int, default=10_000, help="0 = skip recall")
    ap.add_argument("--progress", action="store_true", help="report each phase on stderr as it ends")
    ap.add_argument("--calibrate", action="store_true",
                    help="after the timed steps, fill 256 MiB and add a constant to 256 MiB with plain torch kernels: a known "
                         "amount of HBM traffic to scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters by")
    ap.add_argument("--search", type=int, default=0, metavar="NQ",
                    help="after the build, answer NQ synthetic queries with the index (Alg. 1) and add a "
                         "`search` object to the line: queries per second, recall against brute force")
    ap.add_argument("--search-pool", type=int, default=200, help="candidate pool size P of the search")
    ap.add_argument("--search-expand", type=int, default=50, help="expansion factor E of the search")
    ap.add_argument("--search-iters", type=int, default=4, help="NN-expansion rounds I of the search")
    ap.add_argument("--ablation-init", type=int, default=0, metavar="ITERS",
                    help="after the build, run NN-descent one iteration at a time for ITERS iterations from "
                         "the tree-built initial graph and from a seeded random graph (the starting point of "
                         "plain NN-descent) and add an `ablation_init` object: time and recall after every "
                         "iteration of both")
    ap.add_argument("--conquer-depth", type=int, default=None,
                    help="walk the conquer step of Alg. 3 up to this depth (default: stop at the leaves, "
                         "the configuration the metric is quoted on); distance evaluations above the "
                         "leaves are not counted in `value`")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus N with N > 1 is not supported "
              "(no collectives, no sharding in this library)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1609_07228_amd import efanna, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU fallback", file=sys.stderr)
        sys.exit(3)
    efanna.lib()
    name = args.workload
    p = synth.params(name)
    X = synth.generate(name, n=args.n)
    n, d = X.shape
    if args.progress:
        print(f"generated {name}: {n} x {d}", file=sys.stderr, flush=True)
    K, T, S, I, L = p["K"], p["T"], p["S"], p["I"], p["L"]
    dev = torch.device("cuda:0")
    Xd = torch.from_numpy(X).to(dev)
    L_ = efanna.lib()
    conquer = args.conquer_depth is not None
    ws_tree = torch.empty(L_.efanna_trees_workspace_bytes(n, d, T, S, 1 if conquer else 0),
                          dtype=torch.uint8, device=dev)
    ws_init = torch.empty(max(256, L_.efanna_init_workspace_bytes(n, 64 if conquer else 0)),
                          dtype=torch.uint8, device=dev)
    ws_nnd = torch.empty(L_.efanna_nndescent_workspace_bytes(n, K, L), dtype=torch.uint8, device=dev)
    graph = torch.empty((n, K), dtype=torch.int64, device=dev)
    stats = torch.zeros((I, 4), dtype=torch.int64, device=dev)
    phase_ms = np.zeros((I, 4), dtype=np.float32)
    max_leaves = n // max(1, S // 4) + 16      # generous: mean splits leave leaves ~0.7*S full
    state = {}
    phases = np.zeros(4)
    # dominant kernel: the join of points that gather at most 16 vectors (one launch per iteration)
    k_ms_sum, k_bytes_sum, k_launches = 0.0, 0.0, 0
    all_ms_sum, all_bytes_sum = 0.0, 0.0

    # Phase times come from events on the launch stream, read after the timed region: a step has
    # no host synchronisation of its own (the tree build reads its level counters and the phase
    # timing of efanna_nndescent waits for the stream; both are part of the library calls).
    step_events = []

    def step(timed: bool):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(5)]
        ev[0].record()
        trees = efanna.efanna_build_trees(Xd, T, S, synth.ALGO_SEED, max_leaves=max_leaves,
                                          workspace=ws_tree, with_nodes=conquer)
        perm, leaf_off, n_leaves = trees[:3]
        ev[1].record()
        if conquer:
            efanna.efanna_init_graph(Xd, perm, leaf_off, n_leaves, S, K, graph=graph, workspace=ws_init,
                                     nodes=trees[3], leaf_up=trees[4], tree_depth=trees[5],
                                     conquer_depth=args.conquer_depth)
        else:
            efanna.efanna_init_graph(Xd, perm, leaf_off, n_leaves, S, K, graph=graph, workspace=ws_init)
        ev[2].record()
        efanna.efanna_nndescent(Xd, graph, I, L, synth.ALGO_SEED, stats=stats, workspace=ws_nnd,
                                phase_ms=phase_ms)
        ev[3].record()
        ids, dists = efanna.efanna_get_graph(graph)
        ev[4].record()
        if args.progress:
            torch.cuda.synchronize()
            print("step: trees %.3f ms, init %.3f ms, nndescent %.3f ms, get %.3f ms"
                  % tuple(ev[k].elapsed_time(ev[k + 1]) for k in range(4)), file=sys.stderr, flush=True)
        if timed:
            step_events.append(ev)
            step_phase_ms.append(phase_ms.copy())      # host memory, filled by the call above
        state.update(perm=perm, leaf_off=leaf_off, n_leaves=n_leaves, ids=ids, dists=dists)

    step_phase_ms = []
    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    seconds = (time.perf_counter() - t_begin) / max(1, args.steps)
    for ev in step_events:
        phases[:] += [ev[k].elapsed_time(ev[k + 1]) * 1e-3 for k in range(4)]
    st_steps = stats.cpu().numpy()      # the path is deterministic: the same in every step
    for pm in step_phase_ms:
        k_ms_sum += float(pm[:, 1].sum())
        k_bytes_sum += float((st_steps[:, 3] * (d * 4 + 8)).sum())
        k_launches += I
        all_ms_sum += float(pm[:, 1:].sum())
        all_bytes_sum += float((st_steps[:, 2] * (d * 4 + 8) + st_steps[:, 1] * 8).sum())

    if args.calibrate:
        a = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        a.fill_(1.0)
        torch.cuda.synchronize()
        torch.add(a, 1.0, out=b)      # an elementwise kernel (a plain copy may go to a DMA engine instead)
        torch.cuda.synchronize()
        del a, b

    # work done per step (identical in every step: the path is deterministic)
    st = stats.cpu().numpy()
    off = state["leaf_off"].cpu().numpy().astype(np.int64)
    init_evals = 0
    for t in range(T):
        sizes = np.diff(off[t, :state["n_leaves"][t] + 1])
        init_evals += int((sizes * (sizes - 1) // 2).sum())
    evals = init_evals + int(st[:, 0].sum())

    recall = None
    if args.recall_rows > 0:
        rows = synth.sample_rows(n, args.recall_rows)
        truth = exact_knn_torch(Xd, torch.from_numpy(rows).to(dev), K)
        got = state["ids"][torch.from_numpy(rows).to(dev)].cpu().numpy()
        hits = sum(np.intersect1d(a[a >= 0], b).shape[0] for a, b in zip(got, truth))
        recall = hits / float(truth.size)

    cpu = None
    if args.cpu_rows > 0:
        import oracle
        m = min(n, args.cpu_rows)
        Xs = X[:m]
        c0 = time.perf_counter()
        operm, ooff, onl = oracle.build_trees(Xs, T, S, synth.ALGO_SEED)
        g = oracle.init_graph(Xs, operm, ooff, onl, K)
        g = oracle.nndescent(Xs, *g, I, L, synth.ALGO_SEED)
        c_sec = time.perf_counter() - c0
        c_evals = int(g[3][:, 0].sum())
        for t in range(T):
            sizes = np.diff(ooff[t, :onl[t] + 1]).astype(np.int64)
            c_evals += int((sizes * (sizes - 1) // 2).sum())
        cpu = {"value": c_evals / c_sec, "unit": "distance evals/s", "cores": oracle.num_threads(),
               "kind": "oracle", "seconds": c_sec,
               "sample": f"whole path (trees, leaf init, {I} NN-descent iterations) on the first "
                         f"{m} rows of {name}"}

    search = None
    if args.search > 0:
        # the index of the last step, with the trees built once more to get their nodes
        Q = torch.from_numpy(synth.generate_queries(name, args.search)).to(dev)
        trees = efanna.efanna_build_trees(Xd, T, S, synth.ALGO_SEED, max_leaves=max_leaves, with_nodes=True)
        gids = state["ids"]
        for _ in range(2):      # the first call warms up
            torch.cuda.synchronize()
            s0 = time.perf_counter()
            sid, sdist, schk = efanna.efanna_search(Xd, trees[0], trees[1], trees[2], trees[3], trees[5], S,
                                                    gids, Q, K, args.search_pool, args.search_expand,
                                                    args.search_iters)
            torch.cuda.synchronize()
            s_sec = time.perf_counter() - s0
        truth_q = []
        Q64, X64 = Q.double(), Xd.double()
        xn = (X64 * X64).sum(1)
        for r0 in range(0, args.search, 250):
            G = Q64[r0:r0 + 250] @ X64.T
            G.mul_(-2.0).add_(xn[None, :])
            truth_q.append(torch.topk(G, K, dim=1, largest=False).indices)
        truth_q = torch.cat(truth_q).cpu().numpy()
        got_q = sid.cpu().numpy()
        hits_q = sum(np.intersect1d(a[a >= 0], b).shape[0] for a, b in zip(got_q, truth_q))
        search = {"queries": args.search, "queries_per_s": args.search / s_sec, "ms": s_sec * 1e3,
                  "recall_at_K": hits_q / float(truth_q.size), "K": K, "pool": args.search_pool,
                  "expand": args.search_expand, "iters": args.search_iters,
                  "mean_points_checked": float(schk.float().mean().item())}

    ablation = None
    if args.ablation_init > 0:
        rows = synth.sample_rows(n, max(1000, args.recall_rows))
        rows_d = torch.from_numpy(rows).to(dev)
        truth_a = exact_knn_torch(Xd, rows_d, K)

        def recall_of(g):
            got = efanna.efanna_get_graph(g)[0][rows_d].cpu().numpy()
            return sum(np.intersect1d(a[a >= 0], b).shape[0] for a, b in zip(got, truth_a)) / float(truth_a.size)

        def descend(g, start_ms):
            curve, ms = [{"iterations": 0, "ms": start_ms, "recall_at_K": recall_of(g)}], start_ms
            for it in range(args.ablation_init):
                torch.cuda.synchronize()
                a0 = time.perf_counter()
                efanna.efanna_nndescent(Xd, g, 1, L, synth.ALGO_SEED, first_iter=it, workspace=ws_nnd)
                torch.cuda.synchronize()
                ms += (time.perf_counter() - a0) * 1e3
                curve.append({"iterations": it + 1, "ms": ms, "recall_at_K": recall_of(g)})
            return curve

        def tree_start():
            trees = efanna.efanna_build_trees(Xd, T, S, synth.ALGO_SEED, max_leaves=max_leaves, workspace=ws_tree)
            g = efanna.efanna_init_graph(Xd, trees[0], trees[1], trees[2], S, K, workspace=ws_init)
            return g

        def random_start():
            # K distinct random neighbours per point, never the point itself; a repeated draw leaves its slot empty
            gen = torch.Generator(device=dev)
            gen.manual_seed(synth.ALGO_SEED)
            r = torch.randint(0, n - 1, (n, K), generator=gen, device=dev, dtype=torch.int64)
            own = torch.arange(n, device=dev, dtype=torch.int64)[:, None]
            ids = (r + (r >= own)).sort(dim=1).values
            ids[:, 1:][ids[:, 1:] == ids[:, :-1]] = -1
            dist = efanna.efanna_pair_distances(Xd, own.expand(n, K).reshape(-1).int(),
                                                ids.clamp(min=0).reshape(-1).int()).view(n, K)
            dist[ids < 0] = float("inf")
            return efanna.efanna_set_graph(ids.int(), dist)

        curves = {}
        for label, start in (("tree_init", tree_start), ("random_init", random_start)):
            start()                                   # warm-up
            torch.cuda.synchronize()
            a0 = time.perf_counter()
            g = start()
            torch.cuda.synchronize()
            curves[label] = descend(g, (time.perf_counter() - a0) * 1e3)
        ablation = {"recall_rows": int(rows.shape[0]), **curves}

    achieved = k_bytes_sum / 1e9 / (k_ms_sum / 1e3) if k_ms_sum > 0 else 0.0
    achieved_all = all_bytes_sum / 1e9 / (all_ms_sum / 1e3) if all_ms_sum > 0 else 0.0
    out = {
        "metric": "kNN-graph build seconds + distance evals/sec at recall@K, N=1M d=128 K=10",
        "value": evals / seconds,
        "unit": "distance evals/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": seconds * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": name, "n": n, "d": d, "K": K, "trees": T, "leaf_size": S,
                   "iterations": I, "sample_L": L,
                   "conquer_depth": args.conquer_depth if conquer else "leaves"},
        "build_seconds": seconds,
        "dist_evals_per_step": evals,
        "recall_at_K": recall, "recall_rows": args.recall_rows if recall is not None else 0,
        "phase_ms": {k: float(v) * 1e3 / max(1, args.steps)
                     for k, v in zip(("trees", "init_graph", "nndescent", "get_graph"), phases)},
        "nndescent_iter_ms": {"sample_and_lists": [float(x) for x in phase_ms[:, 0]],
                              "join_le16": [float(x) for x in phase_ms[:, 1]],
                              "join_17_32": [float(x) for x in phase_ms[:, 2]],
                              "join_larger": [float(x) for x in phase_ms[:, 3]]},
        "nndescent_iter_work": {"dist_evals": [int(x) for x in st[:, 0]],
                                "insertions": [int(x) for x in st[:, 1]],
                                "vectors_gathered": [int(x) for x in st[:, 2]],
                                "vectors_gathered_join_le16": [int(x) for x in st[:, 3]]},
        "roofline": {"kernel": "join_reg_kernel<1> (joins of at most 16 vectors)", "bound": "hbm",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": (MEASURED_TRAFFIC_BYTES.get(name, {}).get("calibrated") if args.n is None else None),
                     "traffic_raw_counters": (MEASURED_TRAFFIC_BYTES.get(name, {}).get("raw_counters")
                                              if args.n is None else None),
                     "avg_launch_ms": k_ms_sum / max(1, k_launches),
                     "algorithmic_bytes_per_launch": k_bytes_sum / max(1, k_launches),
                     "all_join_kernels": {"achieved": achieved_all, "frac": achieved_all / HBM_PEAK_GBS,
                                          "ms_per_step": all_ms_sum / max(1, args.steps)}},
        "cpu_baseline": cpu,
    }
    if search is not None:
        out["search"] = search
    if ablation is not None:
        out["ablation_init"] = ablation
    print(json.dumps(out))


if __name__ == "__main__":
    main()
