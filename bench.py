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

TRAFFIC_SUMMARY = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles",
                               "join_kernels_sift1m_like_hbm_traffic.txt")


def measured_traffic(workload: str):
    """HBM bytes per launch of the dominant kernel as the tracked rocprofv3 summary states them
    (`key: value` lines: workload, commit, traffic_bytes_per_launch, ...), or None when the
    summary covers another workload.  The figures are counters of a profiled run, not of this run."""
    try:
        kv = {}
        with open(TRAFFIC_SUMMARY) as f:
            for line in f:
                if ":" in line and not line.startswith(" "):
                    k, v = line.split(":", 1)
                    kv[k.strip()] = v.strip()
        if kv.get("workload") != workload:
            return None
        return {"traffic": float(kv["traffic_bytes_per_launch"]),
                "fetch_bytes": float(kv["fetch_bytes_per_launch"]),
                "write_bytes": float(kv["write_bytes_per_launch"]),
                "commit": kv.get("commit"), "source": "profiles/" + os.path.basename(TRAFFIC_SUMMARY)}
    except (OSError, KeyError, ValueError):
        return None


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


def recall_of_ids(ids_dev, Xd, rows, K):
    """recall@K (eqs. (2)-(3)) of the graph rows `rows` against float64 brute force."""
    import torch
    rows_d = torch.from_numpy(rows).to(Xd.device)
    truth = exact_knn_torch(Xd, rows_d, K)
    got = ids_dev[rows_d].cpu().numpy()
    hits = sum(np.intersect1d(a[a >= 0], b).shape[0] for a, b in zip(got, truth))
    return hits / float(truth.size)


def measure(name, n_rows, steps, warmup, recall_rows, conquer_depth=None, progress=False):
    """`warmup` untimed and `steps` timed builds of workload `name` (trees + initial graph +
    NN-descent + finalise, inputs resident in HBM).  Returns the figures of the timed builds and
    what later legs need (device data, the last build's outputs)."""
    import torch
    from paper_1609_07228_amd import efanna, synth

    p = synth.params(name)
    X = synth.generate(name, n=n_rows)
    n, d = X.shape
    if progress:
        print(f"generated {name}: {n} x {d}", file=sys.stderr, flush=True)
    K, T, S, I, L = p["K"], p["T"], p["S"], p["I"], p["L"]
    dev = torch.device("cuda:0")
    Xd = torch.from_numpy(X).to(dev)
    L_ = efanna.lib()
    conquer = conquer_depth is not None
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
    # Phase times come from events on the launch stream, read after the timed region: a step has
    # no host synchronisation of its own (the tree build reads its level counters and the phase
    # timing of efanna_nndescent waits for the stream; both are part of the library calls).
    step_events, step_phase_ms = [], []

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
                                     conquer_depth=conquer_depth)
        else:
            efanna.efanna_init_graph(Xd, perm, leaf_off, n_leaves, S, K, graph=graph, workspace=ws_init)
        ev[2].record()
        efanna.efanna_nndescent(Xd, graph, I, L, synth.ALGO_SEED, stats=stats, workspace=ws_nnd,
                                phase_ms=phase_ms)
        ev[3].record()
        ids, dists = efanna.efanna_get_graph(graph)
        ev[4].record()
        if progress:
            torch.cuda.synchronize()
            print("step: trees %.3f ms, init %.3f ms, nndescent %.3f ms, get %.3f ms"
                  % tuple(ev[k].elapsed_time(ev[k + 1]) for k in range(4)), file=sys.stderr, flush=True)
        if timed:
            step_events.append(ev)
            step_phase_ms.append(phase_ms.copy())      # host memory, filled by the call above
        state.update(perm=perm, leaf_off=leaf_off, n_leaves=n_leaves, ids=ids, dists=dists)

    for _ in range(warmup):
        step(False)
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for _ in range(steps):
        step(True)
    torch.cuda.synchronize()
    seconds = (time.perf_counter() - t_begin) / max(1, steps)
    phases = np.zeros(4)
    for ev in step_events:
        phases[:] += [ev[k].elapsed_time(ev[k + 1]) * 1e-3 for k in range(4)]
    st = stats.cpu().numpy()      # the path is deterministic: the same in every step
    # dominant kernel: the join of points that gather at most 16 vectors (one launch per iteration)
    k_ms_sum = k_bytes_sum = all_ms_sum = all_bytes_sum = 0.0
    for pm in step_phase_ms:
        k_ms_sum += float(pm[:, 1].sum())
        k_bytes_sum += float((st[:, 3] * (d * 4 + 8)).sum())
        all_ms_sum += float(pm[:, 1:].sum())
        all_bytes_sum += float((st[:, 2] * (d * 4 + 8) + st[:, 1] * 8).sum())
    k_launches = I * len(step_phase_ms)
    # work done per step
    off = state["leaf_off"].cpu().numpy().astype(np.int64)
    init_evals = 0
    for t in range(T):
        sizes = np.diff(off[t, :state["n_leaves"][t] + 1])
        init_evals += int((sizes * (sizes - 1) // 2).sum())
    evals = init_evals + int(st[:, 0].sum())
    recall = None
    if recall_rows > 0:
        recall = recall_of_ids(state["ids"], Xd, synth.sample_rows(n, recall_rows), K)
    achieved = k_bytes_sum / 1e9 / (k_ms_sum / 1e3) if k_ms_sum > 0 else 0.0
    achieved_all = all_bytes_sum / 1e9 / (all_ms_sum / 1e3) if all_ms_sum > 0 else 0.0
    return {
        "name": name, "X": X, "Xd": Xd, "state": state, "params": p, "max_leaves": max_leaves,
        "ws_tree": ws_tree, "ws_init": ws_init, "ws_nnd": ws_nnd,
        "n": n, "d": d, "seconds": seconds, "evals": evals, "recall": recall,
        "phases_ms": {k: float(v) * 1e3 / max(1, steps)
                      for k, v in zip(("trees", "init_graph", "nndescent", "get_graph"), phases)},
        "phase_ms": phase_ms, "stats": st,
        "join_le16": {"achieved": achieved, "avg_launch_ms": k_ms_sum / max(1, k_launches),
                      "bytes_per_launch": k_bytes_sum / max(1, k_launches)},
        "all_joins": {"achieved": achieved_all, "ms_per_step": all_ms_sum / max(1, steps)},
    }


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
    ap.add_argument("--others", default=None, metavar="LIST",
                    help="comma-separated workloads measured after the headline steps (1 warm-up + 2 builds "
                         "each, recall on, no CPU leg) and reported under `other_workloads`; default: the four "
                         "other configurations when the workload is the headline at full size, none otherwise; "
                         "'none' switches them off")
    ap.add_argument("--calibrate", action="store_true",
                    help="after the timed steps, run kernels with a known amount of HBM traffic to scale rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters by: a torch fill of 256 MiB, an elementwise add over "
                         "256 MiB, and efanna_pair_distances over 4M random pairs of the data (random row gathers "
                         "in 64-byte pieces, the join's access pattern: 2 rows fetched and 4 bytes written per pair)")
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
    ap.add_argument("--ablation-split", type=int, default=0, metavar="ITERS",
                    help="also build the trees with the split dimension taken among the five of largest "
                         "variance (Sec. 3.2) and with random-projection splits, and add an `ablation_split` "
                         "object: tree time, accuracy of the initial graph and after every one of ITERS "
                         "iterations, for the three rules")
    ap.add_argument("--ablation-marking", type=int, default=0, metavar="ITERS",
                    help="after the build, run NN-descent one iteration at a time for ITERS iterations with fresh "
                         "entries always marked new (the default) and with the literal marking of Alg. 4 (what a new "
                         "and an old member insert is marked old) and add an `ablation_marking` object: time, "
                         "recall and pairs evaluated after every iteration of both")
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
    conquer = args.conquer_depth is not None
    m = measure(name, args.n, args.steps, args.warmup, args.recall_rows, args.conquer_depth, args.progress)
    X, Xd, state, p = m["X"], m["Xd"], m["state"], m["params"]
    n, d = m["n"], m["d"]
    K, T, S, I, L = p["K"], p["T"], p["S"], p["I"], p["L"]
    dev = Xd.device
    max_leaves, ws_tree, ws_init, ws_nnd = m["max_leaves"], m["ws_tree"], m["ws_init"], m["ws_nnd"]
    seconds, evals, recall, phase_ms, st = m["seconds"], m["evals"], m["recall"], m["phase_ms"], m["stats"]
    phases_ms, join_le16, all_joins = m["phases_ms"], m["join_le16"], m["all_joins"]

    if args.calibrate:
        a = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        a.fill_(1.0)
        torch.cuda.synchronize()
        torch.add(a, 1.0, out=b)      # an elementwise kernel (a plain copy may go to a DMA engine instead)
        torch.cuda.synchronize()
        del a, b
        gen = torch.Generator(device=dev)
        gen.manual_seed(1)
        pa = torch.randint(0, n, (4 * 1024 * 1024,), generator=gen, device=dev, dtype=torch.int32)
        pb = torch.randint(0, n, (4 * 1024 * 1024,), generator=gen, device=dev, dtype=torch.int32)
        torch.cuda.synchronize()
        efanna.efanna_pair_distances(Xd, pa, pb)
        torch.cuda.synchronize()
        del pa, pb

    cpu = None
    if args.cpu_rows > 0:
        import oracle
        mm = min(n, args.cpu_rows)
        Xs = X[:mm]
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
                         f"{mm} rows of {name}"}
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

    marking = None
    if args.ablation_marking > 0:
        rows_m = torch.from_numpy(synth.sample_rows(n, max(1000, args.recall_rows))).to(dev)
        truth_m = exact_knn_torch(Xd, rows_m, K)

        def recall_m(g):
            got = efanna.efanna_get_graph(g)[0][rows_m].cpu().numpy()
            return sum(np.intersect1d(a[a >= 0], b).shape[0] for a, b in zip(got, truth_m)) / float(truth_m.size)

        marking = {"recall_rows": int(rows_m.shape[0])}
        for label, cross_old in (("fresh_entries_new", False), ("literal_new_x_old_marked_old", True)):
            curve = []
            for rep_ in range(2):      # the first round warms up
                trees = efanna.efanna_build_trees(Xd, T, S, synth.ALGO_SEED, max_leaves=max_leaves, workspace=ws_tree)
                g = efanna.efanna_init_graph(Xd, trees[0], trees[1], trees[2], S, K, workspace=ws_init)
                curve, ms, pairs = [], 0.0, 0
                for it in range(args.ablation_marking):
                    torch.cuda.synchronize()
                    a0 = time.perf_counter()
                    stt = efanna.efanna_nndescent(Xd, g, 1, L, synth.ALGO_SEED, first_iter=it, workspace=ws_nnd,
                                                  cross_old=cross_old)
                    torch.cuda.synchronize()
                    ms += (time.perf_counter() - a0) * 1e3
                    pairs += int(stt[0, 0].item())
                    if rep_ == 1:
                        curve.append({"iterations": it + 1, "nndescent_ms": ms, "pairs_evaluated": pairs,
                                      "recall_at_K": recall_m(g)})
            marking[label] = curve

    split = None
    if args.ablation_split > 0:
        rows_s = torch.from_numpy(synth.sample_rows(n, max(1000, args.recall_rows))).to(dev)
        truth_s = exact_knn_torch(Xd, rows_s, K)

        def recall_s(g):
            got = efanna.efanna_get_graph(g)[0][rows_s].cpu().numpy()
            return sum(np.intersect1d(a[a >= 0], b).shape[0] for a, b in zip(got, truth_s)) / float(truth_s.size)

        split = {"recall_rows": int(rows_s.shape[0])}
        for label, rule in (("uniform", efanna.SPLIT_UNIFORM), ("variance", efanna.SPLIT_VARIANCE),
                            ("projection", efanna.SPLIT_PROJECTION)):
            for rep_ in range(2):      # the first round warms up
                torch.cuda.synchronize()
                a0 = time.perf_counter()
                trees = efanna.efanna_build_trees_rule(Xd, T, S, synth.ALGO_SEED, rule, max_leaves=max_leaves,
                                                       workspace=ws_tree)
                torch.cuda.synchronize()
                trees_ms = (time.perf_counter() - a0) * 1e3
                g = efanna.efanna_init_graph(Xd, trees[0], trees[1], trees[2], S, K, workspace=ws_init)
                curve = [{"iterations": 0, "recall_at_K": recall_s(g)}]
                for it in range(args.ablation_split):
                    efanna.efanna_nndescent(Xd, g, 1, L, synth.ALGO_SEED, first_iter=it, workspace=ws_nnd)
                    curve.append({"iterations": it + 1, "recall_at_K": recall_s(g)})
            split[label] = {"trees_ms": trees_ms, "curve": curve}

    # the other configurations: a build each on the same GPU, after the headline's buffers are gone
    others_arg = args.others
    if others_arg is None:
        others_arg = ("gmm10k_d32,sift100k_like,gist1m_like,mixed4m_d96"
                      if name == "sift1m_like" and args.n is None and not conquer else "none")
    others = None
    if others_arg != "none":
        del m, Xd, ws_tree, ws_init, ws_nnd, state
        torch.cuda.empty_cache()
        others = {}
        for other in [o for o in others_arg.split(",") if o]:
            o = measure(other, None, 2, 1, min(args.recall_rows, 10_000) if args.recall_rows > 0 else 0,
                        None, args.progress)
            op = o["params"]
            others[other] = {
                "config": {"n": o["n"], "d": o["d"], "K": op["K"], "trees": op["T"], "leaf_size": op["S"],
                           "iterations": op["I"], "sample_L": op["L"]},
                "steps": 2, "warmup": 1, "ms_per_build": o["seconds"] * 1e3,
                "dist_evals_per_s": o["evals"] / o["seconds"], "dist_evals_per_build": o["evals"],
                "recall_at_K": o["recall"], "phase_ms": o["phases_ms"],
                "join_le16_frac": o["join_le16"]["achieved"] / HBM_PEAK_GBS,
                "all_join_kernels_frac": o["all_joins"]["achieved"] / HBM_PEAK_GBS,
                "all_join_kernels_ms": o["all_joins"]["ms_per_step"]}
            del o
            torch.cuda.empty_cache()

    traffic = measured_traffic(name) if args.n is None and not conquer else None
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
        "phase_ms": phases_ms,
        "nndescent_iter_ms": {"sample_and_lists": [float(x) for x in phase_ms[:, 0]],
                              "join_le16": [float(x) for x in phase_ms[:, 1]],
                              "join_17_32": [float(x) for x in phase_ms[:, 2]],
                              "join_larger": [float(x) for x in phase_ms[:, 3]]},
        "nndescent_iter_work": {"dist_evals": [int(x) for x in st[:, 0]],
                                "insertions": [int(x) for x in st[:, 1]],
                                "vectors_gathered": [int(x) for x in st[:, 2]],
                                "vectors_gathered_join_le16": [int(x) for x in st[:, 3]]},
        "roofline": {"kernel": "join_reg_kernel (joins of at most 16 vectors)", "bound": "hbm",
                     "achieved": join_le16["achieved"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": join_le16["achieved"] / HBM_PEAK_GBS,
                     "traffic": traffic["traffic"] if traffic else None,
                     "traffic_detail": ({k: traffic[k] for k in ("fetch_bytes", "write_bytes", "commit", "source")}
                                        if traffic else None),
                     "avg_launch_ms": join_le16["avg_launch_ms"],
                     "algorithmic_bytes_per_launch": join_le16["bytes_per_launch"],
                     "all_join_kernels": {"achieved": all_joins["achieved"],
                                          "frac": all_joins["achieved"] / HBM_PEAK_GBS,
                                          "ms_per_step": all_joins["ms_per_step"]}},
        "cpu_baseline": cpu,
    }
    if others is not None:
        out["other_workloads"] = others
    if search is not None:
        out["search"] = search
    if ablation is not None:
        out["ablation_init"] = ablation
    if split is not None:
        out["ablation_split"] = split
    if marking is not None:
        out["ablation_marking"] = marking
    print(json.dumps(out))


if __name__ == "__main__":
    main()
