"""Pins for the oracle's leaf-level initial graph (Alg. 3), NN-descent (Alg. 4), the
exact brute force and the accuracy measure (eqs. (2)-(3))."""
import numpy as np
import pytest

import oracle
from paper_1609_07228_amd import synth


# ----------------------------------------------------------------------------------
# exact kNN and accuracy

def test_exact_knn_shortlist_version_equals_definition():
    rng = np.random.default_rng(0)
    X = rng.standard_normal((400, 12)).astype(np.float32)
    X[37] = X[5]                                    # an exact duplicate: distance-0 tie
    ids_def, d_def = oracle.exact_knn_definition(X, 7)
    ids, d = oracle.exact_knn(X, np.arange(400), 7, block=64)
    assert np.array_equal(ids, ids_def) and np.allclose(d, d_def, rtol=1e-12, atol=0)
    assert ids_def[5, 0] == 37 and ids_def[37, 0] == 5


def test_exact_knn_on_a_line():
    X = np.arange(10, dtype=np.float32).reshape(10, 1) ** 2   # 0,1,4,9,...
    ids, d = oracle.exact_knn_definition(X, 2)
    assert ids[0].tolist() == [1, 2] and d[0].tolist() == [1.0, 16.0]
    assert ids[3].tolist() == [2, 4] and d[3].tolist() == [25.0, 49.0]


def test_accuracy_measure():
    t = np.array([[1, 2, 3], [4, 5, 6]])
    assert oracle.recall(t, t) == 1.0
    assert oracle.recall(np.array([[3, 9, 1], [7, 8, -1]]), t) == pytest.approx(2 / 6)
    assert oracle.recall(np.array([[-1, -1, -1], [-1, -1, -1]]), t) == 0.0


# ----------------------------------------------------------------------------------
# Alg. 3 at the leaves

def candidate_sets(perm, off, nl, n):
    cands = [set() for _ in range(n)]
    for t in range(perm.shape[0]):
        for l in range(nl[t]):
            leaf = perm[t, off[t, l]:off[t, l + 1]].tolist()
            for i in leaf:
                cands[i].update(leaf)
    for i in range(n):
        cands[i].discard(i)
    return cands


def test_init_graph_is_exact_knn_restricted_to_leaf_mates_integer_data():
    # integer-valued data: float32 and integer arithmetic agree exactly, ties included
    X = synth.generate("sift100k_like", n=3000)
    K, T, S = 10, 4, 16
    perm, off, nl = oracle.build_trees(X, T, S, seed=11)
    ids, dists, flags = oracle.init_graph(X, perm, off, nl, K)
    Xi = X.astype(np.int64)
    cands = candidate_sets(perm, off, nl, 3000)
    for i in range(3000):
        c = np.array(sorted(cands[i]), dtype=np.int64)
        dd = ((Xi[c] - Xi[i]) ** 2).sum(axis=1)
        order = np.lexsort((c, dd))[:K]
        m = order.shape[0]
        assert ids[i, :m].tolist() == c[order].tolist()
        assert dists[i, :m].tolist() == dd[order].astype(np.float64).tolist()
        assert np.all(ids[i, m:] == -1) and np.all(np.isinf(dists[i, m:]))
        assert np.all(flags[i, :m] == 1) and np.all(flags[i, m:] == 0)


def test_init_graph_float_data_against_float64():
    X = synth.generate("gmm10k_d32", n=2000)
    K, T, S = 10, 4, 8
    perm, off, nl = oracle.build_trees(X, T, S, seed=3)
    ids, dists, flags = oracle.init_graph(X, perm, off, nl, K)
    oracle.check_graph_invariants(X, ids, dists)
    cands = candidate_sets(perm, off, nl, 2000)
    Xd = X.astype(np.float64)
    under = 0
    for i in range(2000):
        c = np.array(sorted(cands[i]), dtype=np.int64)
        dd = ((Xd[c] - Xd[i]) ** 2).sum(axis=1)
        m = min(K, c.shape[0])
        under += m < K
        got = ids[i, :m]
        assert set(got.tolist()) <= set(c.tolist()) and np.all(ids[i, m:] == -1)
        kth = np.sort(dd)[m - 1]
        # every kept candidate is within rounding of the float64 top-m, and
        # nothing clearly closer was left out
        assert np.all(dd[np.isin(c, got)] <= kth * (1 + 1e-5))
        assert np.all(np.isin(c[dd < kth * (1 - 1e-5)], got))
    assert under > 0                 # this workload does produce under-full lists


def test_init_graph_single_leaf_is_the_exact_graph():
    X = synth.generate("sift100k_like", n=300)
    perm, off, nl = oracle.build_trees(X, T=1, S=300, seed=0)
    ids, dists, _ = oracle.init_graph(X, perm, off, nl, 10)
    tid, td = oracle.exact_knn_definition(X, 10)
    assert np.array_equal(ids, tid) and np.array_equal(dists.astype(np.float64), td)


def test_init_graph_row_subset_equals_full():
    X = synth.generate("gmm10k_d32", n=1500)
    perm, off, nl = oracle.build_trees(X, 3, 8, seed=1)
    ids, dists, flags = oracle.init_graph(X, perm, off, nl, 10)
    rows = np.array([0, 7, 99, 1499])
    ids2, dists2, flags2 = oracle.init_graph(X, perm, off, nl, 10, rows=rows)
    assert np.array_equal(ids[rows], ids2) and np.array_equal(dists[rows], dists2)


def test_more_trees_never_lower_init_accuracy():
    X = synth.generate("gmm10k_d32", n=3000)
    tid, _ = oracle.exact_knn(X, np.arange(3000), 10)
    prev = -1.0
    for T in (1, 2, 4, 8):
        perm, off, nl = oracle.build_trees(X, T, 8, seed=5)   # tree t is the same for every T
        ids, _, _ = oracle.init_graph(X, perm, off, nl, 10)
        r = oracle.recall(ids, tid)
        assert r >= prev
        prev = r
    assert prev > 0.3


# ----------------------------------------------------------------------------------
# Alg. 4

def py_iteration(Xi, pools, K, L, seed, it, cross_old=False):
    """One NN-descent iteration written with Python sets on integer data.
    pools: list of dict id -> [dist, is_new].  cross_old: what only pairs of a new and an old
    member offer to a pool enters it marked old (the literal marking of Alg. 4)."""
    n = len(pools)
    new, old = [], []
    for i in range(n):
        order = sorted(pools[i].items(), key=lambda kv: (kv[1][0], kv[0]))
        a, b = [], []
        for j, e in order:
            if len(a) == L:
                break
            if e[1]:
                a.append(j)
                e[1] = 0
            else:
                b.append(j)
        new.append(a)
        old.append(b)

    def reverse(fwd, stream):
        rc = [[] for _ in range(n)]
        for u in range(n):
            for v in fwd[u]:
                rc[v].append((oracle.reverse_hash(seed, stream, v, u), u))
        return [[u for _, u in sorted(c)[:L]] for c in rc]

    rnew, rold = reverse(new, 2 * it), reverse(old, 2 * it + 1)
    proposals = [dict() for _ in range(n)]
    by_new_pairs = [set() for _ in range(n)]      # offered by a pair of two new members
    evals = 0
    for i in range(n):
        un = sorted(set(new[i]) | set(rnew[i]))
        uo = sorted((set(old[i]) | set(rold[i])) - set(un))
        pairs = [(u, v) for a, u in enumerate(un) for v in un[a + 1:]]
        n_new_pairs = len(pairs)
        pairs += [(u, v) for u in un for v in uo]
        for k, (u, v) in enumerate(pairs):
            dist = int(((Xi[u] - Xi[v]) ** 2).sum())
            evals += 1
            proposals[u][v] = dist
            proposals[v][u] = dist
            if k < n_new_pairs:
                by_new_pairs[u].add(v)
                by_new_pairs[v].add(u)
    for u in range(n):
        merged = dict(pools[u])
        for v, dist in proposals[u].items():
            if v not in merged:
                merged[v] = [dist, 1 if (not cross_old or v in by_new_pairs[u]) else 0]
        keep = sorted(merged.items(), key=lambda kv: (kv[1][0], kv[0]))[:K]
        pools[u] = {j: e for j, e in keep}
    return evals


def pools_from_arrays(ids, dists, flags):
    return [{int(j): [int(dd), int(f)] for j, dd, f in zip(r, d, fl) if j >= 0}
            for r, d, fl in zip(ids, dists, flags)]


def arrays_from_pools(pools, K):
    n = len(pools)
    ids = np.full((n, K), -1, dtype=np.int32)
    dists = np.full((n, K), np.inf, dtype=np.float32)
    flags = np.zeros((n, K), dtype=np.uint8)
    for i, p in enumerate(pools):
        for s, (j, e) in enumerate(sorted(p.items(), key=lambda kv: (kv[1][0], kv[0]))):
            ids[i, s], dists[i, s], flags[i, s] = j, e[0], e[1]
    return ids, dists, flags


@pytest.mark.parametrize("K,L,cross_old", [(6, 6, False), (8, 3, False), (6, 6, True), (8, 3, True)])
def test_nndescent_iterations_against_set_based_python(K, L, cross_old):
    X = synth.generate("sift100k_like", n=600)[:, :24].copy()
    Xi = X.astype(np.int64)
    perm, off, nl = oracle.build_trees(X, 2, 6, seed=9)
    ids, dists, flags = oracle.init_graph(X, perm, off, nl, K)
    pools = pools_from_arrays(ids, dists, flags)
    for it in range(4 if cross_old else 3):
        ev = py_iteration(Xi, pools, K, L, seed=77, it=it, cross_old=cross_old)
        ids, dists, flags, stats = oracle.nndescent(X, ids, dists, flags, 1, L, seed=77, iter0=it,
                                                    cross_old=cross_old)
        wi, wd, wf = arrays_from_pools(pools, K)
        assert int(stats[0, 0]) == ev
        assert np.array_equal(ids, wi) and np.array_equal(dists, wd) and np.array_equal(flags, wf)


def test_nndescent_converges_to_exact_graph_on_small_low_dim_input():
    rng = np.random.default_rng(4)
    X = rng.standard_normal((1500, 4)).astype(np.float32)
    K = 10
    tid, _ = oracle.exact_knn_definition(X, K)
    perm, off, nl = oracle.build_trees(X, 4, 10, seed=2)
    ids, dists, flags = oracle.init_graph(X, perm, off, nl, K)
    recalls = [oracle.recall(ids, tid)]
    kth = [dists[:, -1].copy()]
    evals = []
    for it in range(12):
        ids, dists, flags, st = oracle.nndescent(X, ids, dists, flags, 1, K, seed=1, iter0=it)
        oracle.check_graph_invariants(X, ids, dists)
        recalls.append(oracle.recall(ids, tid))
        kth.append(dists[:, -1].copy())
        evals.append(int(st[0, 0]))
    assert all(b >= a for a, b in zip(recalls, recalls[1:]))        # accuracy never drops
    assert all(np.all(b <= a) for a, b in zip(kth, kth[1:]))        # K-th distance never grows
    assert recalls[-1] >= 0.99
    assert evals[-1] < evals[0] // 50                               # work dries up
    # stored distances are the oracle's own distance, bit for bit
    for i in (0, 17, 1499):
        for s in range(K):
            assert dists[i, s].tobytes() == oracle.dist(X[i], X[ids[i, s]]).tobytes()


def test_nndescent_fixed_point_and_resume():
    rng = np.random.default_rng(5)
    X = rng.standard_normal((500, 3)).astype(np.float32)
    perm, off, nl = oracle.build_trees(X, 3, 8, seed=2)
    g0 = oracle.init_graph(X, perm, off, nl, 8)
    a = oracle.nndescent(X, *g0, 5, 8, seed=3)
    b = g0
    for it in range(5):
        b = oracle.nndescent(X, *b, 1, 8, seed=3, iter0=it)[:3]
    assert all(np.array_equal(x, y) for x, y in zip(a[:3], b))      # 5 at once == 1+1+1+1+1
    c = oracle.nndescent(X, *a[:3], 30, 8, seed=3, iter0=5)
    assert int(c[3][-1, 0]) == 0                                    # nothing new: no work left
    d = oracle.nndescent(X, *c[:3], 1, 8, seed=3, iter0=35)
    assert np.array_equal(c[0], d[0]) and not d[2].any()


def test_nndescent_result_independent_of_evaluation_order():
    X = synth.generate("gmm10k_d32", n=4000)
    perm, off, nl = oracle.build_trees(X, 4, 8, seed=2)
    g0 = oracle.init_graph(X, perm, off, nl, 10)
    nt = oracle.num_threads()
    try:
        oracle.set_num_threads(1)
        a = oracle.nndescent(X, *g0, 3, 10, seed=3)
        oracle.set_num_threads(max(nt, 4))
        b = oracle.nndescent(X, *g0, 3, 10, seed=3)
    finally:
        oracle.set_num_threads(nt)
    assert all(np.array_equal(x, y) for x, y in zip(a[:3], b[:3]))
    assert np.array_equal(a[3][:, 0], b[3][:, 0])


def test_sampling_takes_the_L_closest_new_entries_only():
    # 5 points on a line; pool of point 0 = {1,2,3,4} all new; L=2 -> after one
    # iteration the two closest have lost their flag, the others keep it
    X = np.array([[0.0], [1.0], [2.0], [3.0], [4.0]], dtype=np.float32)
    ids = np.array([[1, 2, 3, 4]] + [[-1] * 4] * 4, dtype=np.int32)
    dists = np.array([[1, 4, 9, 16]] + [[np.inf] * 4] * 4, dtype=np.float32)
    flags = np.array([[1, 1, 1, 1]] + [[0] * 4] * 4, dtype=np.uint8)
    ids2, dists2, flags2, st = oracle.nndescent(X, ids, dists, flags, 1, 2, seed=0)
    assert ids2[0].tolist() == [1, 2, 3, 4] and flags2[0].tolist() == [0, 0, 1, 1]
    assert int(st[0, 0]) == 1                       # the only joined pair is (1,2)
    assert ids2[1, 0] == 2 and ids2[2, 0] == 1 and dists2[1, 0] == 1.0 and flags2[1, 0] == 1
    assert np.all(ids2[3:] == -1)


def test_early_termination_stops_where_the_fresh_entries_run_out():
    """delta > 0: the run ends after the first iteration that leaves fewer than delta*n*K
    entries carrying the new mark.  The expected stopping point is read off a run made
    one iteration at a time, with the marks counted here."""
    X = synth.generate("gmm10k_d32", n=2500)
    K, L = 10, 10
    perm, off, nl = oracle.build_trees(X, 3, 8, 42)
    g0 = oracle.init_graph(X, perm, off, nl, K)
    state, fresh = g0, []
    for it in range(8):
        state = oracle.nndescent(X, *state[:3], 1, L, 42, iter0=it)
        fresh.append(int(state[2].sum()))
    assert fresh[0] > fresh[-1]
    for delta in (0.2, 0.02, 0.002):
        limit = delta * X.shape[0] * K
        want = next((i + 1 for i, f in enumerate(fresh) if f < limit), 8)
        ids, dists, flags, stats, done = oracle.nndescent(X, *g0[:3], 8, L, 42, delta=delta)
        assert done == want and stats.shape[0] == want
        ref = oracle.nndescent(X, *g0[:3], want, L, 42)
        assert np.array_equal(ids, ref[0]) and np.array_equal(flags, ref[2])
    # exactly delta*n*K fresh entries is not "fewer": pick delta so that the limit, formed as the
    # paper's delta*N*K in double precision, equals the count after the third iteration
    n = X.shape[0]
    delta = fresh[2] / (n * K)
    for _ in range(64):
        if delta * n * K == fresh[2]:
            break
        delta = float(np.nextafter(delta, 1.0 if delta * n * K < fresh[2] else 0.0))
    assert delta * n * K == fresh[2] and fresh[3] < fresh[2] < fresh[1]
    assert oracle.nndescent(X, *g0[:3], 8, L, 42, delta=delta)[4] == 4
    # a threshold nothing can meet stops after one iteration, zero never stops early
    assert oracle.nndescent(X, *g0[:3], 5, L, 42, delta=2.0)[4] == 1
    assert oracle.nndescent(X, *g0[:3], 3, L, 42)[3].shape[0] == 3


def test_literal_marking_hand_case_and_properties():
    """Alg. 4's second inner loop marks what a new and an old member insert as old.  Five points on a
    line, rows of 2, sample of 2: after one ordinary iteration from a hand-made graph, point 0 has
    the new neighbour 1 and the old neighbour 4... written out below."""
    # points at 0, 1, 2, 10, 11; K = 2.  Row 2 holds {3 (old), 1 (new)}: the join of point 2 pairs the
    # new member 1 with the old member 3 only: 1 <- 3 (dist 81) and 3 <- 1.
    X = np.array([[0.0], [1.0], [2.0], [10.0], [11.0]], dtype=np.float32)
    ids = np.array([[-1, -1], [-1, -1], [1, 3], [-1, -1], [-1, -1]], dtype=np.int32)
    dists = np.array([[np.inf, np.inf], [np.inf, np.inf], [1.0, 64.0], [np.inf, np.inf], [np.inf, np.inf]],
                     dtype=np.float32)
    flags = np.array([[0, 0], [0, 0], [1, 0], [0, 0], [0, 0]], dtype=np.uint8)
    a = oracle.nndescent(X, ids, dists, flags, 1, 2, seed=0)
    b = oracle.nndescent(X, ids, dists, flags, 1, 2, seed=0, cross_old=True)
    # the same entries either way (1 <-> 3 at distance 81, found by the join of point 2) ...
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert a[0][1].tolist() == [3, -1] and a[0][3].tolist() == [1, -1] and a[1][1, 0] == 81.0
    # ... marked new by default and old in the literal reading
    assert a[2][1, 0] == 1 and a[2][3, 0] == 1
    assert b[2][1, 0] == 0 and b[2][3, 0] == 0
    assert int(a[3][0, 0]) == 1 and int(b[3][0, 0]) == 1      # one pair evaluated

    # on real-shaped data: same work in the first iteration (every entry is new: no old members), never
    # more marks than the default afterwards, and the join dries up sooner
    Xs = synth.generate("gmm10k_d32", n=1500)
    perm, off, nl = oracle.build_trees(Xs, 3, 8, seed=2)
    g0 = oracle.init_graph(Xs, perm, off, nl, 8)
    d1 = oracle.nndescent(Xs, *g0, 1, 8, seed=5)
    l1 = oracle.nndescent(Xs, *g0, 1, 8, seed=5, cross_old=True)
    assert all(np.array_equal(x, y) for x, y in zip(d1[:3], l1[:3])) and d1[3][0, 0] == l1[3][0, 0]
    d6 = oracle.nndescent(Xs, *g0, 6, 8, seed=5)
    l6 = oracle.nndescent(Xs, *g0, 6, 8, seed=5, cross_old=True)
    assert l6[3][:, 0].sum() < d6[3][:, 0].sum()
    assert l6[2].sum() <= d6[2].sum()
    tid, _ = oracle.exact_knn(Xs, np.arange(1500), 8)
    assert oracle.recall(l6[0], tid) <= oracle.recall(d6[0], tid) + 0.01
    oracle.check_graph_invariants(Xs, l6[0], l6[1])
