"""Pins for the oracle's search with the index (Alg. 1).  Expected values come from brute
force, from a hand-worked case, from a separate walk of the tree in Python integers, and from
properties of the algorithm - never from the function under test."""
import heapq

import numpy as np
import pytest

import oracle
from paper_1609_07228_amd import synth


def q20(x):
    return int(np.rint(np.float64(x) * 1048576.0))


def brute(X, Q, K):
    d2 = ((Q[:, None, :].astype(np.float64) - X[None].astype(np.float64)) ** 2).sum(-1)
    order = np.lexsort((np.broadcast_to(np.arange(X.shape[0]), d2.shape), d2), axis=1)[:, :K]
    return order, np.take_along_axis(d2, order, 1)


def index(X, T, S, K, iters=3, seed=42):
    t = oracle.build_trees_nodes(X, T, S, seed)
    g = oracle.nndescent(X, *oracle.init_graph(X, *t[:3], K), iters, K, seed)
    return t, g[0]


def test_one_leaf_is_brute_force():
    """A tree whose only leaf holds every point hands all points to the first pool: with
    E = P >= K the answer is the exact kNN of the query, whatever the graph says."""
    rng = np.random.default_rng(1)
    X = rng.integers(0, 50, (60, 5)).astype(np.float32)        # integer data: exact distances, ties by id
    Q = rng.integers(0, 50, (25, 5)).astype(np.float32)
    t, g = index(X, 2, 64, 6)
    assert list(t[2]) == [1, 1]
    ids, dists, checked = oracle.search(X, t[0], t[1], t[2], t[3], 64, g, Q, 6, 60, 60, 2)
    want_ids, want_d = brute(X, Q, 6)
    assert np.array_equal(ids, want_ids)
    assert np.array_equal(dists.astype(np.float64), want_d)
    assert np.all(checked == 60)


def test_hand_case_on_a_line():
    # 0..7 on a line, leaves {0,1} {2,3} {4,5} {6,7}; splits at 3.5, then 1.5 and 5.5.
    X = np.arange(8, dtype=np.float32)[:, None]
    t = oracle.build_trees_nodes(X, 1, 2, 3)
    graph = np.full((8, 1), -1, dtype=np.int32)                 # no edges: only the trees speak
    Q = np.array([[2.2]], dtype=np.float32)
    # N_node = P / S / T + 1 leaves.  P = 1: one leaf, {2,3}.
    ids, dists, checked = oracle.search(X, t[0], t[1], t[2], t[3], 2, graph, Q, 1, 1, 1, 1)
    assert list(ids[0]) == [2] and checked[0] == 2
    # P = 2: two leaves.  Set aside on the way down: the root's right side at (3.5-2.2)^2 = 1.69,
    # the left node's left child {0,1} at (2.2-1.5)^2 = 0.49 -> {0,1} comes second
    ids, dists, checked = oracle.search(X, t[0], t[1], t[2], t[3], 2, graph, Q, 2, 2, 2, 1)
    assert list(ids[0]) == [2, 3] and checked[0] == 4
    assert np.allclose(dists[0], [0.04, 0.64], rtol=1e-5)
    # P = 4: three leaves; the third is reached through the root's right side and then goes to
    # the query's side of 5.5, i.e. {4,5}; the four closest of the six are kept
    ids, _, checked = oracle.search(X, t[0], t[1], t[2], t[3], 2, graph, Q, 4, 4, 4, 1)
    assert list(ids[0]) == [2, 3, 1, 4] and checked[0] == 6
    # P = 6: all four leaves
    ids, _, checked = oracle.search(X, t[0], t[1], t[2], t[3], 2, graph, Q, 6, 6, 6, 1)
    assert list(ids[0]) == [2, 3, 1, 4, 0, 5] and checked[0] == 8
    # E = 1 keeps only point 2 of the leaves; its single graph neighbour is then the only addition
    graph[2, 0] = 7
    ids, _, checked = oracle.search(X, t[0], t[1], t[2], t[3], 2, graph, Q, 2, 2, 1, 1)
    assert list(ids[0]) == [2, 7] and checked[0] == 5
    # a graph neighbour that the leaves already delivered is not evaluated a second time
    graph[2, 0] = 3
    ids, _, checked = oracle.search(X, t[0], t[1], t[2], t[3], 2, graph, Q, 2, 2, 1, 1)
    assert list(ids[0]) == [2] + [-1] and checked[0] == 4


def test_equal_priorities_are_taken_in_link_order():
    # same tree, query on the root's split value 3.5: the root sends it right (not below the
    # mean) and puts its left child aside at priority 0.  Leaf {4,5} is found first and {6,7}
    # put aside at (5.5-3.5)^2 = 4; the left child comes next, leads to {2,3} and puts {0,1}
    # aside at (3.5-1.5)^2 = 4 as well.  Links of leaves are ~index: {6,7} is -4, {0,1} is -1,
    # so the third leaf is {6,7}.
    X = np.arange(8, dtype=np.float32)[:, None]
    t = oracle.build_trees_nodes(X, 1, 2, 3)
    graph = np.full((8, 1), -1, dtype=np.int32)
    Q = np.array([[3.5]], dtype=np.float32)
    ids, dists, checked = oracle.search(X, t[0], t[1], t[2], t[3], 2, graph, Q, 5, 5, 5, 1)
    assert checked[0] == 6
    assert list(ids[0]) == [3, 4, 2, 5, 6]
    assert list(dists[0]) == [0.25, 0.25, 2.25, 2.25, 6.25]


def python_leaves(q, nodes, n_leaves, want):
    """Best-bin-first search written separately, on Python integers and a heap."""
    if n_leaves == 1:
        return [0]
    root = next(j for j in range(1, n_leaves) if int(nodes[j]["parent"]) < 0)
    heap, found, link, prio = [], [], root, 0.0
    while len(found) < want:
        while link >= 0:
            nd = nodes[link]
            dim, cnt, sm = int(nd["dim"]), int(nd["cnt"]), int(nd["sum"])
            if dim >= 0:
                diff = cnt * q20(q[dim]) - sm
                left = diff < 0
                gap = float(diff) / (float(cnt) * 1048576.0)
                other = float(np.float64(gap) * np.float64(gap) + np.float64(prio))
            else:
                left, other = True, prio
            heapq.heappush(heap, (other, int(nd["child"][1 if left else 0])))
            link = int(nd["child"][0 if left else 1])
        found.append(~link)
        if not heap:
            break
        prio, link = heapq.heappop(heap)
    return found


@pytest.mark.parametrize("name,n,T,S,P", [("gmm10k_d32", 3000, 3, 8, 120), ("sift100k_like", 2000, 2, 16, 100)])
def test_first_pool_comes_from_the_leaves_a_separate_search_finds(name, n, T, S, P):
    """With no iterations the answer is the exact kNN over the members of the leaves that an
    independently written best-bin-first search reaches."""
    X = synth.generate(name, n=n)
    rng = np.random.default_rng(5)
    Q = (X[rng.choice(n, 40)] + rng.standard_normal((40, X.shape[1])).astype(np.float32)).astype(np.float32)
    t, g = index(X, T, S, 10, iters=1)
    want_leaves = P // S // T + 1
    ids, dists, checked = oracle.search(X, t[0], t[1], t[2], t[3], S, g, Q, 10, P, P, 0)
    for qi in range(Q.shape[0]):
        cand = set()
        for tr in range(T):
            for leaf in python_leaves(Q[qi], t[3][tr], int(t[2][tr]), want_leaves):
                cand.update(int(v) for v in t[0][tr, t[1][tr, leaf]:t[1][tr, leaf + 1]])
        cand = sorted(cand)
        assert checked[qi] == len(cand)
        dd = ((X[cand].astype(np.float64) - Q[qi].astype(np.float64)) ** 2).sum(1)
        got = [int(v) for v in ids[qi] if v >= 0]
        assert len(got) == min(10, len(cand)) and set(got) <= set(cand)
        kth = np.sort(dd)[len(got) - 1]
        assert np.all(dists[qi, :len(got)].astype(np.float64) <= kth * (1 + 1e-5))


def test_expansion_follows_the_graph_and_never_loses_ground():
    X = synth.generate("gmm10k_d32", n=4000)
    rng = np.random.default_rng(9)
    Q = (X[rng.choice(4000, 100)] + 0.3 * rng.standard_normal((100, 32))).astype(np.float32)
    t, g = index(X, 4, 8, 10, iters=4)
    truth, _ = brute(X, Q, 10)
    last, last_checked = -1.0, None
    for iters in (0, 1, 2, 4, 8):
        ids, dists, checked = oracle.search(X, t[0], t[1], t[2], t[3], 8, g, Q, 10, 60, 20, iters)
        # sorted by (distance, id), distances are the library's distance to the query
        for qi in range(0, 100, 17):
            for c in range(10):
                assert dists[qi, c] == oracle.dist(Q[qi], X[ids[qi, c]])
        assert np.all((dists[:, :-1] < dists[:, 1:]) | ((dists[:, :-1] == dists[:, 1:]) & (ids[:, :-1] < ids[:, 1:])))
        r = np.mean([len(set(a) & set(b)) / 10 for a, b in zip(ids, truth)])
        assert r >= last                       # the pool is the P closest of a growing set
        if last_checked is not None:
            assert np.all(checked >= last_checked)
        last, last_checked = r, checked
    assert last > 0.95
    # one round from a pool of E points checks at most E * Kg more points than the trees did
    _, _, c0 = oracle.search(X, t[0], t[1], t[2], t[3], 8, g, Q, 10, 60, 20, 0)
    _, _, c1 = oracle.search(X, t[0], t[1], t[2], t[3], 8, g, Q, 10, 60, 20, 1)
    assert np.all(c1 - c0 <= 20 * 10)


def test_query_that_is_a_data_point_finds_itself():
    X = synth.generate("gmm10k_d32", n=2000)
    t, g = index(X, 3, 8, 10)
    rows = np.arange(0, 2000, 37)
    ids, dists, _ = oracle.search(X, t[0], t[1], t[2], t[3], 8, g, X[rows], 5, 30, 10, 2)
    assert np.array_equal(ids[:, 0], rows) and np.all(dists[:, 0] == 0)
