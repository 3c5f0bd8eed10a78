"""Pins for the oracle's conquer step with sibling subtrees (Alg. 3 above the leaves).

None of these checks calls the function under test to produce its own expectation: hand
cases worked out on paper, a data set on which the step provably yields the exact kNN
graph, candidate sets rebuilt by a separate walk in Python integers, and invariants."""
import numpy as np
import pytest

import oracle
from paper_1609_07228_amd import synth


def q(x):
    return int(np.rint(np.float64(x) * 1048576.0))


def test_nodes_of_a_perfect_binary_tree():
    # 0..7 on a line, leaves of 2: root splits at the mean 3.5, its children at 1.5 / 5.5
    X = np.arange(8, dtype=np.float32)[:, None]
    perm, off, nl, nodes, up = oracle.build_trees_nodes(X, 1, 2, 3)
    assert nl[0] == 4 and list(off[0, :5]) == [0, 2, 4, 6, 8]
    nd = nodes[0]
    # node numbers = leaf that starts the right part: root 2, left child 1, right child 3
    assert (nd[2]["depth"], nd[2]["cnt"], nd[2]["sum"], nd[2]["parent"]) == (0, 8, 28 << 20, -1)
    assert list(nd[2]["child"]) == [1, 3]
    assert (nd[1]["depth"], nd[1]["cnt"], nd[1]["sum"], nd[1]["parent"]) == (1, 4, 6 << 20, 2)
    assert list(nd[1]["child"]) == [~0, ~1]
    assert (nd[3]["depth"], nd[3]["cnt"], nd[3]["sum"], nd[3]["parent"]) == (1, 4, 22 << 20, 2)
    assert list(nd[3]["child"]) == [~2, ~3]
    assert all(nd[j]["dim"] == 0 for j in (1, 2, 3))
    assert list(up[0, :4]) == [1 * 2 + 0, 1 * 2 + 1, 3 * 2 + 0, 3 * 2 + 1]


def test_hand_case_on_a_line():
    # same tree.  Point 0 lives in leaf {0,1} (depth 2).  Its ancestor at depth 1 has the sibling
    # leaf {2,3}; the root's other subtree holds {4..7} and sends 0 (below its mean 5.5) to {4,5}.
    X = np.arange(8, dtype=np.float32)[:, None]
    t = oracle.build_trees_nodes(X, 1, 2, 3)
    for dep, want in ((2, [1]), (1, [1, 2, 3]), (0, [1, 2, 3, 4, 5])):
        ids, dists, flags = oracle.conquer_graph(X, *t, dep, 6)
        got = [int(v) for v in ids[0] if v >= 0]
        assert got == want, (dep, got)
        assert list(dists[0, :len(want)]) == [float(v * v) for v in want]
        assert list(flags[0]) == [1] * len(want) + [0] * (6 - len(want))
    # point 5 (leaf {4,5}): sibling leaf {6,7}; the root's left subtree sends 5 to its right leaf {2,3}
    ids, _, _ = oracle.conquer_graph(X, *t, 0, 6)
    assert sorted(int(v) for v in ids[5] if v >= 0) == [2, 3, 4, 6, 7]


def test_node_without_a_split_test_sends_every_point_left():
    # same tree, but the root's left child (leaves {0,1} and {2,3}) is made a node that split by
    # position (dimension -1), as nodes below depth 60 are.  Point 5 would pass its test to the
    # right (5 > 1.5); without a test it goes left, to {0,1}.
    X = np.arange(8, dtype=np.float32)[:, None]
    perm, off, nl, nodes, up = oracle.build_trees_nodes(X, 1, 2, 3)
    ids, _, _ = oracle.conquer_graph(X, perm, off, nl, nodes, up, 0, 6)
    assert sorted(int(v) for v in ids[5] if v >= 0) == [2, 3, 4, 6, 7]
    nodes = nodes.copy()
    nodes[0, 1]["dim"] = -1
    ids, _, _ = oracle.conquer_graph(X, perm, off, nl, nodes, up, 0, 6)
    assert sorted(int(v) for v in ids[5] if v >= 0) == [0, 1, 4, 6, 7]


def test_depth_at_or_below_every_leaf_is_the_leaf_step():
    X = synth.generate("gmm10k_d32", n=3000)
    perm, off, nl, nodes, up = oracle.build_trees_nodes(X, 3, 8, 42)
    p2, o2, n2 = oracle.build_trees(X, 3, 8, 42)
    assert np.array_equal(perm, p2) and np.array_equal(off, o2) and np.array_equal(nl, n2)
    deepest = max(int(nodes[t, 1:nl[t]]["depth"].max()) for t in range(3)) + 1
    a = oracle.conquer_graph(X, perm, off, nl, nodes, up, deepest, 10)
    b = oracle.init_graph(X, perm, off, nl, 10)
    for x, y in zip(a, b):
        assert x.tobytes() == y.tobytes()


def test_line_of_equal_leaves_gives_the_exact_graph():
    """1024 distinct values on a line, leaves of exactly 8 (a perfect tree: every mean split
    halves a run of consecutive integers).  Sent down a sibling subtree, a point lands in the
    leaf next to its own side, so conquering to the root collects both neighbouring leaves:
    with K <= 8 the result is the exact kNN graph."""
    rng = np.random.default_rng(3)
    order = rng.permutation(1024)
    X = order.astype(np.float32)[:, None]            # ids shuffled against values
    t = oracle.build_trees_nodes(X, 1, 8, 9)
    assert t[2][0] == 128 and np.all(np.diff(t[1][0, :129]) == 8)
    ids, dists, _ = oracle.conquer_graph(X, *t, 0, 8)
    tid, td = oracle.exact_knn_definition(X, 8)
    assert np.array_equal(ids, tid)
    assert np.array_equal(dists.astype(np.float64), td)
    # stopping one level below the root must lose neighbours across the middle
    ids1, _, _ = oracle.conquer_graph(X, *t, 1, 8)
    assert oracle.recall(ids1, tid) < 1.0


def python_candidates(X, perm, off, nl, nodes, up, dep, i):
    """Candidate set of point i by a separate walk in Python integers."""
    T, n = perm.shape
    out = set()
    for t in range(T):
        pos = int(np.nonzero(perm[t] == i)[0][0])
        leaf = int(np.searchsorted(off[t, :nl[t] + 1], pos, side="right") - 1)
        out.update(int(v) for v in perm[t, off[t, leaf]:off[t, leaf + 1]])
        link = int(up[t, leaf])
        while link >= 0:
            j, side = link >> 1, link & 1
            nd = nodes[t, j]
            if int(nd["depth"]) < dep:
                break
            c = int(nd["child"][1 - side])
            while c >= 0:
                m = nodes[t, c]
                left = int(m["dim"]) < 0 or int(m["cnt"]) * q(X[i, int(m["dim"])]) < int(m["sum"])
                c = int(m["child"][0 if left else 1])
            out.update(int(v) for v in perm[t, off[t, ~c]:off[t, ~c + 1]])
            pj = int(nd["parent"])
            link = -1 if pj < 0 else pj * 2 + (1 if int(nodes[t, pj]["child"][1]) == j else 0)
    out.discard(i)
    return sorted(out)


@pytest.mark.parametrize("name,n,T,S,K,dep", [
    ("gmm10k_d32", 2000, 3, 8, 10, 5),
    ("sift100k_like", 1500, 2, 16, 12, 3),     # integer data: exact distances, ties by id
    ("gmm10k_d32", 700, 2, 4, 6, 0),           # all the way to the root
])
def test_equals_exact_knn_over_rebuilt_candidate_sets(name, n, T, S, K, dep):
    X = synth.generate(name, n=n)
    t = oracle.build_trees_nodes(X, T, S, 42)
    rows = np.random.default_rng(1).choice(n, 60, replace=False)
    ids, dists, _ = oracle.conquer_graph(X, *t, dep, K, rows=rows)
    X64 = X.astype(np.float64)
    for r, i in enumerate(rows):
        cand = python_candidates(X, *t, dep, int(i))
        dd = ((X64[cand] - X64[i]) ** 2).sum(axis=1)
        if name == "sift100k_like":
            order = np.lexsort((cand, dd))[:K]
            want = [cand[o] for o in order]
            assert [int(v) for v in ids[r] if v >= 0] == want
        else:
            got = [int(v) for v in ids[r] if v >= 0]
            assert len(got) == min(K, len(cand)) and set(got) <= set(cand)
            kth = np.sort(dd)[len(got) - 1]
            assert np.all(dists[r, :len(got)].astype(np.float64) <= kth * (1 + 1e-5))


def test_structure_of_the_node_table():
    X = synth.generate("gmm10k_d32", n=4000)
    perm, off, nl, nodes, up = oracle.build_trees_nodes(X, 2, 8, 42)
    for t in range(2):
        L = int(nl[t])
        nd = nodes[t]
        seen_leaf = np.zeros(L, dtype=int)
        roots = 0
        for j in range(1, L):
            roots += int(nd[j]["parent"]) < 0
            for s in (0, 1):
                c = int(nd[j]["child"][s])
                if c >= 0:
                    assert int(nd[c]["parent"]) == j and int(nd[c]["depth"]) == int(nd[j]["depth"]) + 1
                else:
                    seen_leaf[~c] += 1
                    assert int(up[t, ~c]) == j * 2 + s
            # population = positions covered; the split test reproduces the partition
            lo = hi = j
            c = int(nd[j]["child"][0])
            while c >= 0:
                c = int(nd[c]["child"][0])
            lo = ~c
            c = int(nd[j]["child"][1])
            while c >= 0:
                c = int(nd[c]["child"][1])
            hi = ~c
            b, m, e = int(off[t, lo]), int(off[t, j]), int(off[t, hi + 1])
            assert int(nd[j]["cnt"]) == e - b
            dim = int(nd[j]["dim"])
            qs = [q(X[v, dim]) for v in perm[t, b:e]]
            assert int(nd[j]["sum"]) == sum(qs)
            left = [(e - b) * v < sum(qs) for v in qs]
            if any(left) and not all(left):
                assert left == [True] * (m - b) + [False] * (e - m)
        assert roots == 1 and np.all(seen_leaf == 1)


def test_candidates_grow_as_the_depth_drops():
    X = synth.generate("gmm10k_d32", n=3000)
    t = oracle.build_trees_nodes(X, 2, 8, 42)
    tid, _ = oracle.exact_knn(X, np.arange(3000), 10)
    last, first = -1.0, None
    for dep in (40, 8, 6, 4, 2, 0):
        ids, dists, _ = oracle.conquer_graph(X, *t, dep, 10)
        oracle.check_graph_invariants(X, ids, dists)
        r = oracle.recall(ids, tid)
        assert r >= last          # a superset of candidates cannot lose a true neighbour
        last = r
        first = r if first is None else first
    assert last > first + 0.2      # and conquering to the root finds many more of them
