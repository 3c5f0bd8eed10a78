"""Pins for the oracle's random-projection split (split_rule 2; the trees the paper's closing
section proposes for high dimensions): a node's test looks at a sum of eight signed coordinates
instead of one.  Everything is re-derived here in Python integers: the projection from the node's
draw, every split top-down, the sibling-subtree routing of the conquer step, and the best-bin-first
search over projection nodes."""
import heapq

import numpy as np
import pytest

import oracle
from paper_1609_07228_amd import synth

M64 = (1 << 64) - 1
GOLDEN = 0x9E3779B97F4A7C15
TERMS = 8


def mix64(z):
    z &= M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    return z ^ (z >> 31)


def q(x):
    return round(float(x) * 1048576.0)


def code_of(draw):
    return -3 - ((draw >> 34) & 0x3FFFFFFF)


def terms_of(code, d):
    r = -3 - code
    out = []
    for k in range(TERMS):
        z = mix64((r << 8) + k + GOLDEN)
        out.append((z % d, -1 if z >> 63 else 1))
    return out


def value(x, code):
    if code >= 0:
        return q(x[code])
    return sum(s * q(x[j]) for j, s in terms_of(code, len(x)))


def rederive(X, T, S, seed):
    n, d = X.shape
    perms, offs = [], []
    for t in range(T):
        out, off = [], []

        def rec(ids, h, depth):
            if len(ids) <= S:
                off.append(len(out))
                out.extend(ids)
                return
            code = code_of(oracle.node_rand(seed, t, h))
            vs = [value(X[i], code) for i in ids]
            tot = sum(vs)
            left = [i for i, v in zip(ids, vs) if len(ids) * v < tot]
            right = [i for i, v in zip(ids, vs) if not len(ids) * v < tot]
            if not left or not right:
                left, right = ids[:len(ids) // 2], ids[len(ids) // 2:]
            rec(left, 2 * h, depth + 1)
            rec(right, 2 * h + 1, depth + 1)

        rec(list(range(n)), 1, 0)
        off.append(n)
        perms.append(out)
        offs.append(off)
    return perms, offs


def test_mixer_is_the_published_one():
    # SplitMix64 seeded with 0: the first output is the finaliser of the golden constant
    assert mix64(GOLDEN) == 0xE220A8397B1DCDAF


@pytest.mark.parametrize("name,n,T,S", [("gmm10k_d32", 1500, 3, 8), ("sift100k_like", 1200, 2, 16),
                                         ("mixed4m_d96", 900, 2, 64)])
def test_rederivation_in_python_integers(name, n, T, S):
    X = synth.generate(name, n=n)
    perm, off, nl = oracle.build_trees(X, T=T, S=S, seed=synth.ALGO_SEED, split_rule=2)
    perms, offs = rederive(X, T, S, synth.ALGO_SEED)
    for t in range(T):
        assert perm[t].tolist() == perms[t]
        assert off[t, :nl[t] + 1].tolist() == offs[t]
    plain, _, _ = oracle.build_trees(X, T=T, S=S, seed=synth.ALGO_SEED)
    assert not np.array_equal(plain, perm)


def test_node_table_and_hand_cases():
    rng = np.random.default_rng(3)
    X = rng.standard_normal((800, 12)).astype(np.float32)
    perm, off, nl, nodes, up = oracle.build_trees_nodes(X, T=2, S=8, seed=9, split_rule=2)
    for t in range(2):
        for j in range(1, nl[t]):
            nd = nodes[t, j]
            code = int(nd["dim"])
            assert code <= -3 or code == -1
            # the segment of the node: from its leftmost to its rightmost leaf
            lo = hi = j
            c = int(nd["child"][0])
            while c >= 0:
                c = int(nodes[t, c]["child"][0])
            lo = ~c
            c = int(nd["child"][1])
            while c >= 0:
                c = int(nodes[t, c]["child"][1])
            hi = ~c
            ids = perm[t, off[t, lo]:off[t, hi + 1]]
            assert int(nd["cnt"]) == len(ids)
            if code <= -3:
                vs = [value(X[i], code) for i in ids]
                assert int(nd["sum"]) == sum(vs)
                left = perm[t, off[t, lo]:off[t, j]]
                if any(len(ids) * v < sum(vs) for v in vs) and not all(len(ids) * v < sum(vs) for v in vs):
                    assert all(len(ids) * value(X[i], code) < sum(vs) for i in left)
    # one dimension: every term is coordinate 0, the projection is (sum of signs) * q(x); where
    # the signs cancel the node is cut into positional halves, where they are negative the larger
    # values go left
    X = np.arange(16, dtype=np.float32).reshape(16, 1)
    for seed in range(8):
        perm, off, nl, nodes, up = oracle.build_trees_nodes(X, T=1, S=8, seed=seed, split_rule=2)
        code = code_of(oracle.node_rand(seed, 0, 1))
        net = sum(s for _, s in terms_of(code, 1))
        root = next(j for j in range(1, nl[0]) if nodes[0, j]["parent"] == -1)
        assert int(nodes[0, root]["dim"]) == code
        if net < 0:
            assert perm[0].tolist() == list(range(8, 16)) + list(range(8))
        else:      # positive: the smaller values go left; zero: positional halves, nothing moves
            assert perm[0].tolist() == list(range(16))
        assert nl[0] == 2 and off[0, :3].tolist() == [0, 8, 16]
    # the domain is eight times narrower
    big = np.full((1 << 21, 1), 2.0 ** 19, dtype=np.float32)
    oracle.build_trees(big[:4], 1, 2, 0, split_rule=2)
    with pytest.raises(ValueError):
        oracle.build_trees(big, 1, 1 << 21, 0, split_rule=2)
    oracle.build_trees(big, 1, 1 << 21, 0, split_rule=0)


def python_candidates(X, perm, off, nl, nodes, up, dep, i):
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
                left = int(m["dim"]) == -1 or int(m["cnt"]) * value(X[i], int(m["dim"])) < int(m["sum"])
                c = int(m["child"][0 if left else 1])
            out.update(int(v) for v in perm[t, off[t, ~c]:off[t, ~c + 1]])
            pj = int(nd["parent"])
            link = -1 if pj < 0 else pj * 2 + (1 if int(nodes[t, pj]["child"][1]) == j else 0)
    out.discard(i)
    return sorted(out)


def test_conquer_over_projection_nodes():
    X = synth.generate("sift100k_like", n=1500)      # integer data: exact distances, ties by id
    t = oracle.build_trees_nodes(X, 2, 16, 42, split_rule=2)
    rows = np.random.default_rng(1).choice(1500, 50, replace=False)
    K, dep = 12, 3
    ids, dists, _ = oracle.conquer_graph(X, *t, dep, K, rows=rows)
    X64 = X.astype(np.float64)
    for r, i in enumerate(rows):
        cand = python_candidates(X, *t, dep, int(i))
        dd = ((X64[cand] - X64[i]) ** 2).sum(axis=1)
        order = np.lexsort((cand, dd))[:K]
        assert [int(v) for v in ids[r] if v >= 0] == [cand[o] for o in order]


def python_leaves(qv, nodes, n_leaves, want):
    if n_leaves == 1:
        return [0]
    root = next(j for j in range(1, n_leaves) if int(nodes[j]["parent"]) < 0)
    heap, found, link, prio = [], [], root, 0.0
    while len(found) < want:
        while link >= 0:
            nd = nodes[link]
            code, cnt, sm = int(nd["dim"]), int(nd["cnt"]), int(nd["sum"])
            if code != -1:
                diff = cnt * value(qv, code) - sm
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


def test_search_over_projection_nodes():
    n, T, S, P = 2000, 2, 16, 100
    X = synth.generate("sift100k_like", n=n)
    rng = np.random.default_rng(5)
    Q = np.round(X[rng.choice(n, 30)] + 3 * rng.standard_normal((30, X.shape[1]))).astype(np.float32)
    t = oracle.build_trees_nodes(X, T, S, 42, split_rule=2)
    g = oracle.init_graph(X, t[0], t[1], t[2], 10)
    want_leaves = P // S // T + 1
    ids, dists, checked = oracle.search(X, t[0], t[1], t[2], t[3], S, g[0], Q, 10, P, P, 0)
    for qi in range(Q.shape[0]):
        cand = set()
        for tr in range(T):
            for leaf in python_leaves(Q[qi], t[3][tr], int(t[2][tr]), want_leaves):
                cand.update(int(v) for v in t[0][tr, t[1][tr, leaf]:t[1][tr, leaf + 1]])
        cand = sorted(cand)
        assert checked[qi] == len(cand)
        dd = ((X[cand].astype(np.float64) - Q[qi].astype(np.float64)) ** 2).sum(1)
        order = np.lexsort((cand, dd))[:10]
        assert [int(v) for v in ids[qi] if v >= 0] == [cand[o] for o in order]
