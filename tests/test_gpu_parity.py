"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the
same seeded inputs.  Integer / index results must agree bit for bit; the library's
distances use the same fixed order of float32 operations as the oracle, so they agree
bit for bit as well (which is stronger than the 1e-5 relative bound that is also
checked against float64)."""
import numpy as np
import pytest

import oracle
from paper_1609_07228_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ef():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: there is no CPU fallback")
    from paper_1609_07228_amd import efanna
    efanna.lib()
    return efanna


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def host(t):
    return t.cpu().numpy()


def trees_equal(ef, X, T, S, seed):
    perm, off, nl = ef.efanna_build_trees(dev(X), T, S, seed)
    operm, ooff, onl = oracle.build_trees(X, T, S, seed)
    assert np.array_equal(nl, onl)
    assert np.array_equal(host(perm), operm)
    goff = host(off)
    for t in range(T):
        assert np.array_equal(goff[t, :nl[t] + 1], ooff[t, :onl[t] + 1])
    return (perm, off, nl), (operm, ooff, onl)


# ---------------------------------------------------------------------------------
def test_pair_distances_bit_exact(ef):
    rng = np.random.default_rng(0)
    for d in (1, 5, 16, 31, 32, 96, 128, 960, 1000):
        X = (rng.standard_normal((300, d)) * rng.choice([0.01, 1.0, 100.0], (300, 1))).astype(np.float32)
        a = rng.integers(0, 300, 777).astype(np.int32)
        b = rng.integers(0, 300, 777).astype(np.int32)
        got = host(ef.efanna_pair_distances(dev(X), dev(a), dev(b)))
        want = np.array([oracle.dist(X[i], X[j]) for i, j in zip(a, b)], dtype=np.float32)
        assert got.tobytes() == want.tobytes(), f"d={d}"
        ref = ((X[a].astype(np.float64) - X[b].astype(np.float64)) ** 2).sum(axis=1)
        assert np.all(np.abs(got - ref) <= 1e-5 * ref)


@pytest.mark.parametrize("name,n,T,S", [
    ("gmm10k_d32", 10_000, 4, 8),          # the small configuration, full size
    ("gmm10k_d32", 4_097, 3, 5),           # ragged sizes
    ("sift100k_like", 30_000, 8, 16),
    ("mixed4m_d96", 20_000, 16, 64),
    ("gist1m_like", 3_000, 2, 16),
])
def test_trees_bit_exact(ef, name, n, T, S):
    X = synth.generate(name, n=n)
    trees_equal(ef, X, T, S, synth.ALGO_SEED)


def test_trees_edge_cases(ef):
    rng = np.random.default_rng(3)
    # n <= S: one leaf per tree
    X = rng.standard_normal((7, 3)).astype(np.float32)
    trees_equal(ef, X, 2, 7, 0)
    # all points equal: positional halves everywhere
    trees_equal(ef, np.full((1000, 4), 2.5, dtype=np.float32), 2, 3, 5)
    # heavy ties on an integer grid, leaf size 1, d = 1
    trees_equal(ef, rng.integers(0, 4, (5000, 1)).astype(np.float32), 3, 1, 9)
    # strongly skewed data: deep unbalanced trees
    trees_equal(ef, np.exp(rng.standard_normal((20000, 2)) * 4).astype(np.float32).clip(0, 1e5), 2, 4, 1)


def test_trees_reject_bad_input(ef):
    X = np.zeros((100, 4), dtype=np.float32)
    X[17, 2] = np.nan
    with pytest.raises(ef.EfannaError) as e:
        ef.efanna_build_trees(dev(X), 2, 4, 0)
    assert e.value.status == -3
    X[17, 2] = 2.0 ** 21
    with pytest.raises(ef.EfannaError) as e:
        ef.efanna_build_trees(dev(X), 2, 4, 0)
    assert e.value.status == -3
    X[17, 2] = 0
    # beyond 2^23 points n * |x| < 2^43 binds before |x| < 2^20 (64-bit sums of the exact mean test)
    big = torch.zeros(((1 << 24) + 3, 1), dtype=torch.float32, device="cuda:0")
    big[12345, 0] = 2.0 ** 19
    with pytest.raises(ef.EfannaError) as e:
        ef.efanna_build_trees(big, 1, 64, 0, max_leaves=(1 << 20))
    assert e.value.status == -3
    del big
    with pytest.raises(ef.EfannaError) as e:
        ef.efanna_build_trees(dev(X), 2, 4, 0, workspace=torch.empty(256, dtype=torch.uint8, device="cuda:0"))
    assert e.value.status == -2
    with pytest.raises(ef.EfannaError) as e:
        ef.efanna_build_trees(dev(X), 2, 4, 0, max_leaves=3)
    assert e.value.status == -5


def graph_equal(ef, graph, want):
    ids, dists, flags = ef.efanna_get_graph(graph, with_flags=True)
    ids, dists, flags = host(ids), host(dists), host(flags)
    assert np.array_equal(ids, want[0])
    assert dists.tobytes() == want[1].tobytes()
    assert np.array_equal(flags, want[2])
    return ids, dists


@pytest.mark.parametrize("name,n,T,S,K", [
    ("gmm10k_d32", 10_000, 4, 8, 10),
    ("sift100k_like", 20_000, 8, 16, 20),
    ("mixed4m_d96", 12_000, 4, 64, 100),
    ("gist1m_like", 3_000, 3, 16, 10),
    ("gmm10k_d32", 1_003, 2, 3, 16),       # mostly under-full rows
])
def test_init_graph_bit_exact(ef, name, n, T, S, K):
    X = synth.generate(name, n=n)
    (perm, off, nl), (operm, ooff, onl) = trees_equal(ef, X, T, S, synth.ALGO_SEED)
    graph = ef.efanna_init_graph(dev(X), perm, off, nl, S, K)
    want = oracle.init_graph(X, operm, ooff, onl, K)
    ids, dists = graph_equal(ef, graph, want)
    oracle.check_graph_invariants(X, ids, dists)


def test_init_graph_odd_dimension_and_single_leaf(ef):
    rng = np.random.default_rng(5)
    X = rng.standard_normal((40, 21)).astype(np.float32)
    (perm, off, nl), (operm, ooff, onl) = trees_equal(ef, X, 1, 64, 0)
    assert nl[0] == 1
    graph = ef.efanna_init_graph(dev(X), perm, off, nl, 64, 7)
    want = oracle.init_graph(X, operm, ooff, onl, 7)
    ids, _ = graph_equal(ef, graph, want)
    tid, _ = oracle.exact_knn_definition(X, 7)
    assert np.array_equal(ids, tid)          # one leaf holding everything: the exact graph


@pytest.mark.parametrize("d,S,K,T", [
    (4, 16, 3, 3),          # one 16-byte piece per row
    (20, 16, 10, 4),        # d a multiple of 4 but not of 16: ragged last piece
    (100, 13, 10, 3),
    (128, 16, 40, 5),       # K above the number of leaf mates of one tree: rows fill up over trees
    (64, 2, 5, 6),          # leaves of one or two points
    (200, 16, 10, 3),       # more than one 128-coordinate piece, the last one ragged
])
def test_init_graph_small_leaf_shapes(ef, d, S, K, T):
    """Leaves of at most 16 points with d <= 128 take the kernel that keeps rows in registers."""
    rng = np.random.default_rng(d * 131 + S)
    X = rng.standard_normal((5_003, d)).astype(np.float32)
    X[100:140] = X[100]                      # equal points: zero distances, ties broken by id
    (perm, off, nl), (operm, ooff, onl) = trees_equal(ef, X, T, S, 11)
    graph = ef.efanna_init_graph(dev(X), perm, off, nl, S, K)
    want = oracle.init_graph(X, operm, ooff, onl, K)
    ids, dists = graph_equal(ef, graph, want)
    oracle.check_graph_invariants(X, ids, dists)


def tree_nodes_equal(ef, X, T, S, seed, split_rule=None):
    if split_rule is None:
        perm, off, nl, nodes, up, depth = ef.efanna_build_trees(dev(X), T, S, seed, with_nodes=True)
    else:
        perm, off, nl, nodes, up, depth = ef.efanna_build_trees_rule(dev(X), T, S, seed, split_rule, with_nodes=True)
    operm, ooff, onl, onodes, oup = oracle.build_trees_nodes(X, T, S, seed, split_rule or 0)
    assert depth == max([int(onodes[t, 1:onl[t]]["depth"].max()) for t in range(T) if onl[t] > 1], default=-1)
    assert np.array_equal(nl, onl) and np.array_equal(host(perm), operm)
    gn = host(nodes).view(oracle.NODE_DTYPE)[..., 0]
    gu = host(up)
    for t in range(T):
        L = int(nl[t])
        assert np.array_equal(host(off)[t, :L + 1], ooff[t, :L + 1])
        assert gn[t, 1:L].tobytes() == onodes[t, 1:L].tobytes()
        assert np.array_equal(gu[t, :L], oup[t, :L])
    return (perm, off, nl, nodes, up, depth), (operm, ooff, onl, onodes, oup)


@pytest.mark.parametrize("name,n,T,S", [
    ("gmm10k_d32", 10_000, 4, 8),
    ("sift100k_like", 30_000, 3, 16),      # nodes from the device-wide levels and from the in-LDS finish
    ("mixed4m_d96", 20_000, 2, 64),
    ("gmm10k_d32", 1_003, 2, 1),           # leaves of one point: deepest trees
])
def test_tree_nodes_bit_exact(ef, name, n, T, S):
    tree_nodes_equal(ef, synth.generate(name, n=n), T, S, synth.ALGO_SEED)


@pytest.mark.parametrize("name,n,T,S", [
    ("gmm10k_d32", 10_000, 4, 8),
    ("sift100k_like", 40_000, 3, 16),      # device-wide levels and the in-LDS finish
    ("mixed4m_d96", 20_000, 2, 64),
    ("gist1m_like", 3_000, 2, 16),         # fifteen dimensions per lane
    ("gmm10k_d32", 1_003, 2, 1),
])
def test_trees_variance_rule_bit_exact(ef, name, n, T, S):
    X = synth.generate(name, n=n)
    g, _ = tree_nodes_equal(ef, X, T, S, synth.ALGO_SEED, split_rule=1)
    plain = ef.efanna_build_trees(dev(X), T, S, synth.ALGO_SEED)
    same = ef.efanna_build_trees_rule(dev(X), T, S, synth.ALGO_SEED, 0)
    assert torch.equal(plain[0], same[0]) and not torch.equal(plain[0], g[0])


@pytest.mark.parametrize("name,n,T,S", [
    ("gmm10k_d32", 10_000, 4, 8),
    ("sift100k_like", 40_000, 3, 16),      # device-wide levels and the in-LDS finish
    ("mixed4m_d96", 20_000, 2, 64),
    ("gist1m_like", 3_000, 2, 16),
    ("gmm10k_d32", 1_003, 2, 1),
])
def test_trees_projection_rule_bit_exact(ef, name, n, T, S):
    X = synth.generate(name, n=n)
    g, _ = tree_nodes_equal(ef, X, T, S, synth.ALGO_SEED, split_rule=2)
    plain = ef.efanna_build_trees(dev(X), T, S, synth.ALGO_SEED)
    assert not torch.equal(plain[0], g[0])


def test_projection_rule_conquer_search_and_limits(ef):
    rng = np.random.default_rng(41)
    for n, d in ((700, 1), (2_500, 3), (5_000, 70)):      # one dimension: signs may cancel (positional halves)
        X = rng.standard_normal((n, d)).astype(np.float32)
        tree_nodes_equal(ef, X, 2, 6, 9, split_rule=2)
    # the conquer step and the search route through projection nodes
    X = synth.generate("sift100k_like", n=8_000)
    g, o = tree_nodes_equal(ef, X, 3, 16, 5, split_rule=2)
    for S, K, dep in ((16, 12, 7),):
        graph = ef.efanna_init_graph(dev(X), g[0], g[1], g[2], S, K, nodes=g[3], leaf_up=g[4], tree_depth=g[5],
                                     conquer_depth=dep)
        graph_equal(ef, graph, oracle.conquer_graph(X, *o, dep, K))
    Xm = synth.generate("mixed4m_d96", n=5_000)           # the general conquer kernels
    gm, om = tree_nodes_equal(ef, Xm, 2, 40, 5, split_rule=2)
    graph = ef.efanna_init_graph(dev(Xm), gm[0], gm[1], gm[2], 40, 24, nodes=gm[3], leaf_up=gm[4], tree_depth=gm[5],
                                 conquer_depth=4)
    graph_equal(ef, graph, oracle.conquer_graph(Xm, *om, 4, 24))
    K = 10
    graph = ef.efanna_init_graph(dev(X), g[0], g[1], g[2], 16, K)
    ids = ef.efanna_get_graph(graph)[0]
    Q = np.round(X[rng.choice(8_000, 300)] + 3 * rng.standard_normal((300, X.shape[1]))).astype(np.float32)
    got = ef.efanna_search(dev(X), g[0], g[1], g[2], g[3], g[5], 16, ids, dev(Q), K, 100, 50, 3)
    want = oracle.search(X, o[0], o[1], o[2], o[3], 16, host(ids), Q, K, 100, 50, 3)
    assert np.array_equal(host(got[0]), want[0]) and np.array_equal(host(got[1]), want[1])
    assert np.array_equal(host(got[2]), want[2])
    # the domain is eight times narrower: 2^19 * 2^21 * 8 = 2^43
    big = torch.full((1 << 21, 1), 2.0 ** 19, dtype=torch.float32, device="cuda")
    with pytest.raises(ef.EfannaError) as e:
        ef.efanna_build_trees_rule(big, 1, 64, 0, 2)
    assert e.value.status == -3
    ef.efanna_build_trees_rule(big, 1, 64, 0, 0)


def test_trees_variance_rule_shapes(ef):
    rng = np.random.default_rng(31)
    for n, d in ((700, 3), (2_500, 5), (5_000, 70), (300, 1)):      # fewer than five dimensions; a ragged last lane round
        X = rng.standard_normal((n, d)).astype(np.float32)
        tree_nodes_equal(ef, X, 2, 6, 9, split_rule=1)
    X = (rng.integers(-2**19, 2**19, size=(6_000, 8)).astype(np.float32) + 0.5)      # squares beyond 64 bits
    X[:, 5] *= 1e-3
    tree_nodes_equal(ef, X, 2, 10, 2, split_rule=1)
    X = np.repeat(rng.standard_normal((40, 6)).astype(np.float32), 100, axis=0)      # equal points: zero variances, ties
    tree_nodes_equal(ef, X, 2, 16, 4, split_rule=1)
    with pytest.raises(ef.EfannaError) as e:
        ef.efanna_build_trees_rule(dev(X), 2, 16, 4, 3)
    assert e.value.status == -1


def test_tree_nodes_edge_cases(ef):
    X = np.zeros((300, 4), dtype=np.float32)                    # every split positional
    tree_nodes_equal(ef, X, 2, 4, 5)
    X = np.arange(40, dtype=np.float32).reshape(10, 4)
    (_, _, nl, _, up, depth), _ = tree_nodes_equal(ef, X, 3, 16, 1)    # a single leaf: no nodes at all
    assert list(nl) == [1, 1, 1] and host(up)[0, 0] == -1 and depth == -1


@pytest.mark.parametrize("name,n,T,S,K,deps", [
    ("gmm10k_d32", 6_000, 3, 8, 10, (0, 5, 9, 99)),
    ("sift100k_like", 8_000, 4, 16, 20, (7,)),       # integer data: ties, points found again in other trees
    ("gmm10k_d32", 1_003, 2, 3, 16, (0,)),           # up to the root, rows that stay under-full
    ("mixed4m_d96", 9_001, 2, 64, 100, (0, 4, 99)),  # leaves of more than 16 points: the general kernels
    ("mixed4m_d96", 5_000, 3, 40, 24, (3,)),
    ("gist1m_like", 3_000, 2, 33, 12, (2,)),         # d = 960, rows wider than a leaf
])
def test_conquer_above_the_leaves_bit_exact(ef, name, n, T, S, K, deps):
    X = synth.generate(name, n=n)
    g, o = tree_nodes_equal(ef, X, T, S, synth.ALGO_SEED)
    for dep in deps:
        graph = ef.efanna_init_graph(dev(X), g[0], g[1], g[2], S, K, nodes=g[3], leaf_up=g[4],
                                     tree_depth=g[5], conquer_depth=dep)
        want = oracle.conquer_graph(X, *o, dep, K)
        ids, dists = graph_equal(ef, graph, want)
        oracle.check_graph_invariants(X, ids, dists)
    # a depth below every leaf is the leaf step
    plain = ef.efanna_init_graph(dev(X), g[0], g[1], g[2], S, K)
    deep = ef.efanna_init_graph(dev(X), g[0], g[1], g[2], S, K, nodes=g[3], leaf_up=g[4], tree_depth=g[5],
                                conquer_depth=10_000)
    assert torch.equal(ef.efanna_get_graph(plain)[0], ef.efanna_get_graph(deep)[0])


def test_conquer_shapes_and_limits(ef):
    rng = np.random.default_rng(21)
    X = rng.standard_normal((4_001, 200)).astype(np.float32)     # two 128-coordinate pieces, ragged
    g, o = tree_nodes_equal(ef, X, 2, 13, 3)
    graph = ef.efanna_init_graph(dev(X), g[0], g[1], g[2], 13, 10, nodes=g[3], leaf_up=g[4], tree_depth=g[5],
                                 conquer_depth=4)
    graph_equal(ef, graph, oracle.conquer_graph(X, *o, 4, 10))
    for n, d, S, K, dep in ((2_000, 8, 64, 10, 0), (3_001, 30, 40, 48, 5), (1_500, 7, 12, 9, 3), (900, 3, 5, 70, 1)):
        X = rng.standard_normal((n, d)).astype(np.float32)       # d not a multiple of 4, K above the leaf size
        g, o = tree_nodes_equal(ef, X, 2, S, 3)
        graph = ef.efanna_init_graph(dev(X), g[0], g[1], g[2], S, K, nodes=g[3], leaf_up=g[4], tree_depth=g[5],
                                     conquer_depth=dep)
        ids, dists = graph_equal(ef, graph, oracle.conquer_graph(X, *o, dep, K))
        oracle.check_graph_invariants(X, ids, dists)


@pytest.mark.parametrize("name,n,T,S,K,L,I", [
    ("gmm10k_d32", 10_000, 4, 8, 10, 10, 4),      # the small configuration as quoted
    ("sift100k_like", 20_000, 8, 16, 20, 20, 3),
    ("mixed4m_d96", 6_000, 4, 64, 100, 50, 2),
    ("gist1m_like", 2_000, 3, 16, 10, 10, 2),
    ("gmm10k_d32", 3_001, 2, 8, 12, 5, 3),        # L < K: marks survive an iteration
])
def test_nndescent_bit_exact_every_iteration(ef, name, n, T, S, K, L, I):
    X = synth.generate(name, n=n)
    Xd = dev(X)
    (perm, off, nl), (operm, ooff, onl) = trees_equal(ef, X, T, S, synth.ALGO_SEED)
    graph = ef.efanna_init_graph(Xd, perm, off, nl, S, K)
    want = oracle.init_graph(X, operm, ooff, onl, K)
    for it in range(I):
        stats = ef.efanna_nndescent(Xd, graph, 1, L, synth.ALGO_SEED, first_iter=it)
        want = oracle.nndescent(X, *want[:3], 1, L, synth.ALGO_SEED, iter0=it)
        ids, dists = graph_equal(ef, graph, want)
        assert int(host(stats)[0, 0]) == int(want[3][0, 0])      # same pairs evaluated
    oracle.check_graph_invariants(X, ids, dists)


def filter_data(kind, n, d):
    """Data that strains the joins' half-precision Gram filter (a filter that drops a pair it must
    keep shows as a row that differs from the oracle's)."""
    rng = np.random.default_rng(97)
    X = rng.standard_normal((n, d)).astype(np.float32)
    if kind == "large":            # coordinates up to 2^19: scaled down before rounding
        X = X * np.float32(90_000.0)
    elif kind == "just_below":     # largest coordinate just under 2^15: not scaled
        X = X * np.float32(32_000.0 / np.abs(X).max())
    elif kind == "tiny":           # below the smallest normal half-precision number
        X = X * np.float32(3e-6)
    elif kind == "offset":         # norms a thousand times the distances
        X = X + np.float32(900.0)
    elif kind == "far_offset":     # neighbouring points round to the same few half-precision values
        X = X + np.float32(30_000.0)
    elif kind == "outlier":        # one huge coordinate sets the scale, the rest turn subnormal
        X[17, 3] = np.float32(500_000.0)
    elif kind == "integers":       # heavy ties, many zero distances
        X = rng.integers(0, 3, size=(n, d)).astype(np.float32)
    elif kind == "mixed_scales":   # every dimension its own magnitude, 2^-12 .. 2^12
        X = X * np.exp2(rng.integers(-12, 13, size=d)).astype(np.float32)
    return X


@pytest.mark.parametrize("kind", ["large", "just_below", "tiny", "offset", "far_offset", "outlier", "integers",
                                  "mixed_scales"])
@pytest.mark.parametrize("d,K,L", [(128, 10, 10), (36, 10, 16)])      # joins of at most 16 and of 17..32 vectors
def test_nndescent_filter_ranges_bit_exact(ef, kind, d, K, L):
    n, T, S, I = 6_000, 3, 16, 4
    X = filter_data(kind, n, d)
    Xd = dev(X)
    (perm, off, nl), (operm, ooff, onl) = trees_equal(ef, X, T, S, synth.ALGO_SEED)
    graph = ef.efanna_init_graph(Xd, perm, off, nl, S, K)
    want = oracle.init_graph(X, operm, ooff, onl, K)
    for it in range(I):
        ef.efanna_nndescent(Xd, graph, 1, L, synth.ALGO_SEED, first_iter=it)
        want = oracle.nndescent(X, *want[:3], 1, L, synth.ALGO_SEED, iter0=it)
        graph_equal(ef, graph, want)


@pytest.mark.parametrize("n,d,T,S,K,L,I", [
    (3_000, 200, 2, 12, 8, 8, 3),        # long vectors with a ragged last piece (128 + 72): joins by rotations
    (2_500, 132, 2, 16, 10, 10, 2),      # just over one piece
    (3_000, 16, 2, 16, 50, 50, 2),       # rows and lists of exactly fifty entries: one wide read
    (3_000, 16, 2, 16, 52, 25, 2),       # fifty and a remainder of two
    (2_000, 24, 2, 8, 7, 9, 3),          # odd row length (rows not 16-byte aligned), L > K
    (12, 4, 2, 3, 10, 10, 3),            # hardly more points than K (the library wants k < n)
    (33, 8, 1, 64, 5, 5, 2),             # one leaf holds everything
    (65, 4, 3, 1, 4, 2, 4),              # leaves of one point: the initial graph is empty
    (1_025, 8, 2, 16, 10, 10, 3),        # reverse lists by target ranges of 1024: a second range of one point
    (5_000, 8, 2, 16, 16, 16, 2),        # the longest lists with ranges of 1024, a ragged last range
    (2_100, 8, 2, 16, 16, 17, 2),        # one more: ranges of 512 targets
    (3_000, 8, 2, 16, 32, 32, 2),        # the longest rows and lists that scheme takes
    (2_000, 8, 2, 16, 33, 16, 1),        # one more: lists by counters
    (4_096, 12, 2, 16, 3, 1, 4),         # lists of a single key
    (2_000, 16, 2, 16, 64, 32, 2),       # join lists of 128 ids: a wave per point, hash table of 256 slots
    (1_500, 8, 2, 16, 128, 64, 1),       # the longest rows and samples the library takes (lists of 256 ids)
    (1_200, 20, 2, 16, 40, 29, 2),       # lists of 98 ids: just over the switch to a wave per point
])
def test_nndescent_more_shapes(ef, n, d, T, S, K, L, I):
    rng = np.random.default_rng(n + d + K)
    X = rng.standard_normal((n, d)).astype(np.float32)
    Xd = dev(X)
    (perm, off, nl), (operm, ooff, onl) = trees_equal(ef, X, T, S, 11)
    graph = ef.efanna_init_graph(Xd, perm, off, nl, S, K)
    want = oracle.init_graph(X, operm, ooff, onl, K)
    for it in range(I):
        stats = ef.efanna_nndescent(Xd, graph, 1, L, 11, first_iter=it)
        want = oracle.nndescent(X, *want[:3], 1, L, 11, iter0=it)
        ids, dists = graph_equal(ef, graph, want)
        assert int(host(stats)[0, 0]) == int(want[3][0, 0])
    oracle.check_graph_invariants(X, ids, dists)


@pytest.mark.parametrize("n,d,T,S,K,L,I", [
    (6_000, 32, 3, 8, 10, 10, 4),        # joins of at most 16 and of 17..32 vectors, rows of ten
    (4_000, 128, 2, 16, 20, 20, 3),      # tile joins (more than 32 vectors of up to 128 coordinates)
    (3_000, 200, 2, 12, 8, 8, 3),        # long vectors: joins by rotations
    (3_000, 160, 2, 16, 24, 16, 3),      # long vectors and more than 32 of them: rows in LDS
    (2_000, 24, 2, 8, 7, 9, 3),          # odd row length
    (4_000, 16, 2, 16, 50, 25, 3),       # L < K: unsampled entries keep their new mark through the join
])
def test_nndescent_literal_marking_bit_exact(ef, n, d, T, S, K, L, I):
    """The literal marking of Alg. 4's second inner loop (cross_old): entries that a new and an old
    member insert are marked old, pairs of two new members going first.  Ids, distance bits, marks
    and pairs evaluated equal the oracle's after every iteration, in every join kernel."""
    rng = np.random.default_rng(n + d)
    X = (rng.standard_normal((n, d)) + 3.0 * rng.integers(0, 5, (n, 1))).astype(np.float32)
    Xd = dev(X)
    (perm, off, nl), (operm, ooff, onl) = trees_equal(ef, X, T, S, 11)
    graph = ef.efanna_init_graph(Xd, perm, off, nl, S, K)
    want = oracle.init_graph(X, operm, ooff, onl, K)
    marks = []
    for it in range(I):
        stats = ef.efanna_nndescent(Xd, graph, 1, L, 11, first_iter=it, cross_old=True)
        want = oracle.nndescent(X, *want[:3], 1, L, 11, iter0=it, cross_old=True)
        graph_equal(ef, graph, want)
        assert int(host(stats)[0, 0]) == int(want[3][0, 0])
        marks.append(int(want[2].sum()))
    # and all iterations in one call (the passes alternate inside the library)
    graph2 = ef.efanna_init_graph(Xd, perm, off, nl, S, K)
    ef.efanna_nndescent(Xd, graph2, I, L, 11, cross_old=True)
    graph_equal(ef, graph2, want)
    assert any(want[2].ravel() == 0) and marks[-1] < marks[0]


@pytest.mark.parametrize("hubs", [
    [0, 1500, 3000, 4500],      # spread over the ranges of 1024 targets
    [3, 200, 700, 1023],        # all in one range: twenty thousand offers for its thousand lists
])
def test_reverse_lists_of_popular_points(ef, hubs):
    """A few points that are everybody's neighbours: their reverse lists are offered thousands of
    keys, from every block of source rows, and keep the L smallest."""
    rng = np.random.default_rng(5)
    n, d, K, L = 6_000, 32, 10, 10
    X = rng.standard_normal((n, d)).astype(np.float32)      # a Gaussian cloud in 32 dimensions: its points
    X[hubs] = (0.01 * rng.standard_normal((4, d))).astype(np.float32)     # are closer to its centre than to each other
    Xd = dev(X)
    (perm, off, nl), (operm, ooff, onl) = trees_equal(ef, X, 3, 16, 3)
    graph = ef.efanna_init_graph(Xd, perm, off, nl, 16, K)
    want = oracle.init_graph(X, operm, ooff, onl, K)
    for it in range(4):
        ef.efanna_nndescent(Xd, graph, 1, L, 3, first_iter=it)
        want = oracle.nndescent(X, *want[:3], 1, L, 3, iter0=it)
        ids, dists = graph_equal(ef, graph, want)
    indeg = np.bincount(ids.ravel(), minlength=n)
    assert indeg[hubs].min() > 1000      # the case is what it says
    oracle.check_graph_invariants(X, ids, dists)


def test_nndescent_resume_and_recall(ef):
    name = "gmm10k_d32"
    p = synth.params(name)
    X = synth.generate(name)
    Xd = dev(X)
    perm, off, nl = ef.efanna_build_trees(Xd, p["T"], p["S"], synth.ALGO_SEED)
    g1 = ef.efanna_init_graph(Xd, perm, off, nl, p["S"], p["K"])
    g2 = g1.clone()
    ef.efanna_nndescent(Xd, g1, p["I"], p["L"], synth.ALGO_SEED)
    for it in range(p["I"]):
        ef.efanna_nndescent(Xd, g2, 1, p["L"], synth.ALGO_SEED, first_iter=it)
    a, b = ef.efanna_get_graph(g1), ef.efanna_get_graph(g2)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    # recall against exact brute force equals the oracle's (the graphs are identical)
    operm, ooff, onl = oracle.build_trees(X, p["T"], p["S"], synth.ALGO_SEED)
    og = oracle.nndescent(X, *oracle.init_graph(X, operm, ooff, onl, p["K"]), p["I"], p["L"],
                          synth.ALGO_SEED)
    tid, _ = oracle.exact_knn(X, np.arange(X.shape[0]), p["K"])
    r_gpu, r_cpu = oracle.recall(host(a[0]), tid), oracle.recall(og[0], tid)
    assert abs(r_gpu - r_cpu) <= 0.005 and r_gpu > 0.8


def test_early_termination_and_larger_pools(ef):
    """delta > 0 stops where the oracle stops; a pool larger than the graph degree (P > K) is a
    run with k = P whose rows are cut to K at the end."""
    X = synth.generate("gmm10k_d32", n=6000)
    Xd = dev(X)
    K, P, L = 10, 15, 10
    (perm, off, nl), (operm, ooff, onl) = trees_equal(ef, X, 3, 8, synth.ALGO_SEED)
    for delta in (0.05, 0.004):
        graph = ef.efanna_init_graph(Xd, perm, off, nl, 8, P)
        stats, done = ef.efanna_nndescent(Xd, graph, 12, L, synth.ALGO_SEED, delta=delta)
        want = oracle.nndescent(X, *oracle.init_graph(X, operm, ooff, onl, P), 12, L, synth.ALGO_SEED,
                                delta=delta)
        assert done == want[4] and 1 <= done < 12 and stats.shape[0] == done
        ids, dists = graph_equal(ef, graph, want)
        assert np.array_equal(host(stats)[:, 0].astype(np.uint64), want[3][:, 0])
    tid, _ = oracle.exact_knn(X, np.arange(X.shape[0]), K)
    assert oracle.recall(ids[:, :K], tid) > 0.85          # the K closest of the P kept


def build_index(ef, X, T, S, K, iters, seed=synth.ALGO_SEED):
    g, o = tree_nodes_equal(ef, X, T, S, seed)
    Xd = dev(X)
    graph = ef.efanna_init_graph(Xd, g[0], g[1], g[2], S, K)
    if iters:
        ef.efanna_nndescent(Xd, graph, iters, K, seed)
    ids, _ = ef.efanna_get_graph(graph)
    og = oracle.init_graph(X, o[0], o[1], o[2], K)
    if iters:
        og = oracle.nndescent(X, *og, iters, K, seed)
    assert np.array_equal(host(ids), og[0])
    return Xd, g, o, ids


@pytest.mark.parametrize("name,n,T,S,K,P,E,I", [
    ("gmm10k_d32", 6_000, 4, 8, 10, 60, 20, 4),
    ("sift100k_like", 8_000, 4, 16, 20, 200, 50, 3),     # integer data: ties by id
    ("gmm10k_d32", 3_000, 3, 8, 10, 40, 40, 0),          # the trees alone
    ("gmm10k_d32", 2_000, 2, 4, 6, 7, 3, 6),             # one leaf per tree, a pool of 7 that keeps moving
])
def test_search_bit_exact(ef, name, n, T, S, K, P, E, I):
    X = synth.generate(name, n=n)
    Xd, g, o, ids = build_index(ef, X, T, S, K, 3)
    rng = np.random.default_rng(n + P)
    Q = (X[rng.choice(n, 300)] + rng.standard_normal((300, X.shape[1])) * np.float32(0.5)).astype(np.float32)
    Q[:20] = X[rng.choice(n, 20)]                          # some queries are data points
    kq = min(K, P)
    got = ef.efanna_search(Xd, g[0], g[1], g[2], g[3], g[5], S, ids, dev(Q), kq, P, E, I)
    want = oracle.search(X, o[0], o[1], o[2], o[3], S, host(ids), Q, kq, P, E, I)
    assert np.array_equal(host(got[0]), want[0])
    assert host(got[1]).tobytes() == want[1].tobytes()
    assert np.array_equal(host(got[2]), want[2])


def test_search_edge_cases(ef):
    rng = np.random.default_rng(4)
    X = rng.standard_normal((50, 8)).astype(np.float32)            # every tree a single leaf
    Xd, g, o, ids = build_index(ef, X, 2, 64, 5, 0)
    Q = rng.standard_normal((7, 8)).astype(np.float32)
    got = ef.efanna_search(Xd, g[0], g[1], g[2], g[3], g[5], 64, ids, dev(Q), 5, 50, 50, 1)
    want = oracle.search(X, o[0], o[1], o[2], o[3], 64, host(ids), Q, 5, 50, 50, 1)
    assert np.array_equal(host(got[0]), want[0]) and host(got[1]).tobytes() == want[1].tobytes()
    tid, _ = oracle.exact_knn_definition(np.vstack([X, Q[:1]]), 5)   # brute force for the first query
    d2 = ((X.astype(np.float64) - Q[0].astype(np.float64)) ** 2).sum(1)
    assert list(host(got[0])[0]) == list(np.lexsort((np.arange(50), d2))[:5])
    # rows of the graph with empty slots, k larger than what can be found
    X = synth.generate("gmm10k_d32", n=1_003)
    Xd, g, o, ids = build_index(ef, X, 2, 3, 16, 0)
    Q = X[:40] + np.float32(0.01)
    got = ef.efanna_search(Xd, g[0], g[1], g[2], g[3], g[5], 3, ids, dev(Q), 16, 16, 4, 2)
    want = oracle.search(X, o[0], o[1], o[2], o[3], 3, host(ids), Q, 16, 16, 4, 2)
    assert np.array_equal(host(got[0]), want[0]) and np.array_equal(host(got[2]), want[2])
    with pytest.raises(ef.EfannaError) as e:                        # pool below k
        ef.efanna_search(Xd, g[0], g[1], g[2], g[3], g[5], 3, ids, dev(Q), 16, 8, 4, 2)
    assert e.value.status == -1


# ---------------------------------------------------------------------------------
# The hand cases that pin the oracle's readings, put to the library directly: expected values
# are worked out on paper (see the CPU tests of the same names), not taken from the oracle.

def test_distance_hand_cases(ef):
    def dist(where, d):
        X = np.zeros((2, d), dtype=np.float32)
        for j, v in where.items():
            X[0, j] = v
        one = np.zeros(1, dtype=np.int32)
        ab = float(host(ef.efanna_pair_distances(dev(X), dev(one), dev(one + 1)))[0])
        ba = float(host(ef.efanna_pair_distances(dev(X), dev(one + 1), dev(one)))[0])
        assert ab == ba
        return ab
    # sixteen interleaved partial sums
    assert dist({0: 4096.0, 16: 1.0, 17: 1.0}, 32) == 2.0 ** 24
    assert dist({0: 4096.0, 1: 1.0, 17: 1.0}, 32) == 2.0 ** 24 + 2
    assert dist({0: 4096.0, 8: 1.0, 24: 1.0}, 32) == 2.0 ** 24 + 2
    # square and add round once
    assert dist({0: 2.0 ** -12, 16: 1.0 + 2.0 ** -12}, 17) == 1.0 + 2.0 ** -11 + 2.0 ** -23
    # the tree l += l+8, l += l+4, l += l+2, l += l+1
    assert dist({0: 4096.0, 1: 1.0, 3: 1.0}, 16) == 2.0 ** 24 + 2
    assert dist({0: 4096.0, 1: 1.0, 2: 1.0}, 16) == 2.0 ** 24
    assert dist({0: 4096.0, 8: 1.0, 12: 1.0}, 16) == 2.0 ** 24
    assert dist({0: 4096.0, 4: 1.0, 12: 1.0}, 16) == 2.0 ** 24 + 2


def test_tree_hand_cases(ef):
    step = 2.0 ** -20
    for rows, want in (([1.0 * step, 0.0], [1, 0]), ([0.6 * step, 0.0], [1, 0]), ([0.5 * step, 0.0], [0, 1]),
                       ([2.4 * step, 1.5 * step], [0, 1]), ([0.0, -0.6 * step], [1, 0])):
        X = np.array(rows, dtype=np.float32)[:, None]
        perm, off, nl = ef.efanna_build_trees(dev(X), 1, 1, 7)
        assert nl[0] == 2 and list(host(perm)[0]) == want, rows
    # 0..7 on a line, leaves of 2: splits at 3.5, then 1.5 and 5.5; a value equal to the mean goes right
    X = np.arange(8, dtype=np.float32)[:, None]
    perm, off, nl = ef.efanna_build_trees(dev(X), 1, 2, 3)
    assert nl[0] == 4 and list(host(perm)[0]) == list(range(8)) and list(host(off)[0, :5]) == [0, 2, 4, 6, 8]
    X = np.array([[1.0], [3.0], [2.0]], dtype=np.float32)           # mean 2: the 2 goes right, with the 3,
    perm, off, nl = ef.efanna_build_trees(dev(X), 1, 1, 3)          # and left of it at the next split (mean 2.5)
    assert list(host(perm)[0]) == [0, 2, 1] and list(host(off)[0, :4]) == [0, 1, 2, 3]


def test_conquer_and_search_hand_cases(ef):
    # the line 0..7 of the CPU hand cases, every coordinate of a point the same (the conquer step
    # takes dimensions that are multiples of four): whichever dimension a node draws, it splits
    # at the same place; squared distances are four times those on the line
    X = np.repeat(np.arange(8, dtype=np.float32)[:, None], 4, axis=1)
    Xd = dev(X)
    perm, off, nl, nodes, up, depth = ef.efanna_build_trees(Xd, 1, 2, 3, with_nodes=True)
    assert depth == 1

    def neighbours(nodes_t, dep, row):
        graph = ef.efanna_init_graph(Xd, perm, off, nl, 2, 6, nodes=nodes_t, leaf_up=up, tree_depth=depth,
                                     conquer_depth=dep)
        return sorted(int(v) for v in host(ef.efanna_get_graph(graph)[0])[row] if v >= 0)
    assert neighbours(nodes, 2, 0) == [1]
    assert neighbours(nodes, 1, 0) == [1, 2, 3]
    assert neighbours(nodes, 0, 0) == [1, 2, 3, 4, 5]
    assert neighbours(nodes, 0, 5) == [2, 3, 4, 6, 7]
    # the root's left child turned into a node that split by position: every point goes left in it
    edited = host(nodes).copy()
    edited.view(oracle.NODE_DTYPE)[..., 0]["dim"][0, 1] = -1
    assert neighbours(dev(edited), 0, 5) == [0, 1, 4, 6, 7]
    # search, no graph edges: the trees alone
    graph = np.full((8, 1), -1, dtype=np.int32)

    def search(q, k, P, E, iters, g=graph):
        got = ef.efanna_search(Xd, perm, off, nl, nodes, depth, 2, dev(g), dev(np.full((1, 4), q, dtype=np.float32)),
                               k, P, E, iters)
        return list(host(got[0])[0]), list(host(got[1])[0]), int(host(got[2])[0])
    assert search(2.2, 1, 1, 1, 1)[::2] == ([2], 2)
    assert search(2.2, 2, 2, 2, 1)[::2] == ([2, 3], 4)
    assert search(2.2, 4, 4, 4, 1)[::2] == ([2, 3, 1, 4], 6)
    assert search(2.2, 6, 6, 6, 1)[::2] == ([2, 3, 1, 4, 0, 5], 8)
    # equal priorities are taken in link order: the third leaf for a query on the root's split is {6,7}
    ids, dists, checked = search(3.5, 5, 5, 5, 1)
    assert ids == [3, 4, 2, 5, 6] and dists == [1.0, 1.0, 9.0, 9.0, 25.0] and checked == 6
    g2 = graph.copy()
    g2[2, 0] = 7
    assert search(2.2, 2, 2, 1, 1, g2)[::2] == ([2, 7], 5)
    g2[2, 0] = 3                                       # already delivered by the leaves: not evaluated again
    assert search(2.2, 2, 2, 1, 1, g2)[::2] == ([2, -1], 4)


def test_set_get_roundtrip_and_random_start(ef):
    rng = np.random.default_rng(8)
    n, K = 3000, 10
    X = rng.standard_normal((n, 6)).astype(np.float32)
    ids = np.stack([rng.choice(np.delete(np.arange(n), i), K, replace=False) for i in range(n)]).astype(np.int32)
    dists = np.array([[oracle.dist(X[i], X[j]) for j in row] for i, row in enumerate(ids)], dtype=np.float32)
    order = np.lexsort((ids, dists), axis=1)
    ids, dists = np.take_along_axis(ids, order, 1), np.take_along_axis(dists, order, 1)
    ids[5, 7:] = -1
    dists[5, 7:] = np.inf
    flags = (ids >= 0).astype(np.uint8)
    graph = ef.efanna_set_graph(dev(ids), dev(dists), dev(flags))
    graph_equal(ef, graph, (ids, dists, flags))
    # NN-descent from a random graph (the comparison method's starting point)
    ef.efanna_nndescent(dev(X), graph, 6, K, 1)
    want = oracle.nndescent(X, ids, dists, flags, 6, K, 1)
    got_ids, _ = graph_equal(ef, graph, want)
    tid, _ = oracle.exact_knn_definition(X, K)
    assert oracle.recall(got_ids, tid) > 0.9


def test_argument_errors(ef):
    X = dev(np.zeros((100, 4), dtype=np.float32))
    g = torch.zeros((100, 10), dtype=torch.int64, device="cuda:0")
    for kwargs, status in [(dict(iters=1, sample_L=0, seed=0), -1),
                           (dict(iters=1, sample_L=65, seed=0), -1),
                           (dict(iters=-1, sample_L=4, seed=0), -1)]:
        with pytest.raises(ef.EfannaError) as e:
            ef.efanna_nndescent(X, g, **kwargs)
        assert e.value.status == status
    with pytest.raises(ef.EfannaError) as e:
        ef.efanna_nndescent(X, g, 1, 4, 0, workspace=torch.empty(256, dtype=torch.uint8, device="cuda:0"))
    assert e.value.status == -2
    big = dev(np.zeros((300, 4000), dtype=np.float32))
    with pytest.raises(ef.EfannaError) as e:      # joins of up to K+2L = 200 rows of 4000 floats exceed the LDS
        ef.efanna_nndescent(big, torch.zeros((300, 100), dtype=torch.int64, device="cuda:0"), 1, 50, 0)
    assert e.value.status == -6
