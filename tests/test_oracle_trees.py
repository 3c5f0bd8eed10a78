"""Pins for the oracle's randomized truncated KD-trees (Alg. 2): hand-computable
cases, structural invariants, and an independent top-down re-derivation of every
split in Python integers."""
import numpy as np
import pytest

import oracle
from paper_1609_07228_amd import synth


def leaves_of(perm_t, off_t, nl):
    return [perm_t[off_t[l]:off_t[l + 1]] for l in range(nl)]


def test_hand_case_perfect_binary_tree():
    # one dimension, values 0..7, leaf size 2: mean 3.5 -> {0..3},{4..7}; then 1.5
    # and 5.5 -> four leaves of two, whatever the seed (d = 1 leaves no choice)
    X = np.arange(8, dtype=np.float32).reshape(8, 1)
    for seed in (0, 1, 99):
        perm, off, nl = oracle.build_trees(X, T=3, S=2, seed=seed)
        for t in range(3):
            assert nl[t] == 4
            assert off[t, :5].tolist() == [0, 2, 4, 6, 8]
            assert perm[t].tolist() == list(range(8))


def test_hand_case_shuffled_values_stable_partition():
    # values chosen so that ids interleave: mean of [5,1,7,3,6,0,4,2] = 3.5
    X = np.array([5, 1, 7, 3, 6, 0, 4, 2], dtype=np.float32).reshape(8, 1)
    perm, off, nl = oracle.build_trees(X, T=1, S=4, seed=3)
    # left = ids with value < 3.5 in id order, right likewise
    assert perm[0].tolist() == [1, 3, 5, 7, 0, 2, 4, 6]
    assert nl[0] == 2 and off[0, :3].tolist() == [0, 4, 8]


def test_value_equal_to_mean_goes_right():
    X = np.array([0, 2, 4, 2], dtype=np.float32).reshape(4, 1)  # mean 2
    perm, off, nl = oracle.build_trees(X, T=1, S=3, seed=0)
    assert perm[0].tolist() == [0, 1, 2, 3]
    assert off[0, :3].tolist() == [0, 1, 4]


def test_all_equal_points_split_into_positional_halves():
    X = np.full((10, 4), 3.25, dtype=np.float32)
    perm, off, nl = oracle.build_trees(X, T=2, S=3, seed=5)
    for t in range(2):
        assert perm[t].tolist() == list(range(10))          # nothing moves
        assert off[t, :nl[t] + 1].tolist() == [0, 2, 5, 7, 10]  # 10 -> 5+5 -> (2,3)+(2,3)


def test_single_leaf_when_n_le_S():
    X = np.random.default_rng(0).standard_normal((7, 3)).astype(np.float32)
    perm, off, nl = oracle.build_trees(X, T=1, S=7, seed=0)
    assert nl[0] == 1 and off[0, :2].tolist() == [0, 7] and perm[0].tolist() == list(range(7))


def q(x):
    # round-half-even of x * 2^20, exact: Python floats are doubles and the
    # product of a float32 value with 2^20 is exact in a double
    return round(float(x) * 1048576.0)


def variance_dim(X, ids, draw):
    """The split dimension by variance in Python integers: over the node's first 100 ids, the five
    dimensions with the largest m * sum(q^2) - sum(q)^2 (equal ones: smaller dimension first); the
    node's draw picks among them."""
    sample = ids[:100]
    m = len(sample)
    var = []
    for j in range(X.shape[1]):
        qs = [q(X[i, j]) for i in sample]
        var.append(m * sum(v * v for v in qs) - sum(qs) ** 2)
    order = sorted(range(X.shape[1]), key=lambda j: (-var[j], j))[:5]
    return order[draw % len(order)]


def rederive(X, T, S, seed, split_rule=0):
    """Top-down rebuild with Python integers: every segment of every tree must be
    sorted(left ids) ++ sorted(right ids) of the mean split on the node's dimension."""
    n, d = X.shape
    perms, offs = [], []
    for t in range(T):
        out, off = [], []

        def rec(ids, h, depth):
            if len(ids) <= S:
                off.append(len(out))
                out.extend(ids)
                return
            draw = oracle.node_rand(seed, t, h)
            dim = variance_dim(X, ids, draw) if split_rule == 1 else draw % d
            qs = [q(X[i, dim]) for i in ids]
            tot = sum(qs)
            left = [i for i, v in zip(ids, qs) if len(ids) * v < tot]
            right = [i for i, v in zip(ids, qs) if not len(ids) * v < tot]
            if not left or not right:
                left, right = ids[:len(ids) // 2], ids[len(ids) // 2:]
            rec(left, 2 * h, depth + 1)
            rec(right, 2 * h + 1, depth + 1)

        rec(list(range(n)), 1, 0)
        off.append(n)
        perms.append(out)
        offs.append(off)
    return perms, offs


@pytest.mark.parametrize("name,n,T,S", [("gmm10k_d32", 3000, 4, 8), ("sift100k_like", 2500, 3, 16),
                                         ("mixed4m_d96", 2000, 2, 64)])
def test_rederivation_in_python_integers(name, n, T, S):
    X = synth.generate(name, n=n)
    perm, off, nl = oracle.build_trees(X, T=T, S=S, seed=synth.ALGO_SEED)
    perms, offs = rederive(X, T, S, synth.ALGO_SEED)
    for t in range(T):
        assert perm[t].tolist() == perms[t]
        assert off[t, :nl[t] + 1].tolist() == offs[t]


@pytest.mark.parametrize("name,n,T,S", [("gmm10k_d32", 1500, 3, 8), ("sift100k_like", 1200, 2, 16),
                                         ("mixed4m_d96", 900, 2, 64)])
def test_variance_rule_rederivation_in_python_integers(name, n, T, S):
    X = synth.generate(name, n=n)
    perm, off, nl = oracle.build_trees(X, T=T, S=S, seed=synth.ALGO_SEED, split_rule=1)
    perms, offs = rederive(X, T, S, synth.ALGO_SEED, split_rule=1)
    for t in range(T):
        assert perm[t].tolist() == perms[t]
        assert off[t, :nl[t] + 1].tolist() == offs[t]
    plain, _, _ = oracle.build_trees(X, T=T, S=S, seed=synth.ALGO_SEED)
    assert not np.array_equal(plain, perm)


def root_dim(nodes_t, nl_t):
    roots = [int(nd["dim"]) for nd in nodes_t[1:nl_t] if nd["parent"] == -1]
    assert len(roots) == 1
    return roots[0]


def test_variance_rule_hand_cases():
    rng = np.random.default_rng(8)
    # five dimensions spread widely, the others hardly: every split is on one of the five,
    # and the draws use all of them
    wide = [3, 7, 11, 20, 30]
    X = (0.05 * rng.standard_normal((4000, 32))).astype(np.float32)
    X[:, wide] = (10.0 * rng.standard_normal((4000, 5))).astype(np.float32)
    _, _, nl, nodes, _ = oracle.build_trees_nodes(X, T=3, S=8, seed=5, split_rule=1)
    seen = set()
    for t in range(3):
        dims = nodes[t, 1:nl[t]]["dim"]
        assert set(dims.tolist()) <= set(wide)
        seen |= set(dims.tolist())
    assert seen == set(wide)
    # a constant dimension among six: never one of the five
    X = rng.standard_normal((600, 6)).astype(np.float32)
    X[:, 2] = 1.5
    _, _, nl, nodes, _ = oracle.build_trees_nodes(X, T=4, S=4, seed=1, split_rule=1)
    for t in range(4):
        assert 2 not in nodes[t, 1:nl[t]]["dim"].tolist()
    # two dimensions: the order is by variance, the root's draw picks the place in it
    X = np.stack([np.arange(40, dtype=np.float32), 100.0 * ((np.arange(40) * 7) % 40).astype(np.float32)], axis=1)
    for seed in range(6):
        _, _, nl, nodes, _ = oracle.build_trees_nodes(X, T=1, S=20, seed=seed, split_rule=1)
        assert root_dim(nodes[0], nl[0]) == [1, 0][oracle.node_rand(seed, 0, 1) % 2]
    # the variance is taken about the mean: a far-off but narrow dimension loses to a wide one at zero
    X = np.stack([1000.0 + 0.01 * np.arange(30), np.arange(30) - 15.0], axis=1).astype(np.float32)
    for seed in range(4):
        _, _, nl, nodes, _ = oracle.build_trees_nodes(X, T=1, S=15, seed=seed, split_rule=1)
        assert root_dim(nodes[0], nl[0]) == [1, 0][oracle.node_rand(seed, 0, 1) % 2]
    # only the first 100 points of a node are looked at
    X = np.zeros((300, 2), dtype=np.float32)
    X[:100, 0] = np.arange(100)
    X[100:, 1] = 1000.0 * np.arange(200)
    for seed in range(4):
        _, _, nl, nodes, _ = oracle.build_trees_nodes(X, T=1, S=150, seed=seed, split_rule=1)
        assert root_dim(nodes[0], nl[0]) == [0, 1][oracle.node_rand(seed, 0, 1) % 2]
    # equal variances: the smaller dimension comes first
    col = rng.standard_normal(50).astype(np.float32)
    X = np.stack([col, col, col], axis=1)
    for seed in range(6):
        _, _, nl, nodes, _ = oracle.build_trees_nodes(X, T=1, S=25, seed=seed, split_rule=1)
        assert root_dim(nodes[0], nl[0]) == oracle.node_rand(seed, 0, 1) % 3
    # large coordinates: the squares need more than 64 bits
    X = (rng.integers(-2**19, 2**19, size=(500, 8)).astype(np.float32) + 0.5)
    X[:, 5] *= 1e-3
    perm, off, nl = oracle.build_trees(X, T=2, S=10, seed=2, split_rule=1)
    perms, offs = rederive(X, 2, 10, 2, split_rule=1)
    assert perm[0].tolist() == perms[0] and perm[1].tolist() == perms[1]


def test_structural_invariants_and_randomisation():
    X = synth.generate("sift100k_like", n=20000)
    T, S = 4, 16
    perm, off, nl = oracle.build_trees(X, T=T, S=S, seed=1)
    perm2, off2, nl2 = oracle.build_trees(X, T=T, S=S, seed=1)
    assert np.array_equal(perm, perm2) and np.array_equal(off, off2)
    for t in range(T):
        assert np.array_equal(np.sort(perm[t]), np.arange(20000))
        o = off[t, :nl[t] + 1]
        sizes = np.diff(o)
        assert o[0] == 0 and o[-1] == 20000 and sizes.min() >= 1 and sizes.max() <= S
        for leaf in leaves_of(perm[t], o, nl[t]):
            assert np.all(np.diff(leaf) > 0)       # ids ascending inside a leaf
    assert not np.array_equal(perm[0], perm[1])    # trees differ
    perm3, _, _ = oracle.build_trees(X, T=T, S=S, seed=2)
    assert not np.array_equal(perm, perm3)         # seeds differ


def test_split_test_resolves_steps_of_2_to_minus_20():
    # two points 2^-20 apart, the larger one first: quantised to 1 and 0, sum 1, and 2*q < 1 only
    # for the second point, which therefore goes left.  At any coarser resolution both quantise
    # to 0, the split is degenerate and the positional halves keep the first point on the left.
    X = np.array([[2.0 ** -20], [0.0]], dtype=np.float32)
    perm, off, nl = oracle.build_trees(X, 1, 1, 7)
    assert nl[0] == 2 and list(perm[0]) == [1, 0]


def test_coordinates_are_rounded_to_nearest_even_not_truncated():
    step = 2.0 ** -20
    # 0.6 steps rounds to 1 (truncation would give 0 and a degenerate split): the second point goes left
    X = np.array([[0.6 * step], [0.0]], dtype=np.float32)
    assert list(oracle.build_trees(X, 1, 1, 7)[0][0]) == [1, 0]
    # 0.5 steps is a tie and rounds to the even 0: both quantise alike, positional halves
    X = np.array([[0.5 * step], [0.0]], dtype=np.float32)
    assert list(oracle.build_trees(X, 1, 1, 7)[0][0]) == [0, 1]
    # 1.5 steps is a tie and rounds to the even 2, 2.4 steps rounds to 2 as well: alike again
    X = np.array([[2.4 * step], [1.5 * step]], dtype=np.float32)
    assert list(oracle.build_trees(X, 1, 1, 7)[0][0]) == [0, 1]
    # negative values: -0.6 steps rounds to -1, below 0
    X = np.array([[0.0], [-0.6 * step]], dtype=np.float32)
    assert list(oracle.build_trees(X, 1, 1, 7)[0][0]) == [1, 0]


def test_quantisation_ties_and_large_values():
    # values closer than 2^-21 quantise together; mean compare stays exact near 2^20
    X = np.array([[1.0], [1.0 + 2.0 ** -23], [1000000.0], [-1000000.0], [3.0], [5.0]],
                 dtype=np.float32)
    perm, off, nl = oracle.build_trees(X, T=1, S=1, seed=0)
    perms, offs = rederive(X, 1, 1, 0)
    assert perm[0].tolist() == perms[0] and off[0, :nl[0] + 1].tolist() == offs[0]


def test_input_outside_the_exact_domain_is_rejected():
    """The mean test compares cnt * q(x) with a sum of q in 64-bit integers: inputs that could
    overflow them (non-finite, |x| >= 2^20, n * |x| >= 2^43) are refused, not wrapped."""
    X = np.zeros((50, 2), dtype=np.float32)
    for bad in (np.nan, np.inf, -np.inf, 2.0 ** 20, -(2.0 ** 20)):
        Y = X.copy()
        Y[13, 1] = bad
        with pytest.raises(ValueError):
            oracle.build_trees(Y, 1, 4, 0)
    Y = X.copy()
    Y[13, 1] = np.nextafter(np.float32(2.0 ** 20), np.float32(0))      # the largest value inside
    oracle.build_trees(Y, 1, 4, 0)
    # beyond 2^23 points the bound on n * |x| binds first: 2^24 points take |x| < 2^19
    n = 1 << 24
    Z = np.zeros((n, 1), dtype=np.float32)
    Z[5, 0] = 2.0 ** 19
    with pytest.raises(ValueError):
        oracle.build_trees(Z, 1, n, 0)
    Z[5, 0] = np.nextafter(np.float32(2.0 ** 19), np.float32(0))
    perm, off, nl = oracle.build_trees(Z, 1, n, 0)      # S >= n: a single leaf, nothing to sum
    assert nl[0] == 1
