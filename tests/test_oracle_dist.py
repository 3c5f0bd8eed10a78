"""Pins for the oracle's distance (squared L2, float32, 16 interleaved partial
sums added in a fixed pairwise tree) and for its counter-based generator."""
import numpy as np
import pytest

import oracle

M64 = (1 << 64) - 1


def test_distance_is_exact_on_integer_data():
    # values 0..255, d=128: every partial sum is an integer below 2^24, so the
    # float32 result must equal integer arithmetic exactly
    rng = np.random.default_rng(0)
    for d in (1, 7, 16, 17, 32, 96, 128):
        a = rng.integers(0, 256, d)
        b = rng.integers(0, 256, d)
        want = int(((a - b) ** 2).sum())
        assert float(oracle.dist(a, b)) == float(want)


def test_distance_matches_float64_within_bound():
    rng = np.random.default_rng(1)
    for d in (3, 32, 96, 128, 960, 1000):
        for _ in range(20):
            a = rng.standard_normal(d).astype(np.float32)
            b = (a + rng.standard_normal(d).astype(np.float32) * rng.choice([1e-3, 1.0, 50.0])
                 ).astype(np.float32)
            ref = float(((a.astype(np.float64) - b.astype(np.float64)) ** 2).sum())
            bound = (d / 16 + 8) * 2.0 ** -24
            assert abs(float(oracle.dist(a, b)) - ref) <= bound * ref
            assert bound < 1e-5


def test_distance_symmetric_and_zero():
    rng = np.random.default_rng(2)
    a = rng.standard_normal(100).astype(np.float32)
    b = rng.standard_normal(100).astype(np.float32)
    assert oracle.dist(a, b).tobytes() == oracle.dist(b, a).tobytes()
    assert float(oracle.dist(a, a)) == 0.0


def _unit(d, where):
    a = np.zeros(d, dtype=np.float32)
    for j, v in where.items():
        a[j] = v
    return a, np.zeros(d, dtype=np.float32)


def test_interleave_width_is_16():
    # 2^24 + 1 is not a float32.  Dimensions 0 and 16 share a partial sum, so the
    # 1 is absorbed; dimensions 0 and 1 do not, and meet only in the final adds.
    a, b = _unit(32, {0: 4096.0, 16: 1.0, 17: 1.0})
    # partial 0: fma(1,1,2^24) -> 2^24 ; partial 1: 1 ; final 2^24 + 1 -> 2^24
    assert float(oracle.dist(a, b)) == 2.0 ** 24
    a, b = _unit(32, {0: 4096.0, 1: 1.0, 17: 1.0})
    # partial 1 holds 2 (both ones), which survives the final add
    assert float(oracle.dist(a, b)) == 2.0 ** 24 + 2


def test_sixteen_partial_sums_not_eight():
    # dimensions 8 and 24 share partial sum 8, away from the 2^24 in partial sum 0: their ones add
    # to 2 there and survive the final adds.  With eight partial sums they would meet 2^24 one by
    # one and be rounded away.
    a, b = _unit(32, {0: 4096.0, 8: 1.0, 24: 1.0})
    assert float(oracle.dist(a, b)) == 2.0 ** 24 + 2


def test_square_and_add_round_once():
    # (1 + 2^-12)^2 = 1 + 2^-11 + 2^-24 is not a float32.  Added to the 2^-24 already in the
    # partial sum (dimension 0, same partial sum as dimension 16) the exact total 1 + 2^-11 + 2^-23
    # is one, so a fused multiply-add returns it; rounding the square first loses the 2^-24 (tie
    # to even), and adding 2^-24 afterwards loses it again.
    a, b = _unit(17, {0: 2.0 ** -12, 16: 1.0 + 2.0 ** -12})
    assert float(oracle.dist(a, b)) == 1.0 + 2.0 ** -11 + 2.0 ** -23
    assert float(oracle.dist(b, a)) == 1.0 + 2.0 ** -11 + 2.0 ** -23


def test_reduction_tree_shape():
    # partial sums are combined l += l+8, l += l+4, l += l+2, l += l+1.
    # ones in partials 1 and 3 meet each other (step 2) before meeting 2^24;
    # ones in partials 1 and 2 each meet 2^24 alone and are rounded away.
    a, b = _unit(16, {0: 4096.0, 1: 1.0, 3: 1.0})
    assert float(oracle.dist(a, b)) == 2.0 ** 24 + 2
    a, b = _unit(16, {0: 4096.0, 1: 1.0, 2: 1.0})
    assert float(oracle.dist(a, b)) == 2.0 ** 24
    # partials 8 and 12: 8 joins 0 at the first step (lost), 12 joins 4, then 0 (lost)
    a, b = _unit(16, {0: 4096.0, 8: 1.0, 12: 1.0})
    assert float(oracle.dist(a, b)) == 2.0 ** 24
    # partials 4 and 12 meet each other at the first step, survive as 2
    a, b = _unit(16, {0: 4096.0, 4: 1.0, 12: 1.0})
    assert float(oracle.dist(a, b)) == 2.0 ** 24 + 2


def test_generator_reproduces_published_splitmix64_vector():
    # SplitMix64 seeded with 0 yields 0xE220A8397B1DCDAF then 0x6E789E6AA1B965F4
    # (Steele, Lea & Flood 2014 reference stream).  node_rand(0, 0, h) is
    # finaliser(first_output + h); pick h so that the argument is 2*gamma.
    gamma = 0x9E3779B97F4A7C15
    first, second = 0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4
    h = (2 * gamma - first) & M64
    assert oracle.node_rand(0, 0, h) == second
    # tree index enters as seed + gamma*(tree+1): tree 1 with seed -gamma is tree 0 with seed 0
    assert oracle.node_rand((-gamma) & M64, 1, h) == second


def test_generator_spreads():
    dims = [oracle.node_rand(42, t, h) % 128 for t in range(8) for h in range(1, 200)]
    counts = np.bincount(dims, minlength=128)
    assert counts.min() >= 1 and counts.max() < 40
    hs = {oracle.reverse_hash(7, 0, 5, u) for u in range(1000)}
    assert len(hs) > 990
    assert oracle.reverse_hash(7, 0, 5, 6) != oracle.reverse_hash(7, 1, 5, 6)
    assert oracle.reverse_hash(7, 0, 5, 6) != oracle.reverse_hash(7, 0, 6, 5)
