"""The bound behind the joins' half-precision filter, checked on the CPU against an emulation of
the rounding: with a' = (a s) rounded towards zero to half precision, s a power of two that brings
the largest |coordinate| of the data below 2^15,
    |a' - a s| <= u |a'| + r0,   u = 1.01 / 1023,   r0 = 1.01 sqrt(d) 2^-24,
so the distance D' of two rounded vectors is within r(a) + r(b) of s D, and D^2 <= T implies
D'^2 <= T s^2 + rho (2 s sqrt(T) + rho).  The library's host code sets u and r0 where it launches
the register joins; the kernels never drop a pair unless the right-hand side is exceeded.  Float64
arithmetic here, no GPU."""
import numpy as np
import pytest


def to_half_rtz(x):
    """float32 -> float16 rounded towards zero (numpy rounds to nearest: step back where that went up)."""
    h = x.astype(np.float16)
    up = np.abs(h.astype(np.float64)) > np.abs(x.astype(np.float64))
    return np.where(up, np.nextafter(h, np.float16(0)), h).astype(np.float16)


def scale_for(X):
    e = int(np.floor(np.log2(float(np.abs(X).max())))) if np.abs(X).max() > 0 else 0
    return 2.0 ** (14 - e) if e >= 15 else 1.0


CASES = [("unit", 1.0, 0.0), ("large", 9e4, 0.0), ("tiny", 3e-6, 0.0), ("offset", 1.0, 900.0),
         ("small_offset", 0.05, 1.0), ("limit", 8000.0, 0.0)]


@pytest.mark.parametrize("name,mul,add", CASES)
@pytest.mark.parametrize("d", [4, 36, 128])
def test_rounding_radius_and_filter_bound(name, mul, add, d):
    rng = np.random.default_rng(d + len(name))
    X = (rng.standard_normal((400, d)) * mul + add).astype(np.float32)
    if name == "tiny":
        X[0, 0] = np.float32(1.0)          # a large coordinate beside subnormal ones
    s = scale_for(X)
    assert np.abs(X.astype(np.float64) * s).max() < 2.0 ** 15
    H = to_half_rtz((X.astype(np.float64) * s).astype(np.float32)).astype(np.float64)
    Xs = X.astype(np.float64) * s
    u, r0 = 1.01 / 1023.0, 1.01 * np.sqrt(d) * 2.0 ** -24
    err = np.linalg.norm(H - Xs, axis=1)
    rad = u * np.linalg.norm(H, axis=1) + r0
    assert np.all(err <= rad)
    assert np.all(np.abs(H) <= np.abs(Xs))                       # towards zero
    # every pair: the rounded vectors' distance is within the two radii of the scaled true distance,
    # and a threshold at the true squared distance never rejects
    i, j = np.triu_indices(X.shape[0], 1)
    D = np.linalg.norm(Xs[i] - Xs[j], axis=1)
    Dr = np.linalg.norm(H[i] - H[j], axis=1)
    rho = rad[i] + rad[j]
    assert np.all(np.abs(Dr - D) <= rho)
    T = D * D                                                    # threshold = this pair's own distance
    assert np.all(Dr * Dr <= T + rho * (2.0 * np.sqrt(T) + rho) + 1e-300)
    # the radius is not vacuous: somewhere the rounding moves a distance by a good part of it
    if name in ("unit", "large", "limit"):
        assert (np.abs(Dr - D) / rho).max() > 0.02


def test_without_the_radius_pairs_would_be_lost():
    # four dimensions, an offset of a thousand: the rounded distance exceeds the true one by a per cent or more
    # for many pairs, which a filter with no radius would reject at a threshold just above the pair
    rng = np.random.default_rng(5)
    X = (rng.standard_normal((300, 4)) * 0.5 + 1000.0).astype(np.float32)
    H = to_half_rtz(X).astype(np.float64)
    i, j = np.triu_indices(300, 1)
    D = np.linalg.norm(X[i].astype(np.float64) - X[j], axis=1)
    Dr = np.linalg.norm(H[i] - H[j], axis=1)
    assert np.mean(Dr * Dr > 1.01 * D * D) > 0.1
