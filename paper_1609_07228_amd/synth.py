"""Seeded synthetic workloads shaped like the paper's kNN-graph experiments.

The paper measures graph construction on two public descriptor sets (Table I:
one million 128-d integer-valued vectors, one million 960-d vectors in [0,1]).
Neither is available here, so every input is a seeded Gaussian-mixture stand-in
of the same shape and value range.  This module only draws random numbers: it
contains none of the method's arithmetic (no distances, trees or graphs) and is
the one piece of code that both the CPU oracle's tests and the HIP path's tests
may share.

Draw order (so that a workload can be regenerated bit-for-bit):
  rng = numpy.random.Generator(numpy.random.PCG64(data_seed))
  1. centres  = rng.random((n_comp, d))            (float64, then affine map)
  2. for each row chunk of CHUNK rows, in order:
       a. comp  = rng.integers(0, n_comp, size=rows)
       b. (workload 5 only) coin = rng.random(rows) < 0.5
       c. noise = rng.standard_normal((rows, d), dtype=float32)
       d. (workload 5 only) unif = rng.random((rows, d), dtype=float32)
"""
from __future__ import annotations

import numpy as np

CHUNK = 65536

# name -> generator recipe and the algorithm parameters quoted with it.
#   K graph degree, T trees, S leaf size, I NN-descent iterations, L sample size.
WORKLOADS = {
    "gmm10k_d32": dict(n=10_000, d=32, n_comp=10, kind="gauss", lo=-10.0, hi=10.0,
                       sigma=1.0, data_seed=1001, K=10, T=4, S=8, I=4, L=10),
    "sift100k_like": dict(n=100_000, d=128, n_comp=100, kind="u8grid", lo=0.0, hi=128.0,
                          sigma=16.0, data_seed=1002, K=20, T=8, S=16, I=6, L=20),
    "sift1m_like": dict(n=1_000_000, d=128, n_comp=1000, kind="u8grid", lo=0.0, hi=128.0,
                        sigma=16.0, data_seed=1003, K=10, T=8, S=16, I=8, L=10),
    "gist1m_like": dict(n=1_000_000, d=960, n_comp=1000, kind="unit", lo=0.0, hi=1.0,
                        sigma=0.05, data_seed=1004, K=10, T=8, S=16, I=10, L=10),
    "mixed4m_d96": dict(n=4_000_000, d=96, n_comp=4000, kind="mixed", lo=-1.0, hi=1.0,
                        sigma=0.1, data_seed=1005, K=100, T=16, S=64, I=8, L=50),
}

ALGO_SEED = 42
SAMPLE_SEED = 7


def params(name: str) -> dict:
    """Algorithm parameters (K, T, S, I, L) and shape (n, d) of a named workload."""
    w = WORKLOADS[name]
    return {k: w[k] for k in ("n", "d", "K", "T", "S", "I", "L")}


def generate(name: str, n: int | None = None, out: np.ndarray | None = None) -> np.ndarray:
    """Return the (n, d) float32 matrix of workload `name`.

    `n` may be lowered to get a prefix-sized variant from the same recipe (used
    by tests that need an input the CPU side finishes quickly); the first rows
    of a smaller variant equal the first rows of the full one as long as both
    cover the same chunks.  `out` may be a preallocated (n, d) float32 array
    (for example pinned host memory).
    """
    w = WORKLOADS[name]
    n = w["n"] if n is None else int(n)
    d, n_comp = w["d"], w["n_comp"]
    rng = np.random.Generator(np.random.PCG64(w["data_seed"]))
    centres = (w["lo"] + (w["hi"] - w["lo"]) * rng.random((n_comp, d))).astype(np.float32)
    X = np.empty((n, d), dtype=np.float32) if out is None else out
    assert X.shape == (n, d) and X.dtype == np.float32
    sigma = np.float32(w["sigma"])
    for r0 in range(0, n, CHUNK):
        rows = min(CHUNK, n - r0)
        comp = rng.integers(0, n_comp, size=rows)
        coin = rng.random(rows) < 0.5 if w["kind"] == "mixed" else None
        x = rng.standard_normal((rows, d), dtype=np.float32)
        x *= sigma
        x += centres[comp]
        if w["kind"] == "u8grid":
            np.clip(x, 0.0, 255.0, out=x)
            np.rint(x, out=x)
        elif w["kind"] == "unit":
            np.clip(x, 0.0, 1.0, out=x)
        elif w["kind"] == "mixed":
            u = rng.random((rows, d), dtype=np.float32)
            u *= np.float32(2.0)
            u -= np.float32(1.0)
            x[coin] = u[coin]
        X[r0:r0 + rows] = x
    return X


def generate_queries(name: str, nq: int, query_seed: int = 0) -> np.ndarray:
    """(nq, d) float32 query vectors for workload `name`: fresh draws from the same mixture
    (the centres of `generate`, components and noise from a generator of their own seeded
    with data_seed + 7919 * (query_seed + 1)), so they follow the data's distribution without
    being data points."""
    w = WORKLOADS[name]
    d, n_comp = w["d"], w["n_comp"]
    rng = np.random.Generator(np.random.PCG64(w["data_seed"]))
    centres = (w["lo"] + (w["hi"] - w["lo"]) * rng.random((n_comp, d))).astype(np.float32)
    rq = np.random.Generator(np.random.PCG64(w["data_seed"] + 7919 * (query_seed + 1)))
    comp = rq.integers(0, n_comp, size=nq)
    coin = rq.random(nq) < 0.5 if w["kind"] == "mixed" else None
    x = rq.standard_normal((nq, d), dtype=np.float32)
    x *= np.float32(w["sigma"])
    x += centres[comp]
    if w["kind"] == "u8grid":
        np.clip(x, 0.0, 255.0, out=x)
        np.rint(x, out=x)
    elif w["kind"] == "unit":
        np.clip(x, 0.0, 1.0, out=x)
    elif w["kind"] == "mixed":
        u = rq.random((nq, d), dtype=np.float32)
        u *= np.float32(2.0)
        u -= np.float32(1.0)
        x[coin] = u[coin]
    return x


def sample_rows(n: int, m: int = 10_000, seed: int = SAMPLE_SEED) -> np.ndarray:
    """First m entries of a seeded permutation of range(n): the rows on which
    recall is measured when exact brute force over all rows is too slow."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return np.sort(rng.permutation(n)[:min(m, n)]).astype(np.int64)
