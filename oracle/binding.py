"""ctypes binding of efanna_oracle.c (test infrastructure, see the C file's header)."""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "efanna_oracle.c")
# EFANNA_ORACLE_LIBRARY names a library built elsewhere from (a variant of) the C file: the tests
# that plant mistakes in the oracle to see whether the pins notice use it.
_OVERRIDE = os.environ.get("EFANNA_ORACLE_LIBRARY")
_LIB = _OVERRIDE or os.path.join(_HERE, "libefanna_oracle.so")
_lib = None

CFLAGS = ["-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
          "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  -ffp-contract=off keeps the compiler from
    fusing a-b with the following multiply-add; fmaf is called explicitly."""
    if _OVERRIDE:
        return _LIB
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *CFLAGS, "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = C.CDLL(_LIB)
        lib.oracle_dist.restype = C.c_float
        lib.oracle_dist.argtypes = [C.c_void_p, C.c_void_p, C.c_int32]
        lib.oracle_node_rand.restype = C.c_uint64
        lib.oracle_node_rand.argtypes = [C.c_uint64, C.c_int32, C.c_uint64]
        lib.oracle_reverse_hash.restype = C.c_uint32
        lib.oracle_reverse_hash.argtypes = [C.c_uint64, C.c_int32, C.c_int32, C.c_int32]
        lib.oracle_build_trees.restype = C.c_int
        lib.oracle_build_trees.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_int32,
                                           C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.oracle_build_trees_nodes.restype = C.c_int
        lib.oracle_build_trees_nodes.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_int32,
                                                 C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p,
                                                 C.c_void_p, C.c_void_p]
        lib.oracle_build_trees_rule.restype = C.c_int
        lib.oracle_build_trees_rule.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_int32,
                                                C.c_uint64, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                                C.c_void_p, C.c_void_p]
        lib.oracle_conquer_graph.restype = C.c_int
        lib.oracle_conquer_graph.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p,
                                             C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                             C.c_int32, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                             C.c_void_p]
        lib.oracle_init_graph.restype = C.c_int
        lib.oracle_init_graph.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p,
                                          C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int64,
                                          C.c_void_p, C.c_void_p, C.c_void_p]
        lib.oracle_nndescent.restype = C.c_int
        lib.oracle_nndescent.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_void_p,
                                         C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_uint64,
                                         C.c_int32, C.c_void_p]
        lib.oracle_nndescent_until.restype = C.c_int
        lib.oracle_nndescent_until.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_void_p,
                                               C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_uint64,
                                               C.c_int32, C.c_void_p, C.c_double, C.c_void_p]
        lib.oracle_nndescent_opts.restype = C.c_int
        lib.oracle_nndescent_opts.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_void_p,
                                              C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_uint64,
                                              C.c_int32, C.c_void_p, C.c_double, C.c_void_p, C.c_int32]
        lib.oracle_search.restype = C.c_int
        lib.oracle_search.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p,
                                      C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                      C.c_void_p, C.c_void_p]
        lib.oracle_num_threads.restype = C.c_int
        lib.oracle_set_num_threads.argtypes = [C.c_int]
        _lib = lib
    return _lib


def _f32(X):
    X = np.ascontiguousarray(X, dtype=np.float32)
    assert X.ndim == 2
    return X


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(t: int) -> None:
    _load().oracle_set_num_threads(int(t))


def node_rand(seed: int, tree: int, heap_id: int) -> int:
    return int(_load().oracle_node_rand(seed, tree, heap_id))


def reverse_hash(seed: int, it: int, v: int, u: int) -> int:
    return int(_load().oracle_reverse_hash(seed, it, v, u))


def dist(a, b) -> np.float32:
    a = np.ascontiguousarray(a, dtype=np.float32)
    b = np.ascontiguousarray(b, dtype=np.float32)
    assert a.shape == b.shape and a.ndim == 1
    return np.float32(_load().oracle_dist(_p(a), _p(b), a.shape[0]))


def build_trees(X, T: int, S: int, seed: int, split_rule: int = 0):
    """Alg. 2 (split_rule 1: the split dimension is chosen among the five of largest variance; 2: a
    node splits on a random projection, a signed sum of eight coordinates).
    Returns (perm [T,n] int32, leaf_off [T,n+1] int32, n_leaves [T] int32)."""
    X = _f32(X)
    n, d = X.shape
    perm = np.empty((T, n), dtype=np.int32)
    leaf_off = np.full((T, n + 1), -1, dtype=np.int32)
    n_leaves = np.zeros(T, dtype=np.int32)
    if split_rule:
        rc = _load().oracle_build_trees_rule(_p(X), n, d, T, S, seed, split_rule, _p(perm), _p(leaf_off),
                                             _p(n_leaves), None, None)
    else:
        rc = _load().oracle_build_trees(_p(X), n, d, T, S, seed, _p(perm), _p(leaf_off), _p(n_leaves))
    if rc != 0:
        raise ValueError(f"oracle_build_trees failed: {rc}")
    return perm, leaf_off, n_leaves


# one internal node of a tree, numbered by the leaf that starts its right part
NODE_DTYPE = np.dtype([("sum", np.int64), ("dim", np.int32), ("cnt", np.int32), ("parent", np.int32),
                       ("depth", np.int32), ("child", np.int32, (2,))], align=True)
assert NODE_DTYPE.itemsize == 32


def build_trees_nodes(X, T: int, S: int, seed: int, split_rule: int = 0):
    """Alg. 2 with the internal nodes kept for the conquer step of Alg. 3.  Returns (perm,
    leaf_off, n_leaves, nodes [T,n+1] NODE_DTYPE, leaf_up [T,n+1] int32)."""
    X = _f32(X)
    n, d = X.shape
    perm = np.empty((T, n), dtype=np.int32)
    leaf_off = np.full((T, n + 1), -1, dtype=np.int32)
    n_leaves = np.zeros(T, dtype=np.int32)
    nodes = np.zeros((T, n + 1), dtype=NODE_DTYPE)
    leaf_up = np.full((T, n + 1), -1, dtype=np.int32)
    rc = _load().oracle_build_trees_rule(_p(X), n, d, T, S, seed, split_rule, _p(perm), _p(leaf_off),
                                         _p(n_leaves), _p(nodes), _p(leaf_up))
    if rc != 0:
        raise ValueError(f"oracle_build_trees_nodes failed: {rc}")
    return perm, leaf_off, n_leaves, nodes, leaf_up


def conquer_graph(X, perm, leaf_off, n_leaves, nodes, leaf_up, dep: int, K: int, rows=None):
    """Alg. 3 with conquer-to depth `dep` (root = 0).  Returns (ids, dists, flags), each
    [n_rows, K]."""
    X = _f32(X)
    n, d = X.shape
    T = perm.shape[0]
    assert perm.shape == (T, n) and leaf_off.shape == (T, n + 1)
    assert nodes.shape == (T, n + 1) and nodes.dtype == NODE_DTYPE and leaf_up.shape == (T, n + 1)
    rows_arr = None if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
    m = n if rows_arr is None else rows_arr.shape[0]
    ids = np.empty((m, K), dtype=np.int32)
    dists = np.empty((m, K), dtype=np.float32)
    flags = np.empty((m, K), dtype=np.uint8)
    rc = _load().oracle_conquer_graph(_p(X), n, d, _p(np.ascontiguousarray(perm)),
                                      _p(np.ascontiguousarray(leaf_off)),
                                      _p(np.ascontiguousarray(n_leaves)),
                                      _p(np.ascontiguousarray(nodes)),
                                      _p(np.ascontiguousarray(leaf_up)), dep, T, K,
                                      None if rows_arr is None else _p(rows_arr), m,
                                      _p(ids), _p(dists), _p(flags))
    if rc != 0:
        raise ValueError(f"oracle_conquer_graph failed: {rc}")
    return ids, dists, flags


def init_graph(X, perm, leaf_off, n_leaves, K: int, rows=None):
    """Alg. 3 at the leaves.  Returns (ids, dists, flags), each [n_rows, K]."""
    X = _f32(X)
    n, d = X.shape
    T = perm.shape[0]
    assert perm.shape == (T, n) and leaf_off.shape == (T, n + 1)
    rows_arr = None if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
    m = n if rows_arr is None else rows_arr.shape[0]
    ids = np.empty((m, K), dtype=np.int32)
    dists = np.empty((m, K), dtype=np.float32)
    flags = np.empty((m, K), dtype=np.uint8)
    rc = _load().oracle_init_graph(_p(X), n, d, _p(np.ascontiguousarray(perm)),
                                   _p(np.ascontiguousarray(leaf_off)),
                                   _p(np.ascontiguousarray(n_leaves)), T, K,
                                   None if rows_arr is None else _p(rows_arr), m,
                                   _p(ids), _p(dists), _p(flags))
    if rc != 0:
        raise ValueError(f"oracle_init_graph failed: {rc}")
    return ids, dists, flags


def search(X, perm, leaf_off, n_leaves, nodes, S: int, graph_ids, queries, K: int, P: int, E: int,
           iters: int):
    """Alg. 1 for a batch of queries.  Returns (ids [nq,K] int32, dists [nq,K] float32,
    checked [nq] int32 = distances evaluated per query)."""
    X = _f32(X)
    Q = _f32(queries)
    n, d = X.shape
    T = perm.shape[0]
    assert Q.shape[1] == d and nodes.shape == (T, n + 1) and nodes.dtype == NODE_DTYPE
    g = np.ascontiguousarray(graph_ids, dtype=np.int32)
    assert g.shape[0] == n
    nq = Q.shape[0]
    ids = np.empty((nq, K), dtype=np.int32)
    dists = np.empty((nq, K), dtype=np.float32)
    checked = np.zeros(nq, dtype=np.int32)
    rc = _load().oracle_search(_p(X), n, d, _p(np.ascontiguousarray(perm)),
                               _p(np.ascontiguousarray(leaf_off)), _p(np.ascontiguousarray(n_leaves)),
                               _p(np.ascontiguousarray(nodes)), T, S, _p(g), g.shape[1], _p(Q), nq, K, P, E,
                               iters, _p(ids), _p(dists), _p(checked))
    if rc != 0:
        raise ValueError(f"oracle_search failed: {rc}")
    return ids, dists, checked


def nndescent(X, ids, dists, flags, iters: int, L: int, seed: int, iter0: int = 0,
              delta: float = 0.0, cross_old: bool = False):
    """Alg. 4.  Returns new (ids, dists, flags) and stats [iters, 2] =
    (distance evaluations, accepted insertions) per iteration.  With delta > 0 (early
    termination) a fifth value follows: the number of iterations carried out, and stats
    has that many rows.  cross_old: entries inserted by a pair of a new and an old member are
    marked old (the literal marking of Alg. 4), pairs of two new members being inserted first."""
    X = _f32(X)
    n, d = X.shape
    K = ids.shape[1]
    ids = np.array(ids, dtype=np.int32, order="C")
    dists = np.array(dists, dtype=np.float32, order="C")
    flags = np.array(flags, dtype=np.uint8, order="C")
    stats = np.zeros((max(iters, 1), 2), dtype=np.uint64)
    done = C.c_int32(0)
    rc = _load().oracle_nndescent_opts(_p(X), n, d, K, _p(ids), _p(dists), _p(flags), iters, L, seed,
                                       iter0, _p(stats), float(delta), C.byref(done), 1 if cross_old else 0)
    if rc != 0:
        raise ValueError(f"oracle_nndescent failed: {rc}")
    if delta > 0.0:
        return ids, dists, flags, stats[:done.value], int(done.value)
    return ids, dists, flags, stats[:iters]
