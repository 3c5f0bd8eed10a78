"""Thin Python binding of the C ABI declared in include/efanna.h.

Argument marshalling only: every step runs in the HIP kernels of libefanna_hip.so.
torch provides device memory and the current stream.  There is no CPU fallback: a
missing library or a missing GPU raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

from . import build as _build

_lib = None

STATUS = {0: "EFANNA_OK", -1: "EFANNA_EINVAL", -2: "EFANNA_EWORKSPACE", -3: "EFANNA_EINPUT",
          -4: "EFANNA_EHIP", -5: "EFANNA_ECAPACITY", -6: "EFANNA_EUNSUPPORTED", -7: "EFANNA_ESCRATCH"}

# every symbol include/efanna.h declares
SYMBOLS = ["efanna_status_string", "efanna_trees_workspace_bytes", "efanna_build_trees", "efanna_build_trees_rule",
           "efanna_init_workspace_bytes", "efanna_init_graph", "efanna_nndescent_workspace_bytes",
           "efanna_nndescent", "efanna_nndescent_noalloc", "efanna_get_graph", "efanna_set_graph", "efanna_pair_distances",
           "efanna_search_workspace_bytes", "efanna_search"]


class EfannaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().efanna_status_string(status).decode()
        super().__init__(f"{where}: {STATUS.get(status, status)} ({msg})")


def lib():
    """Load libefanna_hip.so (built in-tree by build.py); never builds implicitly on a
    machine without hipcc, never falls back to anything else."""
    global _lib
    if _lib is None:
        path = os.environ.get("EFANNA_HIP_LIBRARY") or _build.LIB   # override: another build of the same sources
        if not os.path.exists(path):
            _build.build()
        L = C.CDLL(path)
        vp, i64, i32, u64, sz = C.c_void_p, C.c_int64, C.c_int32, C.c_uint64, C.c_size_t
        L.efanna_status_string.restype = C.c_char_p
        L.efanna_status_string.argtypes = [C.c_int]
        L.efanna_trees_workspace_bytes.restype = sz
        L.efanna_trees_workspace_bytes.argtypes = [i64, i32, i32, i32, i32]
        L.efanna_build_trees.restype = C.c_int
        L.efanna_build_trees.argtypes = [vp, i64, i32, i32, i32, u64, vp, vp, i32, vp, vp, vp, vp, vp, sz, vp]
        L.efanna_build_trees_rule.restype = C.c_int
        L.efanna_build_trees_rule.argtypes = [vp, i64, i32, i32, i32, u64, i32, vp, vp, i32, vp, vp, vp, vp, vp, sz, vp]
        L.efanna_init_workspace_bytes.restype = sz
        L.efanna_init_workspace_bytes.argtypes = [i64, i32]
        L.efanna_init_graph.restype = C.c_int
        L.efanna_init_graph.argtypes = [vp, i64, i32, vp, vp, i32, vp, vp, vp, i32, i32, i32, i32, i32, vp, vp, sz, vp]
        L.efanna_nndescent_workspace_bytes.restype = sz
        L.efanna_nndescent_workspace_bytes.argtypes = [i64, i32, i32]
        L.efanna_nndescent.restype = C.c_int
        L.efanna_nndescent.argtypes = [vp, i64, i32, i32, vp, i32, i32, u64, i32, C.c_float, i32, vp, vp, vp, vp, sz, vp]
        L.efanna_nndescent_noalloc.restype = C.c_int
        L.efanna_nndescent_noalloc.argtypes = [vp, i64, i32, i32, vp, i32, i32, u64, i32, vp, vp]
        L.efanna_get_graph.restype = C.c_int
        L.efanna_get_graph.argtypes = [vp, i64, i32, vp, vp, vp, vp]
        L.efanna_set_graph.restype = C.c_int
        L.efanna_set_graph.argtypes = [vp, i64, i32, vp, vp, vp, vp]
        L.efanna_pair_distances.restype = C.c_int
        L.efanna_pair_distances.argtypes = [vp, i64, i32, vp, vp, i64, vp, vp]
        L.efanna_search_workspace_bytes.restype = sz
        L.efanna_search_workspace_bytes.argtypes = [i64, i32, i32, i32, i32, i32, i32, i32]
        L.efanna_search.restype = C.c_int
        L.efanna_search.argtypes = [vp, i64, i32, vp, vp, i32, vp, vp, i32, i32, i32, vp, i32, vp, i64,
                                    i32, i32, i32, i32, vp, vp, vp, vp, sz, vp]
        _lib = L
    return _lib


def _check(status: int, where: str):
    if status != 0:
        raise EfannaError(status, where)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, dtype) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError("expected a device tensor")
    if t.dtype != dtype or not t.is_contiguous():
        raise ValueError(f"expected contiguous {dtype}, got {t.dtype}")
    return t


def _workspace(nbytes: int, device) -> torch.Tensor:
    # torch's caching allocator hands out 512-byte aligned blocks
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


NODE_BYTES = 32      # sizeof(efanna_node): int64 sum; int32 dim, cnt, parent, depth, child[2]


SPLIT_UNIFORM, SPLIT_VARIANCE, SPLIT_PROJECTION = 0, 1, 2


def efanna_build_trees_rule(X: torch.Tensor, n_trees: int, leaf_size: int, seed: int, split_rule: int,
                            max_leaves: int | None = None, workspace: torch.Tensor | None = None,
                            with_nodes: bool = False):
    """Alg. 2 with the split dimension taken by `split_rule` (SPLIT_UNIFORM: drawn over all d,
    SPLIT_VARIANCE: drawn among the five dimensions of largest variance, SPLIT_PROJECTION: a signed
    sum of eight coordinates instead of one).  Returns what
    efanna_build_trees returns."""
    return efanna_build_trees(X, n_trees, leaf_size, seed, max_leaves, workspace, with_nodes, _rule=int(split_rule))


def efanna_build_trees(X: torch.Tensor, n_trees: int, leaf_size: int, seed: int,
                       max_leaves: int | None = None, workspace: torch.Tensor | None = None,
                       with_nodes: bool = False, _rule: int | None = None):
    """Alg. 2.  Returns (perm [T,n] int32 device, leaf_off [T,max_leaves+1] int32 device,
    n_leaves [T] int32 numpy) and, with_nodes, also (nodes [T,max_leaves+1,32] uint8 device
    holding efanna_node records, leaf_up [T,max_leaves+1] int32 device, tree_depth int: depth of
    the deepest internal node).  Synchronises the current stream."""
    X = _dev(X, torch.float32)
    n, d = X.shape
    max_leaves = n if max_leaves is None else int(max_leaves)
    perm = torch.empty((n_trees, n), dtype=torch.int32, device=X.device)
    leaf_off = torch.empty((n_trees, max_leaves + 1), dtype=torch.int32, device=X.device)
    n_leaves = np.zeros(n_trees, dtype=np.int32)
    nodes = leaf_up = None
    if with_nodes:
        nodes = torch.zeros((n_trees, max_leaves + 1, NODE_BYTES), dtype=torch.uint8, device=X.device)
        leaf_up = torch.full((n_trees, max_leaves + 1), -1, dtype=torch.int32, device=X.device)
    depth = C.c_int32(-1)
    need = lib().efanna_trees_workspace_bytes(n, d, n_trees, leaf_size, 1 if with_nodes else 0)
    ws = _workspace(need, X.device) if workspace is None else workspace
    tail = (perm.data_ptr(), leaf_off.data_ptr(), max_leaves, n_leaves.ctypes.data_as(C.c_void_p),
            nodes.data_ptr() if with_nodes else None, leaf_up.data_ptr() if with_nodes else None,
            C.byref(depth), ws.data_ptr(), ws.numel(), _stream())
    if _rule is None:
        _check(lib().efanna_build_trees(X.data_ptr(), n, d, n_trees, leaf_size, seed, *tail), "efanna_build_trees")
    else:
        _check(lib().efanna_build_trees_rule(X.data_ptr(), n, d, n_trees, leaf_size, seed, _rule, *tail),
               "efanna_build_trees_rule")
    if with_nodes:
        return perm, leaf_off, n_leaves, nodes, leaf_up, int(depth.value)
    return perm, leaf_off, n_leaves


def efanna_init_graph(X: torch.Tensor, perm: torch.Tensor, leaf_off: torch.Tensor,
                      n_leaves: np.ndarray, leaf_size: int, k: int,
                      graph: torch.Tensor | None = None, workspace: torch.Tensor | None = None,
                      nodes: torch.Tensor | None = None, leaf_up: torch.Tensor | None = None,
                      tree_depth: int = -1, conquer_depth: int = 0):
    """Alg. 3.  Without nodes the conquer step stops at the leaves; with (nodes, leaf_up,
    tree_depth) from efanna_build_trees it walks up to `conquer_depth` (0 = the root).
    Returns the packed graph [n,k] (int64 tensor holding the 64-bit entries)."""
    X = _dev(X, torch.float32)
    n, d = X.shape
    perm = _dev(perm, torch.int32)
    leaf_off = _dev(leaf_off, torch.int32)
    T = perm.shape[0]
    n_leaves = np.ascontiguousarray(n_leaves, dtype=np.int32)
    if (nodes is None) != (leaf_up is None):
        raise ValueError("nodes and leaf_up come together")
    if nodes is not None:
        nodes = _dev(nodes, torch.uint8)
        leaf_up = _dev(leaf_up, torch.int32)
        if nodes.shape != (T, leaf_off.shape[1], NODE_BYTES) or leaf_up.shape != leaf_off.shape:
            raise ValueError("nodes / leaf_up do not match leaf_off")
    if graph is None:
        graph = torch.empty((n, k), dtype=torch.int64, device=X.device)
    levels = 0 if nodes is None else int(tree_depth) - int(conquer_depth) + 1
    need = lib().efanna_init_workspace_bytes(n, levels)
    ws = _workspace(need, X.device) if workspace is None else workspace
    _check(lib().efanna_init_graph(X.data_ptr(), n, d, perm.data_ptr(), leaf_off.data_ptr(),
                                   leaf_off.shape[1] - 1, n_leaves.ctypes.data_as(C.c_void_p),
                                   nodes.data_ptr() if nodes is not None else None,
                                   leaf_up.data_ptr() if nodes is not None else None,
                                   int(tree_depth), int(conquer_depth), T, leaf_size, k, graph.data_ptr(),
                                   ws.data_ptr(), ws.numel(), _stream()), "efanna_init_graph")
    return graph


def efanna_nndescent(X: torch.Tensor, graph: torch.Tensor, iters: int, sample_L: int, seed: int,
                     first_iter: int = 0, stats: torch.Tensor | None = None,
                     workspace: torch.Tensor | None = None, phase_ms: np.ndarray | None = None,
                     delta: float = 0.0, cross_old: bool = False):
    """Alg. 4, in place on `graph`.  Returns stats [iters,4] (int64 device tensor:
    distance evaluations, accepted insertions, vectors gathered, vectors gathered by the
    joins of at most 16 vectors).  `phase_ms`, if given, is a float32 numpy array
    [iters,4] that receives (sampling, small / medium / large joins) times and makes the
    call synchronise.  With delta > 0 (early termination) the call synchronises after every
    iteration and returns (stats of the iterations carried out, their number).  cross_old: the
    literal marking of Alg. 4 (entries inserted by a new and an old member are marked old)."""
    X = _dev(X, torch.float32)
    n, d = X.shape
    graph = _dev(graph, torch.int64)
    k = graph.shape[1]
    if stats is None:
        stats = torch.zeros((max(iters, 1), 4), dtype=torch.int64, device=X.device)
    if phase_ms is not None:
        assert phase_ms.dtype == np.float32 and phase_ms.size >= 4 * iters and phase_ms.flags.c_contiguous
    need = lib().efanna_nndescent_workspace_bytes(n, k, sample_L)
    ws = _workspace(need, X.device) if workspace is None else workspace
    done = C.c_int32(0)
    _check(lib().efanna_nndescent(X.data_ptr(), n, d, k, graph.data_ptr(), iters, sample_L, seed,
                                  first_iter, float(delta), 1 if cross_old else 0, C.byref(done), stats.data_ptr(),
                                  None if phase_ms is None else phase_ms.ctypes.data_as(C.c_void_p),
                                  ws.data_ptr(), ws.numel(), _stream()), "efanna_nndescent")
    if delta > 0.0:
        return stats[:done.value], int(done.value)
    return stats[:iters]


def efanna_nndescent_noalloc(X: torch.Tensor, graph: torch.Tensor, iters: int, sample_L: int, seed: int,
                             stats: torch.Tensor, first_iter: int = 0):
    """efanna_nndescent on the library's fixed scratch array: the call itself allocates nothing,
    so `stats` ([iters,4] int64 device tensor) comes from the caller.  Returns stats."""
    X = _dev(X, torch.float32)
    n, d = X.shape
    graph = _dev(graph, torch.int64)
    stats = _dev(stats, torch.int64)
    if stats.numel() < 4 * max(iters, 1):
        raise ValueError("stats holds fewer than 4 * iters values")
    _check(lib().efanna_nndescent_noalloc(X.data_ptr(), n, d, graph.shape[1], graph.data_ptr(), iters,
                                          sample_L, seed, first_iter, stats.data_ptr(), _stream()),
           "efanna_nndescent_noalloc")
    return stats


def efanna_get_graph(graph: torch.Tensor, with_flags: bool = False):
    """Sorted rows: (ids [n,k] int32, dists [n,k] float32[, flags [n,k] uint8])."""
    graph = _dev(graph, torch.int64)
    n, k = graph.shape
    ids = torch.empty((n, k), dtype=torch.int32, device=graph.device)
    dists = torch.empty((n, k), dtype=torch.float32, device=graph.device)
    flags = torch.empty((n, k), dtype=torch.uint8, device=graph.device) if with_flags else None
    _check(lib().efanna_get_graph(graph.data_ptr(), n, k, ids.data_ptr(), dists.data_ptr(),
                                  flags.data_ptr() if with_flags else None, _stream()),
           "efanna_get_graph")
    return (ids, dists, flags) if with_flags else (ids, dists)


def efanna_set_graph(ids: torch.Tensor, dists: torch.Tensor, flags: torch.Tensor | None = None):
    """Pack rows into a graph tensor [n,k] int64."""
    ids = _dev(ids, torch.int32)
    dists = _dev(dists, torch.float32)
    n, k = ids.shape
    if flags is not None:
        flags = _dev(flags, torch.uint8)
    graph = torch.empty((n, k), dtype=torch.int64, device=ids.device)
    _check(lib().efanna_set_graph(graph.data_ptr(), n, k, ids.data_ptr(), dists.data_ptr(),
                                  flags.data_ptr() if flags is not None else None, _stream()),
           "efanna_set_graph")
    return graph


def efanna_pair_distances(X: torch.Tensor, a_ids: torch.Tensor, b_ids: torch.Tensor):
    X = _dev(X, torch.float32)
    a_ids = _dev(a_ids, torch.int32)
    b_ids = _dev(b_ids, torch.int32)
    out = torch.empty(a_ids.shape[0], dtype=torch.float32, device=X.device)
    _check(lib().efanna_pair_distances(X.data_ptr(), X.shape[0], X.shape[1], a_ids.data_ptr(),
                                       b_ids.data_ptr(), a_ids.shape[0], out.data_ptr(), _stream()),
           "efanna_pair_distances")
    return out


def efanna_search(X: torch.Tensor, perm: torch.Tensor, leaf_off: torch.Tensor, n_leaves: np.ndarray,
                  nodes: torch.Tensor, tree_depth: int, leaf_size: int, graph_ids: torch.Tensor,
                  queries: torch.Tensor, k: int, pool: int, expand: int, iters: int,
                  workspace: torch.Tensor | None = None):
    """Alg. 1 for a batch of queries.  Returns (ids [nq,k] int32, dists [nq,k] float32,
    checked [nq] int32: distances evaluated per query).  Synchronises the current stream."""
    X = _dev(X, torch.float32)
    Q = _dev(queries, torch.float32)
    n, d = X.shape
    nq = Q.shape[0]
    perm = _dev(perm, torch.int32)
    leaf_off = _dev(leaf_off, torch.int32)
    nodes = _dev(nodes, torch.uint8)
    g = _dev(graph_ids, torch.int32)
    T = perm.shape[0]
    n_leaves = np.ascontiguousarray(n_leaves, dtype=np.int32)
    if Q.shape[1] != d or g.shape[0] != n or nodes.shape != (T, leaf_off.shape[1], NODE_BYTES):
        raise ValueError("shapes of queries / graph / nodes do not match")
    ids = torch.empty((nq, k), dtype=torch.int32, device=X.device)
    dists = torch.empty((nq, k), dtype=torch.float32, device=X.device)
    checked = torch.empty((nq,), dtype=torch.int32, device=X.device)
    need = lib().efanna_search_workspace_bytes(nq, d, T, leaf_size, tree_depth, g.shape[1], pool, iters)
    ws = _workspace(need, X.device) if workspace is None else workspace
    _check(lib().efanna_search(X.data_ptr(), n, d, perm.data_ptr(), leaf_off.data_ptr(),
                               leaf_off.shape[1] - 1, n_leaves.ctypes.data_as(C.c_void_p),
                               nodes.data_ptr(), int(tree_depth), T, leaf_size, g.data_ptr(), g.shape[1],
                               Q.data_ptr(), nq, k, pool, expand, iters, ids.data_ptr(), dists.data_ptr(),
                               checked.data_ptr(), ws.data_ptr(), ws.numel(), _stream()), "efanna_search")
    return ids, dists, checked
