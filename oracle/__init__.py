"""CPU oracle (test infrastructure only): plain C implementation of the paper's
Alg. 1 (search), Alg. 2, Alg. 3 (conquer step, down to a chosen depth) and Alg. 4, plus exact brute-force kNN and the
accuracy measure of eqs. (2)-(3).  Only tests, the smoke check and the benchmark's
CPU-baseline leg may import this package; the GPU library never does."""
from .binding import (build, dist, build_trees, build_trees_nodes, conquer_graph, init_graph,
                      nndescent, search, num_threads, set_num_threads, node_rand, reverse_hash, NODE_DTYPE)
from .exact import exact_knn, exact_knn_definition, recall, check_graph_invariants

__all__ = ["build", "dist", "build_trees", "build_trees_nodes", "conquer_graph", "NODE_DTYPE", "init_graph", "search", "nndescent", "num_threads", "set_num_threads",
           "node_rand", "reverse_hash", "exact_knn", "exact_knn_definition", "recall",
           "check_graph_invariants"]
