"""GPU parity at the headline size: the whole path on `sift1m_like` (10^6 x 128, K=10, 8 trees,
leaves of 16, 8 NN-descent iterations, L=10), launched exactly as the benchmark launches it
(caller-provided workspaces, all iterations in one call, phase timing on), against the CPU
oracle run on the same input.  The pipeline is deterministic, so the comparison is of every
element, not of a sample; a sample of rows is also checked against float64 brute force."""
import numpy as np
import pytest

import oracle
from paper_1609_07228_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

NAME = "sift1m_like"


@pytest.mark.timeout(900)
def test_headline_workload_bit_exact_against_oracle():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: there is no CPU fallback")
    from paper_1609_07228_amd import efanna
    L_ = efanna.lib()
    p = synth.params(NAME)
    K, T, S, I, L = p["K"], p["T"], p["S"], p["I"], p["L"]
    X = synth.generate(NAME)
    n, d = X.shape
    assert (n, d) == (1_000_000, 128)
    dev = torch.device("cuda:0")
    Xd = torch.from_numpy(X).to(dev)

    # the benchmark's launch configuration
    ws_tree = torch.empty(L_.efanna_trees_workspace_bytes(n, d, T, S, 0), dtype=torch.uint8, device=dev)
    ws_init = torch.empty(max(256, L_.efanna_init_workspace_bytes(n, 0)), dtype=torch.uint8, device=dev)
    ws_nnd = torch.empty(L_.efanna_nndescent_workspace_bytes(n, K, L), dtype=torch.uint8, device=dev)
    graph = torch.empty((n, K), dtype=torch.int64, device=dev)
    stats = torch.zeros((I, 4), dtype=torch.int64, device=dev)
    phase_ms = np.zeros((I, 4), dtype=np.float32)
    max_leaves = n // max(1, S // 4) + 16
    perm, leaf_off, n_leaves = efanna.efanna_build_trees(Xd, T, S, synth.ALGO_SEED,
                                                         max_leaves=max_leaves, workspace=ws_tree)
    efanna.efanna_init_graph(Xd, perm, leaf_off, n_leaves, S, K, graph=graph, workspace=ws_init)
    init_ids, init_dists, init_flags = [t.cpu().numpy() for t in efanna.efanna_get_graph(graph, with_flags=True)]
    efanna.efanna_nndescent(Xd, graph, I, L, synth.ALGO_SEED, stats=stats, workspace=ws_nnd,
                            phase_ms=phase_ms)
    ids, dists, flags = [t.cpu().numpy() for t in efanna.efanna_get_graph(graph, with_flags=True)]
    st = stats.cpu().numpy()
    print("gpu path done", flush=True)

    # trees: every tree's permutation and leaf boundaries
    operm, ooff, onl = oracle.build_trees(X, T, S, synth.ALGO_SEED)
    assert np.array_equal(n_leaves, onl)
    assert np.array_equal(perm.cpu().numpy(), operm)
    goff = leaf_off.cpu().numpy()
    for t in range(T):
        assert np.array_equal(goff[t, :onl[t] + 1], ooff[t, :onl[t] + 1])
        assert np.diff(ooff[t, :onl[t] + 1]).max() <= S
    print("trees equal", flush=True)

    # initial graph
    want = oracle.init_graph(X, operm, ooff, onl, K)
    assert np.array_equal(init_ids, want[0])
    assert init_dists.tobytes() == want[1].tobytes()
    assert np.array_equal(init_flags, want[2])
    print("initial graph equal", flush=True)

    # refined graph and the number of pairs evaluated in every iteration
    want = oracle.nndescent(X, *want[:3], I, L, synth.ALGO_SEED)
    assert np.array_equal(ids, want[0])
    assert dists.tobytes() == want[1].tobytes()
    assert np.array_equal(flags, want[2])
    assert np.array_equal(st[:, 0], want[3][:, 0])
    print("refined graph equal", flush=True)

    # sampled rows against float64 brute force: structure, distances within 1e-5, accuracy
    rows = synth.sample_rows(n, 1000)
    oracle.check_graph_invariants(X, ids[rows], dists[rows], rows=rows)
    tid, _ = oracle.exact_knn(X, rows, K)
    r_gpu, r_cpu = oracle.recall(ids[rows], tid), oracle.recall(want[0][rows], tid)
    assert abs(r_gpu - r_cpu) <= 0.005
    assert r_gpu > 0.6
    assert (phase_ms[:, 1] > 0).all()
