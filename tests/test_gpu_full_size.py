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


def _progress(msg):
    print(msg, flush=True)      # shown with -s or on failure


@pytest.mark.timeout(600)
def test_sift100k_like_full_size_bit_exact():
    """The 100 000 x 128 configuration (K = 20, L = 20: joins of up to 60 vectors take the
    kernel with rows in LDS) at full size, every element against the oracle."""
    from paper_1609_07228_amd import efanna
    name = "sift100k_like"
    p = synth.params(name)
    X = synth.generate(name)
    Xd = torch.from_numpy(X).to("cuda:0")
    perm, off, nl = efanna.efanna_build_trees(Xd, p["T"], p["S"], synth.ALGO_SEED)
    graph = efanna.efanna_init_graph(Xd, perm, off, nl, p["S"], p["K"])
    stats = efanna.efanna_nndescent(Xd, graph, p["I"], p["L"], synth.ALGO_SEED)
    ids, dists, flags = [t.cpu().numpy() for t in efanna.efanna_get_graph(graph, with_flags=True)]
    operm, ooff, onl = oracle.build_trees(X, p["T"], p["S"], synth.ALGO_SEED)
    assert np.array_equal(perm.cpu().numpy(), operm)
    want = oracle.nndescent(X, *oracle.init_graph(X, operm, ooff, onl, p["K"]), p["I"], p["L"],
                            synth.ALGO_SEED)
    assert np.array_equal(ids, want[0]) and dists.tobytes() == want[1].tobytes()
    assert np.array_equal(flags, want[2])
    assert np.array_equal(stats.cpu().numpy()[:, 0].astype(np.uint64), want[3][:, 0])


def _full_size_properties(name, n_rows_init, n_rows_exact, refine_with_oracle=False):
    """Whole path at full size: trees and sampled rows of the initial graph bit-exact against
    the oracle, the refined graph checked through properties that hold at any size, and -
    where the oracle refines the graph in about half a minute (refine_with_oracle) - every
    element of the refined graph against it as well."""
    from paper_1609_07228_amd import efanna
    p = synth.params(name)
    K, T, S, I, L = p["K"], p["T"], p["S"], p["I"], p["L"]
    X = synth.generate(name)
    n, d = X.shape
    _progress(f"{name}: generated {n} x {d}")
    Xd = torch.from_numpy(X).to("cuda:0")
    max_leaves = n // max(1, S // 4) + 16
    perm, off, nl = efanna.efanna_build_trees(Xd, T, S, synth.ALGO_SEED, max_leaves=max_leaves)
    graph = efanna.efanna_init_graph(Xd, perm, off, nl, S, K)
    init_ids, init_dists = [t.cpu().numpy() for t in efanna.efanna_get_graph(graph)]
    stats = efanna.efanna_nndescent(Xd, graph, I, L, synth.ALGO_SEED).cpu().numpy()
    ids, dists = [t.cpu().numpy() for t in efanna.efanna_get_graph(graph)]
    _progress(f"{name}: gpu path done")
    # trees: every permutation and leaf boundary
    operm, ooff, onl = oracle.build_trees(X, T, S, synth.ALGO_SEED)
    assert np.array_equal(nl, onl) and np.array_equal(perm.cpu().numpy(), operm)
    goff = off.cpu().numpy()
    for t in range(T):
        assert np.array_equal(goff[t, :onl[t] + 1], ooff[t, :onl[t] + 1])
    _progress(f"{name}: trees equal")
    # initial graph: sampled rows, one by one
    rows = synth.sample_rows(n, n_rows_init)
    want = oracle.init_graph(X, operm, ooff, onl, K, rows=rows)
    assert np.array_equal(init_ids[rows], want[0])
    assert init_dists[rows].tobytes() == want[1].tobytes()
    _progress(f"{name}: initial graph rows equal")
    # refined graph: structure, stored distances, monotone improvement, accuracy
    oracle.check_graph_invariants(X, ids[rows], dists[rows], rows=rows)
    for r in rows[:64]:
        for c in (0, K // 2, K - 1):
            assert dists[r, c] == oracle.dist(X[r], X[ids[r, c]])
    assert np.all(dists[rows, K - 1] <= init_dists[rows, K - 1])      # the K-th distance never grows
    sub = rows[:n_rows_exact]
    tid, _ = oracle.exact_knn(X, sub, K)
    r0, r1 = oracle.recall(init_ids[sub], tid), oracle.recall(ids[sub], tid)
    _progress(f"{name}: accuracy {r0:.3f} -> {r1:.3f}")
    assert r1 > r0 + 0.2 and r1 > 0.5
    assert np.all(np.diff(stats[2:, 1].astype(np.int64)) < 0)          # insertions dry up
    if refine_with_oracle:
        full = oracle.nndescent(X, *oracle.init_graph(X, operm, ooff, onl, K), I, L, synth.ALGO_SEED)
        _progress(f"{name}: oracle refined")
        assert np.array_equal(ids, full[0]) and dists.tobytes() == full[1].tobytes()
        assert np.array_equal(stats[:, 0].astype(np.uint64), full[3][:, 0])
    return r1


@pytest.mark.timeout(900)
def test_gist1m_like_full_size_bit_exact():
    _full_size_properties("gist1m_like", 2000, 200, refine_with_oracle=True)


@pytest.mark.timeout(900)
def test_mixed4m_d96_full_size_properties():
    _full_size_properties("mixed4m_d96", 1000, 100)


@pytest.mark.timeout(900)
def test_mixed_d96_prefix_every_element_against_oracle():
    """The parameters of `mixed4m_d96` (K = 100, 16 trees, leaves of 64, L = 50) on its first
    262 144 rows, three iterations: rows of a hundred entries take the per-list counters with their
    overflow queues, the wide overflow kernel and the LDS-row join with its long-row list updates,
    at a size where the queues fill and hubs are fought over.  Every element of the trees, of the
    initial and of the refined graph and the pairs evaluated per iteration against the oracle,
    and both accuracies against exact brute force (Alg. 3 at the leaves, Alg. 4)."""
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: there is no CPU fallback")
    from paper_1609_07228_amd import efanna
    name, n, iters = "mixed4m_d96", 4 * synth.CHUNK, 3
    p = synth.params(name)
    K, T, S, L = p["K"], p["T"], p["S"], p["L"]
    X = synth.generate(name, n=n)
    Xd = torch.from_numpy(X).to("cuda:0")
    perm, off, nl = efanna.efanna_build_trees(Xd, T, S, synth.ALGO_SEED, max_leaves=n // (S // 4) + 16)
    graph = efanna.efanna_init_graph(Xd, perm, off, nl, S, K)
    init = [t.cpu().numpy() for t in efanna.efanna_get_graph(graph, with_flags=True)]
    stats = efanna.efanna_nndescent(Xd, graph, iters, L, synth.ALGO_SEED).cpu().numpy()
    ids, dists, flags = [t.cpu().numpy() for t in efanna.efanna_get_graph(graph, with_flags=True)]
    _progress(f"{name}[:{n}]: gpu path done")
    operm, ooff, onl = oracle.build_trees(X, T, S, synth.ALGO_SEED)
    assert np.array_equal(nl, onl) and np.array_equal(perm.cpu().numpy(), operm)
    goff = off.cpu().numpy()
    for t in range(T):
        assert np.array_equal(goff[t, :onl[t] + 1], ooff[t, :onl[t] + 1])
    _progress(f"{name}[:{n}]: trees equal")
    want = oracle.init_graph(X, operm, ooff, onl, K)
    assert np.array_equal(init[0], want[0])
    assert init[1].tobytes() == want[1].tobytes()
    assert np.array_equal(init[2], want[2])
    _progress(f"{name}[:{n}]: initial graph equal")
    evals = []
    for it in range(iters):      # one iteration per call (equal to one call of three) so that progress shows
        want = oracle.nndescent(X, *want[:3], 1, L, synth.ALGO_SEED, iter0=it)
        evals.append(want[3][0, 0])
        _progress(f"{name}[:{n}]: oracle iteration {it + 1} done")
    want = (*want[:3], np.array(evals, dtype=np.uint64)[:, None])
    assert np.array_equal(ids, want[0])
    assert dists.tobytes() == want[1].tobytes()
    assert np.array_equal(flags, want[2])
    assert np.array_equal(stats[:, 0].astype(np.uint64), want[3][:, 0])
    rows = synth.sample_rows(n, 500)
    oracle.check_graph_invariants(X, ids[rows], dists[rows], rows=rows)
    tid, _ = oracle.exact_knn(X, rows, K)
    r_gpu, r_cpu = oracle.recall(ids[rows], tid), oracle.recall(want[0][rows], tid)
    _progress(f"{name}[:{n}]: accuracy {r_gpu:.4f} (oracle {r_cpu:.4f})")
    assert abs(r_gpu - r_cpu) <= 0.005
    assert r_gpu > oracle.recall(init[0][rows], tid)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("n", [1 << 21, (1 << 21) + 1])
def test_two_million_short_vectors_bit_exact(n):
    """The largest point count whose reverse lists are built by target ranges (2048 ranges, the
    most an offer block's table takes), and one point more, which goes the way of the per-list
    counters: tiny vectors, so that the oracle follows in seconds."""
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: there is no CPU fallback")
    from paper_1609_07228_amd import efanna
    d, T, S, K, L, I = 4, 1, 8, 4, 4, 2
    X = np.random.default_rng(n).standard_normal((n, d)).astype(np.float32)
    Xd = torch.from_numpy(X).to("cuda:0")
    perm, leaf_off, n_leaves = efanna.efanna_build_trees(Xd, T, S, 3, max_leaves=n // 2 + 16)
    graph = efanna.efanna_init_graph(Xd, perm, leaf_off, n_leaves, S, K)
    stats = efanna.efanna_nndescent(Xd, graph, I, L, 3).cpu().numpy()
    ids, dists, flags = [t.cpu().numpy() for t in efanna.efanna_get_graph(graph, with_flags=True)]
    print("gpu path done", flush=True)
    operm, ooff, onl = oracle.build_trees(X, T, S, 3)
    assert np.array_equal(perm.cpu().numpy(), operm)
    want = oracle.nndescent(X, *oracle.init_graph(X, operm, ooff, onl, K), I, L, 3)
    assert np.array_equal(ids, want[0])
    assert np.array_equal(dists.view(np.uint32), want[1].view(np.uint32))
    assert np.array_equal(flags, want[2])
    assert np.array_equal(stats[:, 0].astype(np.int64), want[3][:, 0].astype(np.int64))
