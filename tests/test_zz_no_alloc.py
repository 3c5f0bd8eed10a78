"""efanna_nndescent_noalloc (the entry point for callers that cannot allocate: its scratch is a
fixed device array inside the library) against efanna_nndescent on a caller's workspace: the
same graph, marks and work counters, bit for bit, on two calls in a row, the second with a
smaller input (the array keeps the first call's contents).  Named so that it is collected last."""
import ctypes as C

import numpy as np
import pytest

from paper_1609_07228_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _both_ways(X, K, T, S, L, iters, seed):
    from paper_1609_07228_amd import efanna
    Xd = torch.from_numpy(X).to("cuda:0")
    perm, off, nl = efanna.efanna_build_trees(Xd, T, S, seed)
    start = efanna.efanna_init_graph(Xd, perm, off, nl, S, K)
    # reference: the existing entry point on a workspace of the caller's
    g_ref = start.clone()
    st_ref = efanna.efanna_nndescent(Xd, g_ref, iters, L, seed)
    want = [t.cpu().numpy() for t in efanna.efanna_get_graph(g_ref, with_flags=True)]
    # the entry point under test, straight through the C ABI; everything it touches is allocated before the call
    g = start.clone()
    stats = torch.zeros((iters, 4), dtype=torch.int64, device="cuda:0")
    torch.cuda.synchronize()
    n, d = X.shape
    rc = efanna.lib().efanna_nndescent_noalloc(Xd.data_ptr(), n, d, K, g.data_ptr(), iters, L, seed, 0,
                                               stats.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert rc == 0, efanna.lib().efanna_status_string(rc)
    got = [t.cpu().numpy() for t in efanna.efanna_get_graph(g, with_flags=True)]
    assert np.array_equal(got[0], want[0])
    assert got[1].tobytes() == want[1].tobytes()
    assert np.array_equal(got[2], want[2])
    # distance evaluations and vectors gathered are deterministic (insertions made are not)
    assert np.array_equal(stats.cpu().numpy()[:, [0, 2, 3]], st_ref.cpu().numpy()[:, [0, 2, 3]])
    return got


def test_noalloc_equals_workspace_entry_point_twice():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: there is no CPU fallback")
    p = synth.params("gmm10k_d32")
    X = synth.generate("gmm10k_d32")
    first = _both_ways(X, p["K"], p["T"], p["S"], p["L"], 3, synth.ALGO_SEED)
    # a smaller input next, other row and list lengths (the counter scheme: rows longer than 32)
    second = _both_ways(X[:3001, :20].copy(), 40, 2, 12, 12, 2, 5)
    assert first[0].shape == (10_000, 10) and second[0].shape == (3001, 40)


def test_noalloc_rejects_what_does_not_fit():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: there is no CPU fallback")
    from paper_1609_07228_amd import efanna
    L_ = efanna.lib()
    n, d, K, L = 400_000, 4, 10, 10
    assert L_.efanna_nndescent_workspace_bytes(n, K, L) > 64 << 20
    X = torch.zeros((n, d), dtype=torch.float32, device="cuda:0")
    g = torch.zeros((n, K), dtype=torch.int64, device="cuda:0")
    rc = L_.efanna_nndescent_noalloc(X.data_ptr(), n, d, K, g.data_ptr(), 1, L, 1, 0, None, None)
    assert rc == -7
    assert b"scratch" in L_.efanna_status_string(rc)
    # and the largest point count that does fit is accepted by the size test
    lo, hi = 1000, n
    while hi - lo > 1:
        mid = (lo + hi) // 2
        lo, hi = (mid, hi) if L_.efanna_nndescent_workspace_bytes(mid, K, L) <= 64 << 20 else (lo, mid)
    assert lo > 100_000
