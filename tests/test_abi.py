"""Host-side checks that need no GPU: the library loads, exports every symbol the
header declares, sizes its workspaces sensibly and rejects bad arguments before
touching the device."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_1609_07228_amd import build
    if build.stale():
        build.build()
    from paper_1609_07228_amd import efanna
    return efanna.lib()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "efanna.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(efanna_[a-z_]+)\s*\(", header))
    assert len(declared) >= 10
    from paper_1609_07228_amd import efanna
    assert declared == set(efanna.SYMBOLS)
    for name in declared:
        assert hasattr(lib, name), name


def test_binding_passes_as_many_arguments_as_the_header_declares(lib):
    header = open(os.path.join(ROOT, "include", "efanna.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    protos = re.findall(r"\b(efanna_[a-z_]+)\s*\(([^)]*)\)\s*;", header)
    assert len(protos) >= 10
    for name, args in protos:
        n_args = 0 if args.strip() in ("", "void") else len(args.split(","))
        assert len(getattr(lib, name).argtypes) == n_args, name


def test_status_strings(lib):
    for s in range(0, -7, -1):
        assert lib.efanna_status_string(s)
    assert lib.efanna_status_string(0) == b"ok"


def test_workspace_sizes(lib):
    assert lib.efanna_trees_workspace_bytes(0, 4, 1, 1, 0) == 0
    a = lib.efanna_trees_workspace_bytes(1000, 16, 4, 8, 0)
    b = lib.efanna_trees_workspace_bytes(2000, 16, 4, 8, 0)
    assert 0 < a < b and a % 256 == 0
    assert lib.efanna_trees_workspace_bytes(1000, 16, 4, 8, 1) >= a + 1000 * 4 * 36      # node records
    assert lib.efanna_nndescent_workspace_bytes(1_000_000, 10, 10) < 600 * 2 ** 20
    assert lib.efanna_init_workspace_bytes(1000, 0) == 256
    assert lib.efanna_init_workspace_bytes(1000, 5) >= 1000 * 5 * 4


def test_argument_errors_are_caught_on_the_host(lib):
    null = None
    one = C.c_void_p(256)      # never dereferenced: every call below must fail first
    assert lib.efanna_build_trees(null, 10, 4, 1, 2, 0, one, one, 10, one, None, None, None, one, 1 << 20, None) == -1
    assert lib.efanna_build_trees(one, 10, 0, 1, 2, 0, one, one, 10, one, None, None, None, one, 1 << 20, None) == -1
    assert lib.efanna_build_trees(one, 10, 4, 65, 2, 0, one, one, 10, one, None, None, None, one, 1 << 20, None) == -1
    assert lib.efanna_build_trees(one, 10, 4, 1, 65, 0, one, one, 10, one, None, None, None, one, 1 << 20, None) == -1
    assert lib.efanna_build_trees(one, 10, 4, 1, 2, 0, one, one, 10, one, None, None, None, None, 0, None) == -2
    assert lib.efanna_build_trees(one, 10, 4, 1, 2, 0, one, one, 10, one, None, None, None, C.c_void_p(257), 1 << 20, None) == -2
    assert lib.efanna_build_trees(one, 10, 4, 1, 2, 0, one, one, 10, one, None, None, None, one, 16, None) == -2
    # nodes without leaf_up (and the reverse) is an argument error
    assert lib.efanna_build_trees(one, 10, 4, 1, 2, 0, one, one, 10, one, one, None, None, one, 1 << 20, None) == -1
    assert lib.efanna_init_graph(one, 10, 4, one, one, 10, one, None, one, 5, 0, 1, 2, 3, one, one, 256, None) == -1
    assert lib.efanna_nndescent(one, 10, 4, 10, one, 1, 4, 0, 0, 0.0, 0, None, None, None, one, 1 << 20, None) == -1  # k >= n
    assert lib.efanna_nndescent(one, 100, 4, 129, one, 1, 4, 0, 0, 0.0, 0, None, None, None, one, 1 << 30, None) == -1
    assert lib.efanna_nndescent(one, 100, 4, 10, one, 1, 4, 0, 0, -1.0, 0, None, None, None, one, 1 << 30, None) == -1  # delta < 0
    assert lib.efanna_get_graph(null, 10, 4, one, one, None, None) == -1
    assert lib.efanna_set_graph(one, 10, 0, one, one, None, None) == -1
    assert lib.efanna_pair_distances(one, 10, 4, null, one, 5, one, None) == -1


def test_bench_refuses_more_than_one_gpu_and_has_no_cpu_fallback():
    import subprocess
    import sys
    bench = os.path.join(ROOT, "bench.py")
    run = subprocess.run([sys.executable, bench, "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert run.returncode == 2 and "one GPU" in run.stderr and run.stdout.strip() == ""
    import torch
    if not torch.cuda.is_available():      # on a box without a GPU the bench must stop, not fall back
        run = subprocess.run([sys.executable, bench, "--steps", "1", "--warmup", "0"], capture_output=True,
                             text=True, timeout=300)
        assert run.returncode == 3 and "no CPU fallback" in run.stderr and run.stdout.strip() == ""


def test_product_path_does_not_import_the_oracle():
    """Only tests, the smoke check and the bench's cpu_baseline leg may touch oracle/."""
    pkg = os.path.join(ROOT, "paper_1609_07228_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".c", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(import|from)\s+oracle\b|#include.*oracle|libefanna_oracle", text, flags=re.M), \
                    os.path.join(dirpath, f)
    bench = open(os.path.join(ROOT, "bench.py")).read()
    assert bench.count("import oracle") == 1 and "if args.cpu_rows > 0:" in bench
