"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, validates
arguments, and its host-side adjacency normalisation equals the oracle's bit for bit."""
import os
import re
import shutil
import subprocess

import numpy as np
import pytest

import paper_2105_09837_amd as P
from oracle import pdadmm_oracle as O
from workloads import get_workload, make_graph, scaled_workload, stream_rng

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(P.library_path()):
        from paper_2105_09837_amd.build import build_library
        build_library()
    return P.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "pdadmm.h")).read()
    declared = set(re.findall(r"\b(pdadmm_[a-z_]+)\s*\(", header))
    assert declared == set(P.exported_symbols())
    for name in declared:
        assert hasattr(lib, name), name


def test_header_is_plain_c_and_a_c_program_links_against_the_library(lib, tmp_path):
    """The boundary is a C ABI: the header must compile as C99 without warnings, and a C program that
    names every entry point must link against the shared library (no compute calls: no GPU here)."""
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    header = os.path.join(ROOT, "include", "pdadmm.h")
    res = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c", header],
                         capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    src = tmp_path / "link.c"
    names = sorted(P.exported_symbols())
    src.write_text('#include "pdadmm.h"\n#include <stdio.h>\nint main(void) {\n  const void* f[] = {' +
                   ", ".join(f"(const void*)(size_t){n}" for n in names) +
                   '};\n  printf("%d\\n", (int)(sizeof f / sizeof f[0]));\n  return f[0] == 0;\n}\n')
    exe = tmp_path / "link"
    libdir = os.path.dirname(P.library_path())
    res = subprocess.run([gcc, "-std=c99", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe),
                          "-L", libdir, "-l:libpdadmm.so", f"-Wl,-rpath,{libdir}"], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    # config validation through the linked program's view of the ABI: an invalid config needs no GPU
    cfg = P.Config(n_nodes=0, dims=[4, 2], rho=1.0, nu=1.0)
    assert P.pdadmm_workspace_bytes(cfg) == 0


@pytest.mark.parametrize("name,n", [("C1", 2000), ("C2", 5000), ("C3", 3000)])
def test_normalize_adj_matches_oracle_bit_for_bit(lib, name, n):
    w = scaled_workload(name, n)
    rp, ci = make_graph(w.graph, w.n_nodes, w.graph_param, stream_rng(w, 0))
    a = O.normalize_adj(rp, ci)
    b = P.pdadmm_normalize_adj(rp, ci)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert np.array_equal(a[2].view(np.uint32), b[2].view(np.uint32))


def test_normalize_adj_edge_cases_and_errors(lib):
    rp, ci, v = P.pdadmm_normalize_adj(np.zeros(1, dtype=np.int32), np.zeros(0, dtype=np.int32))
    assert rp.tolist() == [0] and ci.size == 0
    rp, ci, v = P.pdadmm_normalize_adj(np.zeros(4, dtype=np.int32), np.zeros(0, dtype=np.int32))
    assert ci.tolist() == [0, 1, 2] and np.all(v == 1.0)          # isolated nodes: A~ = I
    with pytest.raises(P.PdadmmError):                             # self-loop in the input
        P.pdadmm_normalize_adj(np.array([0, 1], dtype=np.int32), np.array([0], dtype=np.int32))
    with pytest.raises(P.PdadmmError):                             # column out of range
        P.pdadmm_normalize_adj(np.array([0, 1, 1], dtype=np.int32), np.array([5], dtype=np.int32))
    with pytest.raises(P.PdadmmError):                             # unsorted columns
        P.pdadmm_normalize_adj(np.array([0, 2, 2, 2], dtype=np.int32), np.array([2, 1], dtype=np.int32))


def test_workspace_size_and_config_validation(lib):
    w = get_workload("C2")
    good = P.Config(w.n_nodes, list(w.dims), w.rho, w.nu)
    nbytes = P.pdadmm_workspace_bytes(good)
    state = 4 * w.n_nodes * sum(w.dims)            # one [N, n] array per width, fp32
    assert nbytes > 3 * state and nbytes < 12 * state
    import dataclasses
    for bad in (dict(rho=0.0), dict(nu=-1.0), dict(n_nodes=0), dict(bt_eta=1.0), dict(dims=[5, 0, 3]),
                dict(quantize=1, q_levels=1), dict(quantize=1, q_levels=65537), dict(quantize=1, q_lo=1.0, q_hi=1.0),
                dict(quantize=3), dict(quantize=-1), dict(bt_max_trials=0), dict(tau0=0.0)):
        assert P.pdadmm_workspace_bytes(dataclasses.replace(good, **bad)) == 0, bad
    # p_l resident as indices: one byte each up to 256 levels, two above (two planes per layer)
    elems = 2 * w.n_nodes * sum(w.dims[1:-1])
    b8, b16 = (P.pdadmm_workspace_bytes(dataclasses.replace(good, quantize=1, q_levels=lv)) for lv in (256, 257))
    assert abs((b16 - b8) - elems) <= 1e-3 * elems
    q = dataclasses.replace(good, quantize=1)
    assert P.pdadmm_workspace_bytes(q) > nbytes
