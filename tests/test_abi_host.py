"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, and its host logic
(graph construction, argument checking) agrees bit for bit with the oracle's graph part.  No GPU call."""
import os
import re

import numpy as np
import pytest

from oracle.graph import OracleGraph
from paper_2112_09335_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "cadmm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cadmm_[a-zA-Z_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = binding.load_library()
    names = declared_symbols()
    assert len(names) >= 20
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def host_solver():
    return binding.Solver(device=-1)


def check_graph(N, src, dst, M, comm):
    s = host_solver()
    s.build_graph(N, src, dst, M, comm)
    g = s.get_graph()
    o = OracleGraph(N, src, dst, M, comm)
    nnz, nseg, nhalo = s.graph_sizes()
    assert (nnz, nseg, nhalo) == (o.nnz, o.n_segments, o.n_halo_rows)
    assert np.array_equal(g["perm"], o.perm)
    assert np.array_equal(g["row_ptr"], o.row_ptr)
    assert np.array_equal(g["col"], o.col)
    assert np.array_equal(g["val"].view(np.uint32), o.val.astype(np.float32).view(np.uint32))   # bit-exact
    assert np.array_equal(g["seg_ptr"], o.seg_ptr)
    assert np.array_equal(g["seg_row"], o.seg_row)
    assert np.array_equal(g["seg_comm"], o.seg_comm)
    assert np.array_equal(g["comm_row_ptr"], o.comm_row_ptr)
    assert np.array_equal(g["neighbour"], o.neighbour)
    # the (community, row) order is a stable sort of the segments on their community
    order = s.get_segment_order()
    assert np.array_equal(order, np.argsort(o.seg_comm, kind="stable"))
    s.close()


def test_graph_matches_oracle_on_config_1():
    w = synth.config(1)
    check_graph(w.N, w.src, w.dst, w.M, w.comm)


@pytest.mark.parametrize("idx,scale", [(2, 0.25), (3, 0.05), (4, 0.01), (5, 0.02)])
def test_graph_matches_oracle_on_scaled_configs(idx, scale):
    w = synth.config(idx, scale)
    check_graph(w.N, w.src, w.dst, w.M, w.comm)


def test_graph_with_noise_edges_empty_communities_and_default_partition():
    rng = np.random.default_rng(0)
    N, M = 300, 7
    src = rng.integers(0, N, size=2000)
    dst = rng.integers(0, N, size=2000)
    src[::7] = dst[::7]                                   # self pairs
    src = np.concatenate([src, dst[:500]])                # reversed repeats
    dst = np.concatenate([dst, src[:500]])
    comm = rng.choice([0, 1, 3, 6], size=N)               # communities 2, 4, 5 are empty
    check_graph(N, src, dst, M, comm.astype(np.int32))
    check_graph(N, src, dst, 4, None)                     # contiguous chunks
    check_graph(N, src, dst, 1, None)                     # one community
    check_graph(5, np.zeros(0, np.int32), np.zeros(0, np.int32), 2, None)    # no edges


def test_bad_arguments_are_rejected_with_error_codes():
    s = host_solver()
    with pytest.raises(binding.CadmmError, match="out of range"):
        s.build_graph(4, [0], [4], 1)
    with pytest.raises(binding.CadmmError, match="community"):
        s.build_graph(4, [0], [1], 2, np.array([0, 1, 2, 0], np.int32))
    with pytest.raises(binding.CadmmError):
        s.build_graph(4, [0], [1], 0)
    with pytest.raises(binding.CadmmError, match="build_graph"):
        s.workspace_bytes()
    s.build_graph(4, [0], [1], 2)
    hyper = dict(nu=1e-3, rho=1e-3, tau0=1e-3, theta0=1e-3, eta=2.0, max_backtrack=60, fista_iters=10)
    with pytest.raises(binding.CadmmError):
        s.set_model([3, 2], **hyper)                      # one layer only
    with pytest.raises(binding.CadmmError):
        s.set_model([3, 2, 2], **dict(hyper, eta=1.0))
    with pytest.raises(binding.CadmmError):
        s.set_model([3, 2, 2], **dict(hyper, dual_form=2))
    s.set_model([3, 2, 2], **hyper)
    assert s.workspace_bytes() > 0
    with pytest.raises(binding.CadmmError):
        s.run(1)                                          # out of order
    s.close()


def test_workspace_size_is_plausible_for_the_large_configs():
    """Sized from the state alone: Z, H, T, G per layer are N x C fp32."""
    s = host_solver()
    w = synth.config(2, 0.5)
    s.build_graph(w.N, w.src, w.dst, w.M, w.comm)
    h = w.hyper
    s.set_model(w.dims, nu=h["nu"], rho=h["rho"], tau0=h["tau0"], theta0=h["theta0"], eta=h["eta"],
                max_backtrack=h["max_backtrack"], fista_iters=h["fista_iters"])
    state = 4 * w.N * sum(w.dims)
    assert state < s.workspace_bytes() < 12 * state
    s.close()
