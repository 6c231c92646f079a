"""The library's partitioner (cadmm_partition, host work) against its CPU twin, bit for bit, and end to end:
a graph partitioned by the library feeds cadmm_build_graph.  No GPU call."""
import numpy as np
import pytest

from oracle import partition as twin
from oracle.graph import OracleGraph
from paper_2112_09335_amd import binding, synth


def both(N, src, dst, M):
    s = binding.Solver(device=-1)
    got = s.partition(N, src, dst, M)
    s.close()
    want = twin.partition(N, src, dst, M)
    assert got.dtype == np.int32 and got.shape == (N,)
    np.testing.assert_array_equal(got, want)
    return got


@pytest.mark.parametrize("idx,scale", [(1, 1.0), (2, 0.25), (3, 0.025), (4, 0.0025), (5, 0.004)])
def test_partition_equals_the_twin_on_the_benchmark_recipes(idx, scale):
    w = synth.config(idx, scale)
    comm = both(w.N, w.src, w.dst, w.M)
    assert np.bincount(comm, minlength=w.M).max() <= twin.size_cap(w.N, w.M)


def test_partition_equals_the_twin_on_awkward_inputs():
    rng = np.random.default_rng(8)
    N = 500
    src = rng.integers(0, N - 30, 1500).astype(np.int32)        # 30 isolated nodes
    dst = rng.integers(0, N - 30, 1500).astype(np.int32)
    for M in (1, 2, 7, 64, 499, 500, 800):                      # also more communities than clusters
        both(N, src, dst, M)
    both(N, np.concatenate([src, dst, src]), np.concatenate([dst, src, src]), 5)     # repeats, both ways, self pairs
    both(9, np.zeros(0, np.int32), np.zeros(0, np.int32), 4)    # no edges
    both(1, np.zeros(0, np.int32), np.zeros(0, np.int32), 1)
    # a hub: one node adjacent to everything
    both(400, np.zeros(399, np.int32), np.arange(1, 400, dtype=np.int32), 4)


def test_bad_arguments():
    s = binding.Solver(device=-1)
    with pytest.raises(binding.CadmmError):
        s.partition(5, np.array([0, 9], np.int32), np.array([1, 2], np.int32), 2)
    with pytest.raises(binding.CadmmError):
        s.partition(5, np.array([0], np.int32), np.array([1], np.int32), 0)
    s.close()


def test_partition_feeds_build_graph():
    w = synth.config(2, 0.1)
    s = binding.Solver(device=-1)
    comm = s.partition(w.N, w.src, w.dst, w.M)
    s.build_graph(w.N, w.src, w.dst, w.M, comm)
    g = s.get_graph()
    o = OracleGraph(w.N, w.src, w.dst, w.M, comm)
    assert np.array_equal(g["perm"], o.perm) and np.array_equal(g["col"], o.col)
    # far fewer (row, community) segments than with a partition that ignores the graph
    _, nseg, _ = s.graph_sizes()
    s2 = binding.Solver(device=-1)
    s2.build_graph(w.N, w.src, w.dst, w.M, None)                # contiguous chunks of the scrambled ids
    assert nseg - w.N < 0.25 * (s2.graph_sizes()[1] - w.N)      # segments beyond a row's own community
    assert twin.edge_cut(w.src, w.dst, comm) <= 1.15 * twin.edge_cut(w.src, w.dst, w.comm)
    s.close()
    s2.close()
