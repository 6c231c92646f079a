"""Pins for the oracle's graph part: closed forms, invariants and brute force on tiny graphs.

Everything here is checked against what the mathematics fixes (paper, Section 2:
A~ = (D+I)^(-1/2)(A+I)(D+I)^(-1/2), the sets N_m, the blocks A~_{m,r}), never against
the oracle itself.
"""
import itertools
import os

import numpy as np
import pytest

from oracle.graph import OracleGraph

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def dense_norm_adj(N, edges):
    """Brute force from the definition with dense matrices, in the caller's node order."""
    A = np.zeros((N, N))
    for u, v in edges:
        if u != v:
            A[u, v] = A[v, u] = 1.0
    d = A.sum(axis=1) + 1.0
    return (A + np.eye(N)) / np.sqrt(np.outer(d, d)), A


def dense_of(g):
    """Oracle A~ as a dense matrix in the caller's node order."""
    Ad = g.A.toarray()
    out = np.zeros_like(Ad)
    out[np.ix_(g.perm, g.perm)] = Ad
    return out


def random_graph(rng, N, M, p=0.15, scrambled=True):
    edges = [(u, v) for u, v in itertools.combinations(range(N), 2) if rng.random() < p]
    # add noise the builder must normalise away: reversed copies, repeats, self pairs
    noisy = edges + [(v, u) for u, v in edges[::3]] + edges[::5] + [(i, i) for i in range(0, N, 4)]
    order = rng.permutation(len(noisy))
    noisy = [noisy[i] for i in order]
    comm = rng.integers(0, M, size=N) if scrambled else np.sort(rng.integers(0, M, size=N))
    return edges, noisy, comm.astype(np.int32)


def test_empty_graph_gives_identity():
    g = OracleGraph(5, [], [], 2, [0, 1, 0, 1, 1])
    assert np.array_equal(dense_of(g), np.eye(5))
    assert g.nnz == 5 and g.n_segments == 5 and g.n_halo_rows == 0
    assert not g.neighbour.any()


def test_complete_graph_gives_uniform_matrix():
    n = 7
    e = list(itertools.combinations(range(n), 2))
    g = OracleGraph(n, [a for a, _ in e], [b for _, b in e], 3, [0, 0, 1, 1, 2, 2, 2])
    np.testing.assert_allclose(dense_of(g), np.full((n, n), 1.0 / n), rtol=0, atol=1e-16)
    X = np.arange(n * 2, dtype=np.float64).reshape(n, 2)
    agg = np.vstack([g.aggregate_block(m, g.to_new(X)) for m in range(3)])
    np.testing.assert_allclose(agg, np.tile(X.mean(axis=0), (n, 1)), rtol=1e-14)


def test_path3_matches_closed_form_fixture():
    want = np.loadtxt(os.path.join(GOLDEN, "path3_normalised_adjacency.txt"))
    g = OracleGraph(3, [0, 2], [1, 1], 1, None)
    np.testing.assert_allclose(dense_of(g), want, rtol=0, atol=1e-16)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_matches_dense_brute_force_and_invariants(seed):
    rng = np.random.default_rng(seed)
    N, M = 40, 4
    edges, noisy, comm = random_graph(rng, N, M)
    g = OracleGraph(N, [a for a, _ in noisy], [b for _, b in noisy], M, comm)
    want, A = dense_norm_adj(N, edges)
    got = dense_of(g)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-15)
    assert g.E == len(edges)
    assert g.nnz == 2 * len(edges) + N
    assert np.array_equal(got, got.T)                                   # symmetric
    d = A.sum(axis=1) + 1.0
    np.testing.assert_allclose(got @ np.sqrt(d), np.sqrt(d), rtol=1e-13)  # eigenvector sqrt(d~), eigenvalue 1
    assert np.max(np.abs(np.linalg.eigvalsh(got))) <= 1.0 + 1e-12       # spectral radius <= 1


@pytest.mark.parametrize("seed", [3, 4])
def test_permutation_csr_segments_and_neighbour_sets_brute_force(seed):
    rng = np.random.default_rng(seed)
    N, M = 48, 5
    edges, noisy, comm = random_graph(rng, N, M, p=0.08)
    g = OracleGraph(N, [a for a, _ in noisy], [b for _, b in noisy], M, comm)
    # permutation: nodes ordered by (community, original id)
    want_perm = sorted(range(N), key=lambda i: (comm[i], i))
    assert list(g.perm) == want_perm
    assert list(g.comm_row_ptr) == [sum(1 for c in comm if c < m) for m in range(M + 1)]
    new_of_old = {o: n for n, o in enumerate(want_perm)}
    adj = [set([i]) for i in range(N)]
    for u, v in edges:
        adj[new_of_old[u]].add(new_of_old[v])
        adj[new_of_old[v]].add(new_of_old[u])
    comm_new = [comm[o] for o in want_perm]
    # CSR: sorted columns per row
    for i in range(N):
        assert list(g.col[g.row_ptr[i]:g.row_ptr[i + 1]]) == sorted(adj[i])
    # N_m from the definition
    for m in range(M):
        want_nb = {comm[v] for u, v in edges if comm[u] == m} | {comm[u] for u, v in edges if comm[v] == m}
        want_nb.discard(m)
        assert set(g.nbrs(m)) == {int(x) for x in want_nb}
    # segments: one per (row, community present among the row's columns), in row-major order
    want_seg = []
    for i in range(N):
        for c in sorted({comm_new[j] for j in adj[i]}):
            cols = [j for j in sorted(adj[i]) if comm_new[j] == c]
            want_seg.append((i, c, cols))
    assert g.n_segments == len(want_seg)
    for s, (i, c, cols) in enumerate(want_seg):
        assert g.seg_row[s] == i and g.seg_comm[s] == c
        assert list(g.col[g.seg_ptr[s]:g.seg_ptr[s + 1]]) == cols
    assert g.n_halo_rows == sum(1 for i in range(N) if any(comm_new[j] != comm_new[i] for j in adj[i]))


@pytest.mark.parametrize("seed", [5, 6])
def test_blocked_aggregation_with_halo_equals_full_graph_bit_exact(seed):
    """Small-integer features and the unnormalised A+I make every sum exact in floating point, so
    the community-blocked sum (halo blocks kept) must equal the dense product bit for bit."""
    rng = np.random.default_rng(seed)
    N, M = 60, 4
    edges, noisy, comm = random_graph(rng, N, M, p=0.1)
    g = OracleGraph(N, [a for a, _ in noisy], [b for _, b in noisy], M, comm)
    X = rng.integers(-8, 9, size=(N, 5)).astype(np.float64)
    blocks = g.split_blocks(g.A_plus_I)
    got = g.to_old(np.vstack([g.aggregate_block(m, g.to_new(X), blocks) for m in range(M)]))
    _, A = dense_norm_adj(N, edges)
    want = (A + np.eye(N)) @ X
    assert np.array_equal(got, want)
    # and with the real A~: equal to rounding
    got = g.to_old(np.vstack([g.aggregate_block(m, g.to_new(X)) for m in range(M)]))
    np.testing.assert_allclose(got, dense_norm_adj(N, edges)[0] @ X, rtol=0, atol=1e-13)


def test_dropping_halo_blocks_would_change_the_result():
    """The inter-community blocks matter: a planted mistake (intra blocks only) fails the identity."""
    rng = np.random.default_rng(7)
    N, M = 30, 3
    edges, noisy, comm = random_graph(rng, N, M, p=0.2)
    g = OracleGraph(N, [a for a, _ in noisy], [b for _, b in noisy], M, comm)
    X = rng.standard_normal((N, 3))
    intra_only = g.to_old(np.vstack([g.block[(m, m)] @ g.to_new(X)[g.rows(m)] for m in range(M)]))
    assert np.max(np.abs(intra_only - dense_norm_adj(N, edges)[0] @ X)) > 1e-3


def test_relabelling_nodes_and_communities_is_a_permutation_of_the_result():
    rng = np.random.default_rng(8)
    N, M = 36, 4
    edges, _, comm = random_graph(rng, N, M, p=0.12)
    g1 = OracleGraph(N, [a for a, _ in edges], [b for _, b in edges], M, comm)
    node_map = rng.permutation(N)
    comm_map = rng.permutation(M)
    comm2 = np.empty(N, dtype=np.int32)
    comm2[node_map] = comm_map[comm]
    g2 = OracleGraph(N, [node_map[a] for a, _ in edges], [node_map[b] for _, b in edges], M, comm2)
    D1, D2 = dense_of(g1), dense_of(g2)
    assert np.array_equal(D2[np.ix_(node_map, node_map)], D1)
    assert g1.n_segments == g2.n_segments and g1.n_halo_rows == g2.n_halo_rows
    for m in range(M):
        assert {int(comm_map[q]) for q in g1.nbrs(m)} == set(g2.nbrs(int(comm_map[m])))


def test_default_partition_and_input_errors():
    g = OracleGraph(10, [0], [9], 3, None)          # chunks of ceil(10/3) = 4
    assert list(g.comm_row_ptr) == [0, 4, 8, 10]
    with pytest.raises(ValueError):
        OracleGraph(4, [0], [4], 1, None)
    with pytest.raises(ValueError):
        OracleGraph(4, [0], [1], 2, [0, 1, 2, 0])
    with pytest.raises(ValueError):
        OracleGraph(4, [0], [1], 0, None)
