"""Pins of the partitioner's CPU twin (oracle/partition.py): brute force on tiny graphs, invariants, planted
partitions.  The paper only names METIS (Section 2), so nothing printed there pins the result."""
import itertools

import numpy as np
import pytest

from oracle.partition import edge_cut, partition, propagation_round, size_cap, takes_part
from paper_2112_09335_amd import synth


def cliques_joined_in_a_ring(k, n_cliques):
    src, dst = [], []
    for c in range(n_cliques):
        base = c * k
        for a, b in itertools.combinations(range(k), 2):
            src.append(base + a)
            dst.append(base + b)
        src.append(base + k - 1)                       # one bridge to the next clique
        dst.append(((c + 1) % n_cliques) * k)
    return np.array(src, np.int32), np.array(dst, np.int32)


def brute_force_min_cut(N, src, dst, M, cap):
    best = None
    for lab in itertools.product(range(M), repeat=N):
        if lab[0] != 0:                                # fix one label: partitions up to renaming
            continue
        sizes = np.bincount(lab, minlength=M)
        if sizes.max() > cap or sizes.min() == 0:
            continue
        cut = edge_cut(src, dst, np.array(lab))
        if best is None or cut < best:
            best = cut
    return best


def test_two_triangles_and_three_squares_reach_the_brute_force_cut():
    src, dst = cliques_joined_in_a_ring(3, 2)          # two triangles, two bridges (0-5 and 2-3)
    comm = partition(6, src, dst, 2)
    assert sorted(np.bincount(comm).tolist()) == [3, 3]
    assert comm[0] == comm[1] == comm[2] and comm[3] == comm[4] == comm[5]
    assert edge_cut(src, dst, comm) == brute_force_min_cut(6, src, dst, 2, size_cap(6, 2)) == 2
    src, dst = cliques_joined_in_a_ring(4, 3)          # three 4-cliques in a ring
    comm = partition(12, src, dst, 3)
    assert edge_cut(src, dst, comm) == brute_force_min_cut(12, src, dst, 3, size_cap(12, 3)) == 3
    for c in range(3):
        assert len(set(comm[4 * c:4 * c + 4].tolist())) == 1


def test_cap_formula_and_participation_rule():
    assert size_cap(2000, 4) == 500 + 25 + 1
    assert size_cap(10, 3) == 4 + 0 + 1
    # about half of the nodes take part in a round, and the set changes with the round
    a = np.array([takes_part(v, 0) for v in range(100000)])
    b = np.array([takes_part(v, 1) for v in range(100000)])
    assert 0.45 < a.mean() < 0.55 and 0.45 < b.mean() < 0.55 and 0.2 < (a != b).mean()
    # the rule itself on a value worked by hand: v = 3, r = 2 -> (3 * 2654435761 + 81006) >> 16 = 121511 (odd)
    assert (3 * 2654435761 + 2 * 40503) >> 16 == 121511 and not takes_part(3, 2)


def test_one_round_by_hand_on_a_path():
    # path 0-1-2-3, unit weights, every node its own label, cap 2.  Whoever takes part asks for the smaller
    # neighbour label (every neighbour label pulls with weight 1, its own label with 0); requests are granted in
    # node order while the target had room at the start of the round (cap - 1 = 1 each).
    nb = [{1: 1}, {0: 1, 2: 1}, {1: 1, 3: 1}, {2: 1}]
    label, size = [0, 1, 2, 3], {0: 1, 1: 1, 2: 1, 3: 1}
    r = 0
    moved = propagation_round(nb, [1, 1, 1, 1], label, size, 2, r)
    expect = [0, 1, 2, 3]
    room = {c: 1 for c in range(4)}
    for v in range(4):
        if takes_part(v, r):
            want = min(nb[v])                          # neighbour labels are the neighbour ids here
            if room[want] > 0:
                room[want] -= 1
                expect[v] = want
    assert label == expect and moved == sum(1 for v in range(4) if expect[v] != v)
    assert sorted(size.items()) == sorted((c, expect.count(c)) for c in range(4))


def test_one_weighted_round_by_hand():
    # star: centre 0 (label 9, weight 1) with four leaves of weights 5, 2, 4, 1 (in node order), each labelled by its own
    # number and pulled towards label 9 only.  cap 8: the room of label 9 is 8 - 1 = 7.  In node order: the first
    # leaf (5) fits -> room 2, the second (2) fits -> room 0, the third (4) and the fourth (1) do not.
    r = 2
    assert not takes_part(0, r)
    leaves = [v for v in range(1, 40) if takes_part(v, r)][:4]
    n = leaves[-1] + 1
    pulls = dict(zip(leaves, (3, 1, 1, 1)))
    nb = [dict() for _ in range(n)]
    for v, w in pulls.items():
        nb[0][v] = w
        nb[v][0] = w
    weight = [1] * n
    for v, w in zip(leaves, (5, 2, 4, 1)):
        weight[v] = w
    label = list(range(n))
    label[0] = 9 + n
    size = {label[v]: weight[v] for v in range(n)}
    assert propagation_round(nb, weight, label, size, 8, r) == 2
    assert [label[v] for v in leaves] == [9 + n, 9 + n, leaves[2], leaves[3]] and size[9 + n] == 8
    assert size[leaves[0]] == 0 and size[leaves[1]] == 0 and size[leaves[2]] == 4 and size[leaves[3]] == 1
    # the centre, when it takes part, follows the heaviest pull, not the most neighbours
    r0 = next(r for r in range(100000) if takes_part(0, r) and not any(takes_part(v, r) for v in leaves))
    a, b = leaves[0], leaves[1]
    def fresh():
        lab = list(range(n))
        lab[0] = 9 + n
        for v in leaves[1:]:
            lab[v] = b                                      # three leaves share label b: pull 1 + 1 + 1 = 3
        return lab, {9 + n: 1, a: 5, b: 7}
    lab, size = fresh()
    assert propagation_round(nb, weight, lab, size, 8, r0) == 1 and lab[0] == a     # 3 against 3: the smaller label, a
    nb[0][b] = 2
    nb[b][0] = 2                                            # now label b pulls with 4, but 1 + 7 fits cap 8 exactly
    lab, size = fresh()
    assert propagation_round(nb, weight, lab, size, 8, r0) == 1 and lab[0] == b and size[b] == 8
    lab, size = fresh()
    assert propagation_round(nb, weight, lab, size, 7, r0) == 0                     # and with cap 7 it does not


@pytest.mark.parametrize("idx,scale,slack", [(1, 1.0, 1.15), (2, 0.25, 1.15), (3, 0.025, 1.02), (4, 0.0025, 1.10)])
def test_planted_communities_are_found_again(idx, scale, slack):
    w = synth.config(idx, scale)
    comm = partition(w.N, w.src, w.dst, w.M)
    assert comm.dtype == np.int32 and comm.shape == (w.N,)
    assert comm.min() >= 0 and comm.max() < w.M
    sizes = np.bincount(comm, minlength=w.M)
    assert sizes.max() <= size_cap(w.N, w.M)
    assert edge_cut(w.src, w.dst, comm) <= slack * edge_cut(w.src, w.dst, w.comm)


def test_noise_in_the_edge_list_isolated_nodes_and_small_M():
    rng = np.random.default_rng(3)
    N = 300
    src = rng.integers(0, N - 20, 900).astype(np.int32)       # the last 20 nodes have no edge at all
    dst = rng.integers(0, N - 20, 900).astype(np.int32)
    base = partition(N, src, dst, 5)
    noisy_src = np.concatenate([src, dst, src[:50], np.arange(10, dtype=np.int32)])
    noisy_dst = np.concatenate([dst, src, dst[:50], np.arange(10, dtype=np.int32)])
    np.testing.assert_array_equal(partition(N, noisy_src, noisy_dst, 5), base)
    assert np.bincount(base, minlength=5).max() <= size_cap(N, 5) and len(np.unique(base)) == 5
    np.testing.assert_array_equal(partition(N, src, dst, 1), np.zeros(N, np.int32))
    none = partition(7, np.zeros(0, np.int32), np.zeros(0, np.int32), 3)       # no edges: smallest clusters merge
    assert sorted(np.bincount(none, minlength=3).tolist()) == [2, 2, 3]
    with pytest.raises(ValueError):
        partition(5, np.array([0, 7]), np.array([1, 2]), 2)
