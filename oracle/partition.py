"""CPU oracle, part 3: the built-in community partitioner.  TEST INFRASTRUCTURE ONLY.

The paper cuts the graph into M communities with METIS (Section 2, the paragraph that introduces the
communities V_m) and says nothing more about it; METIS is a third-party heuristic that is not part of this
build.  The library instead ships a small deterministic partitioner of its own, and this file is its slow
twin: the definition written out step by step in plain Python, every tie-break stated, so that the two can
be compared bit for bit.  Nothing in the paper pins the result ("parity unpinned" by the paper); the tests
hold it by its invariants, by a hand-worked example and by planted partitions it has to recover.

Definition (all integer work):
  graph     simple undirected graph of the edge list: self pairs dropped, repeated pairs counted once.
  cap       ceil(N / M) + floor(floor(N / M) / 20) + 1     (about 5 % slack on a community's size)
  round r   synchronous label propagation under the size cap.  Node v takes part in round r if
            ((v * 2654435761 + r * 40503) mod 2^64) >> 16 is even  (half of the nodes, so that two
            neighbours do not swap labels for ever).  It counts the labels of its neighbours, picks the most
            frequent one (ties: the smallest label) and asks to move there if that count exceeds the count
            of its own label.  Requests are granted in increasing v while the target has room, where
            room = cap - (size of the target at the start of the round); all granted moves happen at once.
  phase 1   every node starts in a cluster of its own (label = node id); rounds r = 0 .. 11.
  phase 2   clusters are numbered in increasing order of their label.  While there are more than M of them,
            merge the pair (a < b) joined by the most edges among the pairs whose sizes add up to at most
            cap (ties: smallest a, then smallest b); b disappears into a.  Stop if no pair qualifies.
  phase 3   while there are still more than M clusters, merge the two smallest (ties: smaller number), the
            one with the larger number into the other, whatever the cap.
  phase 4   the clusters that are left become communities 0, 1, .. in increasing order of their number.
  phase 5   four more rounds r = 12 .. 15 of the same propagation, now on community labels.
Fewer than M clusters may remain; the communities after the last one are then empty.
"""
from __future__ import annotations

import numpy as np

ROUNDS_GROW = 12
ROUNDS_REFINE = 4
MASK64 = (1 << 64) - 1


def size_cap(N: int, M: int) -> int:
    return -(-N // M) + (N // M) // 20 + 1


def takes_part(v: int, r: int) -> bool:
    return ((((v * 2654435761 + r * 40503) & MASK64) >> 16) & 1) == 0


def neighbour_lists(N, src, dst):
    nb = [set() for _ in range(N)]
    for a, b in zip(np.asarray(src).tolist(), np.asarray(dst).tolist()):
        if not (0 <= a < N and 0 <= b < N):
            raise ValueError("edge endpoint out of range")
        if a != b:
            nb[a].add(b)
            nb[b].add(a)
    return [sorted(s) for s in nb]


def propagation_round(nb, label, size, cap, r):
    """One synchronous round; label and size are updated in place.  Returns the number of moves."""
    N = len(nb)
    requests = []
    for v in range(N):
        if not takes_part(v, r) or not nb[v]:
            continue
        count = {}
        for u in nb[v]:
            count[label[u]] = count.get(label[u], 0) + 1
        best = min(count, key=lambda c: (-count[c], c))
        if count[best] > count.get(label[v], 0):
            requests.append((v, best))
    room = {}
    moves = []
    for v, c in requests:                       # increasing v by construction
        if c not in room:
            room[c] = cap - size.get(c, 0)
        if room[c] > 0:
            room[c] -= 1
            moves.append((v, c))
    for v, c in moves:
        size[label[v]] -= 1
        size[c] = size.get(c, 0) + 1
        label[v] = c
    return len(moves)


def partition(N, src, dst, M):
    """Community of every node, int32 [N], values in [0, M)."""
    N, M = int(N), int(M)
    if N < 1 or M < 1:
        raise ValueError("N and M must be positive")
    nb = neighbour_lists(N, src, dst)
    cap = size_cap(N, M)
    # phase 1
    label = list(range(N))
    size = {v: 1 for v in range(N)}
    for r in range(ROUNDS_GROW):
        propagation_round(nb, label, size, cap, r)
    # phase 2: cluster graph
    names = sorted(set(label))
    number = {c: i for i, c in enumerate(names)}
    cl = [number[c] for c in label]
    K = len(names)
    csize = [0] * K
    for c in cl:
        csize[c] += 1
    weight = {}
    for v in range(N):
        for u in nb[v]:
            if v < u and cl[v] != cl[u]:
                key = (min(cl[v], cl[u]), max(cl[v], cl[u]))
                weight[key] = weight.get(key, 0) + 1
    alive = [True] * K
    into = list(range(K))
    n_alive = K
    while n_alive > M:
        best = None
        for (a, b), w in weight.items():
            if csize[a] + csize[b] <= cap and (best is None or (-w, a, b) < (-weight[best], best[0], best[1])):
                best = (a, b)
        if best is None:
            break
        a, b = best
        merged = {}
        for (x, y), w in weight.items():
            if (x, y) == (a, b):
                continue
            x2 = a if x == b else x
            y2 = a if y == b else y
            key = (min(x2, y2), max(x2, y2))
            merged[key] = merged.get(key, 0) + w
        weight = merged
        csize[a] += csize[b]
        csize[b] = 0
        alive[b] = False
        into[b] = a
        n_alive -= 1
    # phase 3
    while n_alive > M:
        order = sorted((csize[c], c) for c in range(K) if alive[c])
        a, b = sorted((order[0][1], order[1][1]))
        csize[a] += csize[b]
        csize[b] = 0
        alive[b] = False
        into[b] = a
        n_alive -= 1
    # phase 4
    def root(c):
        while into[c] != c:
            c = into[c]
        return c
    survivors = [c for c in range(K) if alive[c]]
    community = {c: i for i, c in enumerate(survivors)}
    label = [community[root(c)] for c in cl]
    # phase 5
    size = {}
    for c in label:
        size[c] = size.get(c, 0) + 1
    for r in range(ROUNDS_GROW, ROUNDS_GROW + ROUNDS_REFINE):
        propagation_round(nb, label, size, cap, r)
    return np.asarray(label, dtype=np.int32)


def edge_cut(src, dst, comm):
    comm = np.asarray(comm)
    return int(np.count_nonzero(comm[np.asarray(src)] != comm[np.asarray(dst)]))
