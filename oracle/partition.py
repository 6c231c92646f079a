"""CPU oracle, part 3: the built-in community partitioner.  TEST INFRASTRUCTURE ONLY.

The paper cuts the graph into M communities with METIS (Section 2, the paragraph that introduces the
communities V_m) and says nothing more about it; METIS is a third-party heuristic that is not part of this
build.  The library instead ships a small deterministic partitioner of its own, and this file is its slow
twin: the definition written out step by step in plain Python, every tie-break stated, so that the two can
be compared bit for bit.  Nothing in the paper pins the result ("parity unpinned" by the paper); the tests
hold it by its invariants, by brute force on tiny graphs, by a hand-worked round and by planted partitions it
has to recover.

Definition (all integer work):
  graph     simple undirected graph of the edge list: self pairs dropped, repeated pairs counted once.
            Every node has weight 1 and every edge weight 1 on the finest level.
  cap       ceil(N / M) + floor(floor(N / M) / 20) + 1     (about 5 % slack on a community's size)
  round r   synchronous label propagation under the size cap, on a graph with node and edge weights.
            Node v takes part in round r if ((v * 2654435761 + r * 40503) mod 2^64) >> 16 is even (half of
            the nodes, so that two neighbours do not swap labels for ever).  It adds up the edge weights
            towards every label among its neighbours, picks the heaviest label (ties: the smallest label)
            and asks to move there if that weight exceeds the weight towards its own label.  Requests are
            looked at in increasing v: a request is granted if the node's weight fits into the room of its
            target, room = cap - (weight of the target at the start of the round) minus what was granted
            before; all granted moves happen at once.
  level     every node starts with a label of its own (its number); rounds r = 0, 1, .. until two rounds in
            a row moved nothing, at most 100.  Then the graph is contracted: the clusters, numbered in
            increasing order of their label, are the nodes of the next level (weight = sum of the members'
            weights; edge weight = sum of the edge weights between two clusters).
  levels    repeat while a level has more than M nodes and the last one shrank the graph by at least 5 %
            (20 K <= 19 n for n nodes contracted to K).
  merge     on the last graph: while it has more than M nodes, merge the pair (a < b) joined by the heaviest
            edge among the pairs whose weights add up to at most cap (ties: smallest a, then smallest b);
            b disappears into a.  Stop if no pair qualifies; then, while there are still more than M, merge
            the two lightest nodes (ties: smaller number), the larger number into the smaller, whatever
            the cap.
  result    the nodes that are left become communities 0, 1, .. in increasing order of their number; every
            original node gets the community of the chain of clusters it went into; then the propagation
            runs on the finest graph again, rounds r = 0, 1, .. until two rounds in a row moved nothing, at
            most 100, which moves the borders where the coarse levels left them in the wrong place.
Fewer than M communities may remain; the ones after the last are then empty.
"""
from __future__ import annotations

import numpy as np

MAX_ROUNDS = 100
MASK64 = (1 << 64) - 1


def size_cap(N: int, M: int) -> int:
    return -(-N // M) + (N // M) // 20 + 1


def takes_part(v: int, r: int) -> bool:
    return ((((v * 2654435761 + r * 40503) & MASK64) >> 16) & 1) == 0


def neighbour_lists(N, src, dst):
    """nb[v] = {u: edge weight} of the simple graph."""
    nb = [dict() for _ in range(N)]
    for a, b in zip(np.asarray(src).tolist(), np.asarray(dst).tolist()):
        if not (0 <= a < N and 0 <= b < N):
            raise ValueError("edge endpoint out of range")
        if a != b:
            nb[a][b] = 1
            nb[b][a] = 1
    return nb


def propagation_round(nb, weight, label, size, cap, r):
    """One synchronous round; label (list) and size (dict label -> weight) are updated in place.
    Returns the number of moves."""
    requests = []
    for v in range(len(nb)):
        if not takes_part(v, r) or not nb[v]:
            continue
        pull = {}
        for u, w in nb[v].items():
            pull[label[u]] = pull.get(label[u], 0) + w
        best = min(pull, key=lambda c: (-pull[c], c))
        if pull[best] > pull.get(label[v], 0):
            requests.append((v, best))
    room = {}
    moves = []
    for v, c in requests:                       # increasing v by construction
        if c not in room:
            room[c] = cap - size.get(c, 0)
        if weight[v] <= room[c]:
            room[c] -= weight[v]
            moves.append((v, c))
    for v, c in moves:
        size[label[v]] -= weight[v]
        size[c] = size.get(c, 0) + weight[v]
        label[v] = c
    return len(moves)


def one_level(nb, weight, cap):
    """Labels after the propagation has come to rest (or MAX_ROUNDS)."""
    n = len(nb)
    label = list(range(n))
    size = {v: weight[v] for v in range(n)}
    quiet = 0
    for r in range(MAX_ROUNDS):
        quiet = quiet + 1 if propagation_round(nb, weight, label, size, cap, r) == 0 else 0
        if quiet == 2:
            break
    return label


def contract(nb, weight, label):
    names = sorted(set(label))
    number = {c: i for i, c in enumerate(names)}
    member_of = [number[c] for c in label]
    K = len(names)
    cweight = [0] * K
    cnb = [dict() for _ in range(K)]
    for v in range(len(nb)):
        a = member_of[v]
        cweight[a] += weight[v]
        for u, w in nb[v].items():
            b = member_of[u]
            if a != b:
                cnb[a][b] = cnb[a].get(b, 0) + w
    return cnb, cweight, member_of


def merge_down_to(nb, weight, M, cap):
    """Community of every node of the last graph."""
    K = len(nb)
    nb = [dict(d) for d in nb]
    weight = list(weight)
    alive = [True] * K
    into = list(range(K))
    n_alive = K

    def absorb(a, b):
        nonlocal n_alive
        weight[a] += weight[b]
        weight[b] = 0
        alive[b] = False
        into[b] = a
        n_alive -= 1

    while n_alive > M:
        best = None
        for a in range(K):
            for b, w in nb[a].items():
                if a < b and weight[a] + weight[b] <= cap and (best is None or (-w, a, b) < best[0]):
                    best = ((-w, a, b), a, b)
        if best is None:
            break
        _, a, b = best
        for x, w in nb[b].items():
            if x == a:
                continue
            nb[a][x] = nb[a].get(x, 0) + w
            del nb[x][b]
            nb[x][a] = nb[a][x]
        del nb[a][b]
        nb[b] = {}
        absorb(a, b)
    while n_alive > M:
        order = sorted((weight[c], c) for c in range(K) if alive[c])
        a, b = sorted((order[0][1], order[1][1]))
        absorb(a, b)

    def root(c):
        while into[c] != c:
            c = into[c]
        return c
    community = {c: i for i, c in enumerate(c for c in range(K) if alive[c])}
    return [community[root(c)] for c in range(K)]


def partition(N, src, dst, M):
    """Community of every node, int32 [N], values in [0, M)."""
    N, M = int(N), int(M)
    if N < 1 or M < 1:
        raise ValueError("N and M must be positive")
    finest = neighbour_lists(N, src, dst)
    cap = size_cap(N, M)
    nb, weight = finest, [1] * N
    chain = []                                   # chain[i][v] = node of level i+1 that node v of level i went into
    while len(nb) > M:
        n = len(nb)
        label = one_level(nb, weight, cap)
        nb, weight, member_of = contract(nb, weight, label)
        chain.append(member_of)
        if 20 * len(nb) > 19 * n:
            break
    top = merge_down_to(nb, weight, M, cap)
    label = []
    for v in range(N):
        c = v
        for member_of in chain:
            c = member_of[c]
        label.append(top[c])
    size = {}
    for c in label:
        size[c] = size.get(c, 0) + 1
    unit = [1] * N
    quiet = 0
    for r in range(MAX_ROUNDS):
        quiet = quiet + 1 if propagation_round(finest, unit, label, size, cap, r) == 0 else 0
        if quiet == 2:
            break
    return np.asarray(label, dtype=np.int32)


def edge_cut(src, dst, comm):
    comm = np.asarray(comm)
    return int(np.count_nonzero(comm[np.asarray(src)] != comm[np.asarray(dst)]))
