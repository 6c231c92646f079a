"""Seeded synthetic workloads: stochastic-block-model graphs, features, labels, initial weights.

This module only draws random inputs.  It holds none of the method's arithmetic
(no adjacency normalisation, no aggregation, no ADMM step) and imports neither the
HIP binding nor the CPU oracle; both consume the arrays it returns.

The graphs stand in for the node-classification workloads of the paper's
experiments (Section 4, Table 2: co-purchase graphs with a few thousand nodes,
hundreds of features, about ten classes), which are not available offline.
Every array comes from one ``numpy.random.Generator(PCG64(seed))`` in a fixed
draw order, so a (recipe, seed) pair always yields the same bytes.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np


@dataclass
class Workload:
    """One problem instance in the caller's (scrambled) node order."""

    name: str
    N: int
    M: int
    src: np.ndarray            # int32 [E]  undirected edges, one orientation, no self pairs, no duplicates
    dst: np.ndarray            # int32 [E]
    comm: np.ndarray           # int32 [N]  community of every node
    X: np.ndarray              # float32 [N, C0]
    labels: np.ndarray         # int32 [N]  class id, -1 = unlabelled
    dims: List[int]            # C_0 .. C_L
    W0: List[np.ndarray]       # float32 [C_{l-1}, C_l], l = 1..L
    iters: int
    hyper: Dict[str, float] = field(default_factory=dict)

    @property
    def L(self) -> int:
        return len(self.dims) - 1

    @property
    def E(self) -> int:
        return int(self.src.shape[0])


DEFAULT_HYPER = dict(nu=1e-3, rho=1e-3, tau0=1e-3, theta0=1e-3, eta=2.0,
                     max_backtrack=60, fista_iters=10, risk=0, dual_form=0, schedule=0,
                     step_policy=0, fista_mode=0)


def _dedup_pairs(a: np.ndarray, b: np.ndarray, N: int):
    """Drop self pairs and repeated unordered pairs; keep first-seen orientation lo<hi."""
    keep = a != b
    a, b = a[keep], b[keep]
    lo = np.minimum(a, b).astype(np.int64)
    hi = np.maximum(a, b).astype(np.int64)
    key = np.unique(lo * N + hi)
    return (key // N).astype(np.int32), (key % N).astype(np.int32)


def _equal_blocks(N: int, M: int) -> np.ndarray:
    """Community of node i in generator order: contiguous blocks, sizes differ by at most one."""
    bounds = (np.arange(M + 1, dtype=np.int64) * N) // M
    comm = np.empty(N, dtype=np.int32)
    for c in range(M):
        comm[bounds[c]:bounds[c + 1]] = c
    return comm


def sbm_bernoulli(rng, N, M, p_in, p_out):
    """Exact Bernoulli SBM over all unordered pairs (small N only)."""
    comm = _equal_blocks(N, M)
    iu, ju = np.triu_indices(N, k=1)
    same = comm[iu] == comm[ju]
    p = np.where(same, p_in, p_out)
    hit = rng.random(iu.shape[0]) < p
    return iu[hit].astype(np.int32), ju[hit].astype(np.int32), comm


def sbm_expected_degree(rng, N, M, avg_degree, frac_intra, weights: Optional[np.ndarray] = None):
    """Fixed-expected-degree SBM.

    round(frac_intra * E) endpoint pairs are drawn inside a community (community chosen
    in proportion to its size), the rest between two distinct communities.  With
    ``weights`` the endpoints are drawn in proportion to the node weights inside the
    chosen community (degree-corrected SBM); otherwise uniformly.
    """
    comm = _equal_blocks(N, M)
    bounds = (np.arange(M + 1, dtype=np.int64) * N) // M
    sizes = np.diff(bounds)
    E = int(round(N * avg_degree / 2.0))
    E_in = int(round(frac_intra * E))
    E_out = E - E_in if M > 1 else 0
    if M == 1:
        E_in = E

    if weights is None:
        cum = None
    else:
        cum = np.concatenate([[0.0], np.cumsum(weights.astype(np.float64))])

    def draw_nodes(c: np.ndarray) -> np.ndarray:
        """One node inside community c[k] for every k."""
        if cum is None:
            return bounds[c] + (rng.random(c.shape[0]) * sizes[c]).astype(np.int64)
        lo_w, hi_w = cum[bounds[c]], cum[bounds[c + 1]]
        t = lo_w + rng.random(c.shape[0]) * (hi_w - lo_w)
        idx = np.searchsorted(cum, t, side="right") - 1
        return np.clip(idx, bounds[c], bounds[c + 1] - 1)

    c_in = rng.choice(M, size=E_in, p=sizes / sizes.sum())
    a_in, b_in = draw_nodes(c_in), draw_nodes(c_in)
    if E_out > 0:
        c1 = rng.choice(M, size=E_out, p=sizes / sizes.sum())
        shift = 1 + (rng.random(E_out) * (M - 1)).astype(np.int64)
        c2 = (c1 + shift) % M
        a_out, b_out = draw_nodes(c1), draw_nodes(c2)
        a = np.concatenate([a_in, a_out])
        b = np.concatenate([b_in, b_out])
    else:
        a, b = a_in, b_in
    src, dst = _dedup_pairs(a, b, N)
    return src, dst, comm


def powerlaw_weights(rng, N, avg_degree, exponent):
    """Node weights u^(-1/(exponent-1)), u ~ U(0,1], capped at sqrt(N * avg_degree)."""
    u = 1.0 - rng.random(N)
    w = u ** (-1.0 / (exponent - 1.0))
    return np.minimum(w, np.sqrt(N * avg_degree))


def draw_labels(rng, comm, n_classes, purity=0.8, labelled_fraction=1.0):
    """Community c has home class c mod n_classes; a node keeps it with probability purity."""
    N = comm.shape[0]
    home = (comm % n_classes).astype(np.int32)
    keep = rng.random(N) < purity
    other = (home + 1 + (rng.random(N) * (n_classes - 1)).astype(np.int32)) % n_classes
    labels = np.where(keep, home, other).astype(np.int32)
    if labelled_fraction < 1.0:
        labels = np.where(rng.random(N) < labelled_fraction, labels, -1).astype(np.int32)
    return labels


def xavier_uniform(rng, dims):
    out = []
    for l in range(1, len(dims)):
        a = np.sqrt(6.0 / (dims[l - 1] + dims[l]))
        out.append(((rng.random((dims[l - 1], dims[l])) * 2.0 - 1.0) * a).astype(np.float32))
    return out


def _scramble(rng, src, dst, comm):
    """Relabel nodes at random so that communities are not contiguous in the caller's order."""
    N = comm.shape[0]
    new_of_old = rng.permutation(N).astype(np.int32)
    comm2 = np.empty_like(comm)
    comm2[new_of_old] = comm
    return new_of_old[src], new_of_old[dst], comm2


def make_workload(name, seed, N, M, dims, n_classes, iters, *, graph, features,
                  avg_degree=None, frac_intra=None, p_in=None, p_out=None, exponent=None,
                  labelled_fraction=1.0, scramble=True, hyper=None) -> Workload:
    rng = np.random.Generator(np.random.PCG64(seed))
    if graph == "bernoulli":
        src, dst, comm = sbm_bernoulli(rng, N, M, p_in, p_out)
    elif graph == "sbm":
        src, dst, comm = sbm_expected_degree(rng, N, M, avg_degree, frac_intra)
    elif graph == "dcsbm":
        w = powerlaw_weights(rng, N, avg_degree, exponent)
        src, dst, comm = sbm_expected_degree(rng, N, M, avg_degree, frac_intra, weights=w)
    elif graph == "empty":
        src = np.zeros(0, np.int32)
        dst = np.zeros(0, np.int32)
        comm = _equal_blocks(N, M)
    else:
        raise ValueError(graph)
    if scramble:
        src, dst, comm = _scramble(rng, src, dst, comm)
    src = np.ascontiguousarray(src, dtype=np.int32)
    dst = np.ascontiguousarray(dst, dtype=np.int32)
    if features == "bernoulli":
        X = (rng.random((N, dims[0]), dtype=np.float32) < 0.01).astype(np.float32)
    elif features == "gaussian":
        X = rng.standard_normal((N, dims[0]), dtype=np.float32)
    else:
        raise ValueError(features)
    labels = draw_labels(rng, comm, n_classes, labelled_fraction=labelled_fraction)
    assert dims[-1] == n_classes
    W0 = xavier_uniform(rng, dims)
    h = dict(DEFAULT_HYPER)
    if hyper:
        h.update(hyper)
    return Workload(name, N, M, src, dst, comm, X, labels, list(dims), W0, iters, h)


def add_hubs(w: Workload, seed: int, hubs: int, degree: int, concentrate: float = 0.0) -> Workload:
    """Give `hubs` nodes about `degree` extra neighbours each, as the heaviest nodes of a power-law graph have at full
    size (config 4: up to 3 * 10^4) and a scaled-down sample of the recipe does not.  A share `concentrate` of a hub's
    new neighbours is drawn inside ONE other community, so that this (row, community) segment is long too; the rest
    uniformly over all nodes.  Returns a new workload; features, labels and weights are kept."""
    rng = np.random.Generator(np.random.PCG64(seed))
    N = w.N
    hub_ids = rng.choice(N, size=hubs, replace=False)
    a, b = [w.src.astype(np.int64)], [w.dst.astype(np.int64)]
    for h in hub_ids:
        n_one = int(round(concentrate * degree))
        others = np.flatnonzero(w.comm != w.comm[h])
        target = w.comm[others[rng.integers(others.shape[0])]] if others.shape[0] else w.comm[h]
        pool = np.flatnonzero(w.comm == target)
        picks = [rng.choice(pool, size=min(n_one, pool.shape[0]), replace=False)] if n_one else []
        picks.append(rng.choice(N, size=degree - n_one, replace=False))
        nb = np.concatenate(picks)
        a.append(np.full(nb.shape[0], h, np.int64))
        b.append(nb.astype(np.int64))
    src, dst = _dedup_pairs(np.concatenate(a), np.concatenate(b), N)
    return Workload(w.name + "+hubs", N, w.M, np.ascontiguousarray(src), np.ascontiguousarray(dst), w.comm, w.X,
                    w.labels, list(w.dims), w.W0, w.iters, dict(w.hyper))


# The five benchmark configurations (index = seed), and two more for the serial-versus-community comparison.  `scale` shrinks N (and keeps degree,
# community count, widths) for CPU-sized samples of the same recipe.
def config(index: int, scale: float = 1.0, M: Optional[int] = None) -> Workload:
    def n(v):
        return max(int(round(v * scale)), 8)
    if index == 1:
        return make_workload("tiny_sbm", 1, n(2000), M or 4, [256, 64, 7], 7, 10, graph="bernoulli",
                             features="bernoulli", p_in=0.02 / scale if scale < 1 else 0.02,
                             p_out=0.001 / scale if scale < 1 else 0.001)
    if index == 2:
        return make_workload("mid_sbm", 2, n(20000), M or 8, [500, 128, 3], 3, 50, graph="sbm",
                             features="gaussian", avg_degree=10, frac_intra=0.90)
    if index == 3:
        return make_workload("large_sbm", 3, n(200000), M or 32, [128, 256, 256, 10], 10, 20, graph="sbm",
                             features="gaussian", avg_degree=15, frac_intra=0.85)
    if index == 4:
        return make_workload("powerlaw_dcsbm", 4, n(2000000), M or 64, [128, 256, 16], 16, 10, graph="dcsbm",
                             features="gaussian", avg_degree=25, frac_intra=0.80, exponent=2.5)
    if index == 5:
        return make_workload("deep_wide_sbm", 5, n(500000), M or 16, [512] * 8 + [10], 10, 10, graph="sbm",
                             features="gaussian", avg_degree=12, frac_intra=0.85)
    # Shapes of the two graphs of the paper's speed-up experiment (Section 4.1, Tables 2 and 3: node, feature and
    # class counts as printed; two layers with 1000 hidden units; 3 communities).  The paper prints no edge counts:
    # the average degree is an assumption of this recipe, and the graphs are SBM stand-ins, not the datasets.
    if index == 6:
        return make_workload("computers_shape_sbm", 6, n(13752), M or 3, [767, 1000, 10], 10, 50, graph="sbm",
                             features="bernoulli", avg_degree=36, frac_intra=0.90)
    if index == 7:
        return make_workload("photo_shape_sbm", 7, n(7650), M or 3, [745, 1000, 8], 8, 50, graph="sbm",
                             features="bernoulli", avg_degree=31, frac_intra=0.90,
                             hyper=dict(nu=1e-4, rho=1e-4))
    raise ValueError("config index must be 1..7")
