"""CPU oracle, part 1: graph, normalised adjacency, community blocks.  TEST INFRASTRUCTURE ONLY.

Plain numpy / scipy.sparse in fp64, written from the paper's Section 2 (problem
formulation).  It shares no code with the HIP library and must never be imported by
the product path; only tests, the smoke check and the benchmark's CPU-baseline leg
use it.

What it builds (paper, Section 2):
  * the normalised adjacency  A~ = (D+I)^(-1/2) (A+I) (D+I)^(-1/2)  of an undirected,
    unweighted graph, D = degree matrix of A        (text below Problem 1);
  * the partition of the nodes into M communities V_m (given, the paper uses METIS),
    the neighbour-community sets N_m                (text above the block matrix);
  * the block split A~_{m,r} of A~                   (block matrix above Problem 3).

Readings taken where the paper is silent: repeated edges, both orientations and self
pairs in the input are normalised away before I is added; nodes are renumbered by a
stable sort on (community, original id) so that each community is a contiguous row
range; 1/sqrt(d_i d_j) is evaluated as 1.0 / sqrt(double(d_i) * double(d_j)).
"""
from __future__ import annotations

import numpy as np
import scipy.sparse as sp


class OracleGraph:
    def __init__(self, N, src, dst, M, comm=None, split=True):
        N = int(N)
        M = int(M)
        src = np.asarray(src, dtype=np.int64).ravel()
        dst = np.asarray(dst, dtype=np.int64).ravel()
        if N < 1 or M < 1:
            raise ValueError("N and M must be positive")
        if src.shape != dst.shape:
            raise ValueError("src/dst length mismatch")
        if src.size and (src.min() < 0 or dst.min() < 0 or src.max() >= N or dst.max() >= N):
            raise ValueError("edge endpoint out of range")
        if comm is None:
            chunk = -(-N // M)
            comm = np.arange(N, dtype=np.int64) // chunk
        comm = np.asarray(comm, dtype=np.int64).ravel()
        if comm.shape[0] != N or comm.min() < 0 or comm.max() >= M:
            raise ValueError("community id out of range")
        self.N, self.M = N, M

        # undirected simple graph: unordered pairs, no self pairs, no repeats
        keep = src != dst
        lo = np.minimum(src[keep], dst[keep])
        hi = np.maximum(src[keep], dst[keep])
        key = np.unique(lo * N + hi)
        lo, hi = key // N, key % N
        self.E = int(key.shape[0])

        # degree of A, and d~ = 1 + degree
        deg = np.bincount(lo, minlength=N) + np.bincount(hi, minlength=N)
        dt = (deg + 1).astype(np.int64)

        # community-contiguous numbering: perm[new] = old
        self.perm = np.argsort(comm, kind="stable").astype(np.int64)
        self.inv_perm = np.empty(N, dtype=np.int64)
        self.inv_perm[self.perm] = np.arange(N, dtype=np.int64)
        self.comm_new = comm[self.perm]
        self.comm_row_ptr = np.concatenate([[0], np.cumsum(np.bincount(comm, minlength=M))]).astype(np.int64)
        self.dtilde = dt[self.perm]

        # A + I in the new numbering, both orientations
        r = np.concatenate([self.inv_perm[lo], self.inv_perm[hi], np.arange(N, dtype=np.int64)])
        c = np.concatenate([self.inv_perm[hi], self.inv_perm[lo], np.arange(N, dtype=np.int64)])
        ones = np.ones(r.shape[0], dtype=np.float64)
        AI = sp.csr_matrix((ones, (r, c)), shape=(N, N))
        AI.sum_duplicates()
        AI.sort_indices()
        self.A_plus_I = AI                      # unnormalised, entries exactly 1.0
        rows = np.repeat(np.arange(N, dtype=np.int64), np.diff(AI.indptr))
        cols = AI.indices.astype(np.int64)
        val = 1.0 / np.sqrt(self.dtilde[rows].astype(np.float64) * self.dtilde[cols].astype(np.float64))
        self.A = sp.csr_matrix((val, AI.indices.copy(), AI.indptr.copy()), shape=(N, N))
        self.row_ptr = self.A.indptr.astype(np.int64)
        self.col = self.A.indices.astype(np.int32)
        self.val = self.A.data.astype(np.float64)
        self.nnz = int(self.A.nnz)

        # neighbour-community sets N_m (as a boolean M x M matrix without the diagonal)
        cr, cc = self.comm_new[rows], self.comm_new[cols]
        nb = np.zeros((M, M), dtype=bool)
        nb[cr, cc] = True
        np.fill_diagonal(nb, False)
        self.neighbour = nb

        # per-row community segments: maximal runs of equal column community inside a row
        # (columns are sorted and communities are contiguous column ranges)
        first = np.ones(self.nnz, dtype=bool)
        if self.nnz > 1:
            first[1:] = (rows[1:] != rows[:-1]) | (cc[1:] != cc[:-1])
        starts = np.flatnonzero(first).astype(np.int64)
        self.seg_ptr = np.concatenate([starts, [self.nnz]]).astype(np.int64)
        self.seg_row = rows[starts].astype(np.int32)
        self.seg_comm = cc[starts].astype(np.int32)
        self.n_segments = int(starts.shape[0])
        halo = np.zeros(N, dtype=bool)
        halo[rows[cr != cc]] = True
        self.n_halo_rows = int(halo.sum())

        # blocks A~_{m,r}, r in N_m or r == m (skipped for very large graphs that only use the full-graph forms)
        self.block = self.split_blocks(self.A) if split else None

    def split_blocks(self, matrix):
        """Cut an N x N sparse matrix into the blocks (m, r), r in N_m or r == m."""
        block = {}
        for m in range(self.M):
            rm = self.rows(m)
            Am = matrix[rm.start:rm.stop, :].tocsc()
            for q in self.nbr_and_self(m):
                rq = self.rows(q)
                block[(m, q)] = Am[:, rq.start:rq.stop].tocsr()
        return block

    def rows(self, m) -> slice:
        return slice(int(self.comm_row_ptr[m]), int(self.comm_row_ptr[m + 1]))

    def nbrs(self, m):
        """N_m of the paper: communities other than m joined to m by at least one edge."""
        return [int(q) for q in np.flatnonzero(self.neighbour[m])]

    def nbr_and_self(self, m):
        return sorted(self.nbrs(m) + [m])

    def aggregate_block(self, m, Z, block=None):
        """Row block m of A~ Z in the paper's blocked form:  A~_{m,m} Z_m + sum_{r in N_m} A~_{m,r} Z_r.
        ``block`` substitutes the blocks of another matrix with the same sparsity (used by tests)."""
        block = self.block if block is None else block
        out = block[(m, m)] @ Z[self.rows(m)]
        for q in self.nbrs(m):
            out = out + block[(m, q)] @ Z[self.rows(q)]
        return out

    def to_new(self, X_old):
        """Reorder rows from the caller's node order to the community-contiguous order."""
        return np.asarray(X_old)[self.perm]

    def to_old(self, X_new):
        out = np.empty_like(X_new)
        out[self.perm] = X_new
        return out
