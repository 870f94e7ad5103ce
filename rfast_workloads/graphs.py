"""Seeded builders for the two communication graphs of R-FAST.

Notation (Section "Network Model" and Assumption 1 of the paper): W is the
row-stochastic pull matrix (called R here, after the build's vocabulary) and A
is the column-stochastic push matrix (called C here).  Both are stored as CSR
with ROW = RECEIVER: row i lists the in-neighbours j of node i, the mandatory
self-loop included, columns ascending.  For R each row sums to one; for C each
COLUMN sums to one (entry (i, j) is the share of node j's mass pushed to i).

This module only lays out indices and weights.  It holds none of the method's
arithmetic and is imported by the tests and the benchmark, never by the oracle
or the HIP library.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class CSRGraph:
    """CSR with row = receiver, diagonal included, columns ascending."""

    n: int
    rowptr: np.ndarray  # int32 [n+1]
    col: np.ndarray     # int32 [nnz]
    w: np.ndarray       # float64 [nnz]; exactly the values the fp32 API receives, upcast

    @property
    def nnz(self) -> int:
        return int(self.col.shape[0])

    @property
    def nnz_off(self) -> int:
        return self.nnz - self.n

    def dense(self) -> np.ndarray:
        m = np.zeros((self.n, self.n), dtype=np.float64)
        for i in range(self.n):
            for k in range(self.rowptr[i], self.rowptr[i + 1]):
                m[i, self.col[k]] = self.w[k]
        return m

    def off_edges(self):
        """(receiver, sender) of every off-diagonal entry, in CSR order.

        The position in this list is the edge id used by every per-edge array
        (delays, drops, stamps, rho rings)."""
        out = []
        for i in range(self.n):
            for k in range(self.rowptr[i], self.rowptr[i + 1]):
                j = int(self.col[k])
                if j != i:
                    out.append((i, j))
        return out

    def w32(self) -> np.ndarray:
        return self.w.astype(np.float32)


def from_dense(m: np.ndarray, fp32_weights: bool = True) -> CSRGraph:
    """CSR of the non-zeros of a dense n x n weight matrix.

    With fp32_weights the stored float64 values are the fp32 roundings (the
    instance the GPU library is given); otherwise they are kept exact."""
    n = m.shape[0]
    rowptr = [0]
    col, w = [], []
    for i in range(n):
        for j in range(n):
            if m[i, j] != 0.0:
                col.append(j)
                w.append(m[i, j])
        rowptr.append(len(col))
    w = np.asarray(w, dtype=np.float64)
    if fp32_weights:
        w = w.astype(np.float32).astype(np.float64)
    return CSRGraph(n, np.asarray(rowptr, np.int32), np.asarray(col, np.int32), w)


def _row_uniform(adj: np.ndarray) -> np.ndarray:
    """r_ij = 1 / (1 + in-degree of i): the rule of the appendix on weight
    matrices (weights follow from the number of in-neighbours)."""
    a = adj.astype(np.float64)
    return a / a.sum(axis=1, keepdims=True)


def _col_uniform(adj: np.ndarray) -> np.ndarray:
    """c_ij = 1 / (1 + out-degree of j) (weights from the number of
    out-neighbours)."""
    a = adj.astype(np.float64)
    return a / a.sum(axis=0, keepdims=True)


def directed_ring(n: int):
    """Edges j -> j+1 (mod n) plus self-loops; every weight 1/2."""
    adj = np.eye(n, dtype=bool)
    for j in range(n):
        adj[(j + 1) % n, j] = True  # receiver (j+1) hears sender j
    return _row_uniform(adj), _col_uniform(adj)


def bidirectional_ring(n: int):
    adj = np.eye(n, dtype=bool)
    for j in range(n):
        adj[(j + 1) % n, j] = True
        adj[(j - 1) % n, j] = True
    return _row_uniform(adj), _col_uniform(adj)


def exponential(n: int):
    """Node j sends to j + 2^k (mod n) for every 2^k < n; uniform weights."""
    adj = np.eye(n, dtype=bool)
    k = 1
    while k < n:
        for j in range(n):
            adj[(j + k) % n, j] = True
        k *= 2
    return _row_uniform(adj), _col_uniform(adj)


def tree_pull_star_push(n: int):
    """R: every node i > 0 mixes 1/2 itself + 1/2 its parent (i-1)//2 in a
    balanced binary tree rooted at 0 (root keeps weight 1).  C: every node
    j > 0 keeps 1/2 and pushes 1/2 straight to node 0 (root keeps 1).  The two
    spanning trees differ and share root 0 (Assumption 2)."""
    r = np.zeros((n, n))
    c = np.zeros((n, n))
    r[0, 0] = 1.0
    c[0, 0] = 1.0
    for i in range(1, n):
        r[i, i] = 0.5
        r[i, (i - 1) // 2] = 0.5
        c[i, i] = 0.5
        c[0, i] = 0.5
    return r, c


def line_tree(n: int):
    """R: oriented line rooted at 0 (i pulls from i-1); C: the reversed line
    (i pushes to i-1).  Weights 1/2, root 1."""
    r = np.zeros((n, n))
    c = np.zeros((n, n))
    r[0, 0] = 1.0
    c[0, 0] = 1.0
    for i in range(1, n):
        r[i, i] = 0.5
        r[i, i - 1] = 0.5
        c[i, i] = 0.5
        c[i - 1, i] = 0.5
    return r, c


def binary_tree(n: int):
    """The tree pair of the experiments on general topologies: G(R) is the oriented
    balanced binary tree rooted at 0 (node i > 0 hears its parent (i-1)//2), G(C) its
    inverse (node i > 0 sends to its parent); weights from the degrees, so 1/2 and 1/2
    off the root, 1 at the root of R, and a parent with k children receives 1/2 from each
    while keeping 1 itself in its own column."""
    adj_r = np.eye(n, dtype=bool)
    adj_c = np.eye(n, dtype=bool)
    for i in range(1, n):
        adj_r[i, (i - 1) // 2] = True   # receiver i hears its parent
        adj_c[(i - 1) // 2, i] = True   # receiver parent hears child i
    return _row_uniform(adj_r), _col_uniform(adj_c)


def mesh(n: int, cols: int = 0):
    """Bidirectional 2-D grid (4-neighbourhood, no wrap-around), row-major on `cols`
    columns (default: ceil(sqrt(n))); the last row may be short.  Strongly connected, so
    every node is a common root.  The paper shows its mesh only as a figure: the grid is
    this repository's reading of the word."""
    if cols <= 0:
        cols = int(np.ceil(np.sqrt(n)))
    adj = np.eye(n, dtype=bool)
    for a in range(n):
        r, c = divmod(a, cols)
        for b in ((r, c + 1), (r + 1, c)):
            j = b[0] * cols + b[1]
            if b[1] < cols and j < n:
                adj[a, j] = adj[j, a] = True
    return _row_uniform(adj), _col_uniform(adj)


def multi_root_split(n: int, servers: int):
    """Parameter-server-like split of the appendix on topology design: nodes 0..servers-1
    exchange both ways on a ring among themselves in both graphs; a worker w >= servers
    hears server w mod servers in G(R) and sends to it in G(C).  The common roots are
    exactly the servers."""
    assert 1 <= servers <= n
    adj_r = np.eye(n, dtype=bool)
    adj_c = np.eye(n, dtype=bool)
    for a in range(servers):
        for b in ((a + 1) % servers, (a - 1) % servers):
            adj_r[a, b] = adj_c[a, b] = True
    for w in range(servers, n):
        adj_r[w, w % servers] = True
        adj_c[w % servers, w] = True
    return _row_uniform(adj_r), _col_uniform(adj_c)


def random_digraph(n: int, rng: np.random.Generator, extra: float = 0.3):
    """A random strongly connected pair (ring backbone plus random chords with
    random positive weights); used by property tests."""
    adj_r = np.eye(n, dtype=bool)
    adj_c = np.eye(n, dtype=bool)
    perm = rng.permutation(n)
    for a in range(n):
        adj_r[perm[(a + 1) % n], perm[a]] = True
        adj_c[perm[(a + 1) % n], perm[a]] = True
    adj_r |= rng.random((n, n)) < extra
    adj_c |= rng.random((n, n)) < extra
    wr = adj_r * rng.uniform(0.2, 1.0, (n, n))
    wc = adj_c * rng.uniform(0.2, 1.0, (n, n))
    wr /= wr.sum(axis=1, keepdims=True)
    wc /= wc.sum(axis=0, keepdims=True)
    return wr, wc
