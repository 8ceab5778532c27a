"""Helpers shared by the tests (graph fixtures, small numpy utilities)."""
from __future__ import annotations

import numpy as np
import torch

import graphgen


def csr_from_pairs(n, pairs):
    """Sorted symmetric CSR (int64 xadj, int32 adj) from undirected (u, v) pairs."""
    nbrs = [set() for _ in range(n)]
    for u, v in pairs:
        if u == v:
            continue
        nbrs[u].add(v)
        nbrs[v].add(u)
    xadj = np.zeros(n + 1, dtype=np.int64)
    adj = []
    for v in range(n):
        row = sorted(nbrs[v])
        adj.extend(row)
        xadj[v + 1] = len(adj)
    return xadj, np.asarray(adj, dtype=np.int32)


def csr_numpy(csr: graphgen.CSR):
    return (csr.xadj.cpu().numpy().astype(np.int64), csr.adj.cpu().numpy().astype(np.int32))


def dense_from_csr(xadj, adj):
    n = xadj.size - 1
    A = np.zeros((n, n), dtype=np.int64)
    for v in range(n):
        A[v, adj[xadj[v]:xadj[v + 1]]] = 1
    return A


def config1_graph(seed=1, holdout=0.1):
    """Config 1: 1,024 vertices, 8,192 uniform-endpoint draws, 10 % of edges held out."""
    edges = graphgen.er_gnm(1024, 8192, seed)
    train, test = graphgen.holdout_split(edges, holdout, seed + 1000)
    return 1024, train, test


def rel_err(a, b):
    """max |a - b| / max |b| -- the relative error the parity bar is stated in."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-30))


def corrupt(c, offsets64, seed, stray=0):
    """A copy of the CSR arrays with offsets that leave adj, entries that name no vertex and
    `stray` entries replaced by arbitrary vertices (their rows are no longer ascending).
    Returns (xadj, adj, rows whose offsets were touched)."""
    rng = np.random.default_rng(seed)
    n = c.xadj.numel() - 1
    xadj = c.xadj.numpy().astype(np.int64 if offsets64 else np.int32).copy()
    adj = c.adj.numpy().copy()
    nnz = adj.size
    where = rng.choice(np.arange(2, n - 2, 4), size=12, replace=False)  # no two touch one row
    huge = (1 << 40) if offsets64 else 2**31 - 1
    for v, bad in zip(where, [nnz + 7, -3, huge, -huge, nnz + 1, -1] * 2):
        xadj[v] = bad
    touched = set(int(v) for v in where) | set(int(v) - 1 for v in where)
    entries = rng.choice(nnz, size=40, replace=False)
    for j, bad in zip(entries, [n, -1, 2**31 - 1, -2**31, n + 100] * 8):
        adj[j] = bad
    for j in rng.choice(nnz, size=stray, replace=False):
        adj[j] = rng.integers(0, n)
    return xadj, adj, touched


def one_ulp_away(M, seed=0):
    """A copy of the fp32 matrix with every entry moved to a neighbouring fp32 value."""
    rng = np.random.default_rng(seed)
    toward = np.where(rng.integers(0, 2, M.shape) == 1, np.float32(np.inf), np.float32(-np.inf)).astype(np.float32)
    return np.nextafter(M, toward)


def oracle_sensitivity(run, M0):
    """How far the oracle's own result moves (max |diff| / max |M|) when every entry of its
    input moves by one unit in the last place.  `run(M)` trains M in place with the oracle.
    A stable run returns about 1e-6 (ten or so times the perturbation); a run whose rows are
    so long that lr * |row|^2 / 4 exceeds 1 takes SGD steps larger than the curvature of the
    logistic loss allows and amplifies any difference by orders of magnitude -- there the
    oracle's value is one of many equally good ones, and no implementation that rounds
    differently can match it to 1e-5."""
    a, b = M0.copy(), one_ulp_away(M0)
    run(a)
    run(b)
    return a, rel_err(b, a)


def conditioned_bar(sensitivity):
    """Sequential-order bar for one run: 1e-5 relative (the kernel's fp32 dot product, fp32
    sigmoid and fused axpys differ from the oracle's fp64 arithmetic by a few units of 2^-24
    per update); for a run that the oracle itself cannot repeat to 1e-6 from an input moved by
    one ulp, eight times that sensitivity -- the kernel's differences enter at every update,
    not once at the start."""
    return max(1e-5, 8.0 * float(sensitivity))
