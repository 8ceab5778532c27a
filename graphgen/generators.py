"""Edge-list generators and CSR construction (inputs only, no method arithmetic).

All generators return an int64 tensor ``edges`` of shape [m', 2] holding each
undirected edge once as (u, v) with u < v, sorted by (u, v), without self loops
or duplicates.  ``m'`` can be slightly below the requested number of draws
because loops and repeated pairs are dropped, not redrawn.
"""
from __future__ import annotations

from dataclasses import dataclass

import torch


@dataclass
class CSR:
    """Compressed sparse row adjacency of a symmetric graph.

    ``xadj`` has n+1 offsets (int32 or int64), ``adj`` holds the neighbour ids
    (int32) of vertex 0, then vertex 1, ... ; every row is sorted ascending,
    has no duplicates and no self loop.
    """

    n: int
    xadj: torch.Tensor
    adj: torch.Tensor

    @property
    def nnz(self) -> int:
        return int(self.adj.numel())

    def to(self, device) -> "CSR":
        return CSR(self.n, self.xadj.to(device), self.adj.to(device))


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _canonical(u: torch.Tensor, v: torch.Tensor, n: int) -> torch.Tensor:
    """Drop loops, order endpoints, drop duplicates; result sorted by (u, v)."""
    keep = u != v
    u, v = u[keep], v[keep]
    lo = torch.minimum(u, v)
    hi = torch.maximum(u, v)
    del u, v
    key = torch.unique(lo * n + hi)  # sorted
    del lo, hi
    return torch.stack((key // n, key % n), dim=1)


def er_gnm(n: int, m: int, seed: int, device="cpu") -> torch.Tensor:
    """Erdos-Renyi G(n, m)-style graph: m pairs with independent uniform endpoints."""
    g = _gen(seed, device)
    u = torch.randint(0, n, (m,), generator=g, device=device, dtype=torch.int64)
    v = torch.randint(0, n, (m,), generator=g, device=device, dtype=torch.int64)
    return _canonical(u, v, n)


def rmat(scale: int, m: int, seed: int, a=0.57, b=0.19, c=0.19, d=0.05,
         device="cpu", permute=True, chunk=1 << 24) -> torch.Tensor:
    """R-MAT graph on n = 2**scale vertices from m recursive-quadrant draws.

    Each draw descends ``scale`` levels; at every level the (row, column) bit pair
    is (0,0), (0,1), (1,0), (1,1) with probability a, b, c, d.  Vertex labels are
    then shuffled with a seeded permutation so that degree is not a function of id.
    """
    assert abs(a + b + c + d - 1.0) < 1e-9
    n = 1 << scale
    g = _gen(seed, device)
    us, vs = [], []
    for start in range(0, m, chunk):
        cnt = min(chunk, m - start)
        u = torch.zeros(cnt, dtype=torch.int64, device=device)
        v = torch.zeros(cnt, dtype=torch.int64, device=device)
        for _ in range(scale):
            r = torch.rand(cnt, generator=g, device=device, dtype=torch.float64)
            ubit = (r >= a + b).to(torch.int64)
            vbit = (((r >= a) & (r < a + b)) | (r >= a + b + c)).to(torch.int64)
            u = (u << 1) | ubit
            v = (v << 1) | vbit
        us.append(u)
        vs.append(v)
    u = torch.cat(us)
    v = torch.cat(vs)
    del us, vs
    if permute:
        perm = torch.randperm(n, generator=g, device=device)
        u = perm[u]
        v = perm[v]
    return _canonical(u, v, n)


def _power_law_cdf(n: int, m: int, gamma: float, device) -> torch.Tensor:
    """Cumulative endpoint distribution for weights w_i = (i + i0)^(-1/(gamma-1)).

    The shift i0 is the smallest value for which the largest expected degree,
    2m * w_0 / sum(w), does not exceed sqrt(2m) -- the usual condition that keeps
    every Chung-Lu pair probability below one.
    """
    alpha = 1.0 / (gamma - 1.0)
    idx = torch.arange(n, dtype=torch.float64, device=device)
    cap = (2.0 * m) ** 0.5

    def max_deg(i0: float) -> float:
        w = (idx + i0) ** (-alpha)
        return float(2.0 * m * w[0] / w.sum())

    lo, hi = 1.0, 2.0
    while max_deg(hi) > cap:
        lo, hi = hi, hi * 2.0
    if max_deg(lo) <= cap:
        hi = lo
    else:
        for _ in range(40):
            mid = 0.5 * (lo + hi)
            if max_deg(mid) > cap:
                lo = mid
            else:
                hi = mid
    w = (idx + hi) ** (-alpha)
    # The running sum is taken on the host: a device scan adds its partial sums in an order
    # that depends on timing, so its fp64 result differs in the last bits from run to run, and
    # among billions of draws a few then land on the other side of a boundary.  The graph must
    # be a function of the seed alone.
    cdf = torch.cumsum(w.cpu(), 0)
    return (cdf / cdf[-1]).to(device)


def chung_lu(n: int, m: int, seed: int, gamma=2.1, device="cpu", permute=True,
             chunk=1 << 26) -> torch.Tensor:
    """Chung-Lu style power-law graph: m pairs, both endpoints drawn independently
    with probability proportional to a power-law weight sequence of exponent gamma."""
    g = _gen(seed, device)
    cdf = _power_law_cdf(n, m, gamma, device)
    keys = []
    perm = torch.randperm(n, generator=g, device=device) if permute else None
    for start in range(0, m, chunk):
        cnt = min(chunk, m - start)
        ends = []
        for _ in range(2):
            r = torch.rand(cnt, generator=g, device=device, dtype=torch.float64)
            e = torch.searchsorted(cdf, r).clamp_(max=n - 1)
            ends.append(perm[e] if perm is not None else e)
        u, v = ends
        keep = u != v
        u, v = u[keep], v[keep]
        keys.append(torch.minimum(u, v) * n + torch.maximum(u, v))
        del u, v, ends
    key = torch.unique(torch.cat(keys))
    del keys
    return torch.stack((key // n, key % n), dim=1)


def two_cliques(size: int, bridges: int = 1) -> torch.Tensor:
    """Two cliques of ``size`` vertices joined by ``bridges`` edges (a graph whose
    community structure any sensible embedding must recover)."""
    e = []
    for base in (0, size):
        for i in range(size):
            for j in range(i + 1, size):
                e.append((base + i, base + j))
    for t in range(bridges):
        e.append((t, size + t))
    e = torch.tensor(sorted(e), dtype=torch.int64)
    return e


def holdout_split(edges: torch.Tensor, frac: float, seed: int):
    """Split undirected edges into (train, test); ``frac`` of them go to test."""
    m = edges.shape[0]
    g = _gen(seed, edges.device)
    perm = torch.randperm(m, generator=g, device=edges.device)
    n_test = int(round(m * frac))
    test_idx = torch.sort(perm[:n_test]).values
    train_idx = torch.sort(perm[n_test:]).values
    return edges[train_idx], edges[test_idx]


def to_csr(n: int, edges: torch.Tensor, offsets64: bool = False) -> CSR:
    """Symmetrise an undirected edge list (each edge once as (u, v), u < v, sorted by
    (u, v)) into sorted CSR.

    The row of a vertex r is its smaller neighbours (pairs in which r is the larger
    endpoint) followed by its larger neighbours (pairs in which r is the smaller one);
    both runs are ascending, so only the reversed pairs need a sort."""
    dev = edges.device
    m = edges.shape[0]
    u, v = edges[:, 0], edges[:, 1]
    cnt_hi = torch.bincount(u, minlength=n)  # larger neighbours of each vertex
    cnt_lo = torch.bincount(v, minlength=n)  # smaller neighbours of each vertex
    xadj = torch.zeros(n + 1, dtype=torch.int64, device=dev)
    torch.cumsum(cnt_lo + cnt_hi, 0, out=xadj[1:])
    adj = torch.empty(2 * m, dtype=torch.int32, device=dev)
    ar = torch.arange(m, dtype=torch.int64, device=dev)
    # forward pairs are already grouped by u with v ascending
    start_hi = torch.cumsum(cnt_hi, 0) - cnt_hi
    pos = xadj[:-1][u] + cnt_lo[u] + (ar - start_hi[u])
    adj[pos] = v.to(torch.int32)
    del pos, start_hi, cnt_hi
    # reversed pairs: sort by (v, u)
    key = torch.sort(v * n + u).values
    vs = key // n
    us = (key - vs * n).to(torch.int32)
    del key
    start_lo = torch.cumsum(cnt_lo, 0) - cnt_lo
    pos = xadj[:-1][vs] + (ar - start_lo[vs])
    adj[pos] = us
    del pos, vs, us, ar, start_lo, cnt_lo
    if not offsets64:
        assert int(xadj[-1]) < 2 ** 31
        xadj = xadj.to(torch.int32)
    return CSR(n, xadj, adj)
