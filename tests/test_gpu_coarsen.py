"""gosh_coarsen_device (coarse CSR rebuilt on the GPU) against the oracle's Alg. 4 and
against gosh_coarsen: the hierarchy is unique, so everything is compared bit for bit."""
import numpy as np
import pytest
import torch

import graphgen
import paper_2008_12336_amd as G
from oracle import gosh_oracle as O
from tests.test_coarsen import assert_same_hierarchy
from tests.util import csr_from_pairs

pytestmark = pytest.mark.gpu


def device_hierarchy(n, xadj, adj, offsets64, **kw):
    xt = torch.from_numpy(np.asarray(xadj, dtype=np.int64 if offsets64 else np.int32))
    at = torch.from_numpy(np.asarray(adj, dtype=np.int32))
    return G.gosh_coarsen_device(n, xt, at, **kw)


CASES = {
    "er1024": lambda: (1024, graphgen.er_gnm(1024, 8192, 1)),
    "rmat4096": lambda: (4096, graphgen.rmat(12, 1 << 15, 2)),
    "cl5000": lambda: (5000, graphgen.chung_lu(5000, 40000, 3)),
    "rmat65536": lambda: (1 << 16, graphgen.rmat(16, 1 << 19, 5)),
}


@pytest.mark.parametrize("name", sorted(CASES))
@pytest.mark.parametrize("offsets64", [False, True])
def test_device_hierarchy_matches_oracle(name, offsets64):
    n, edges = CASES[name]()
    c = graphgen.to_csr(n, edges)
    xadj, adj = c.xadj.numpy(), c.adj.numpy()
    for kw in (dict(threshold=100, min_shrink=1.0), dict(threshold=50, min_shrink=0.8),
               dict(threshold=10, min_shrink=1.0, max_levels=3)):
        graphs, maps, mults = O.coarsen(xadj, adj, **kw)
        h = device_hierarchy(n, xadj, adj, offsets64, **kw)
        assert_same_hierarchy(h, graphs, maps, mults)
        assert h.levels >= 2
        h.free()


def test_device_tiny_and_degenerate():
    rng = np.random.default_rng(11)
    for n in (2, 3, 7, 33, 64, 65):
        for m in (0, 1, n, 4 * n):
            pairs = [(int(a), int(b)) for a, b in rng.integers(0, n, size=(m, 2))]
            xadj, adj = csr_from_pairs(n, pairs)
            graphs, maps, mults = O.coarsen(xadj, adj, threshold=1, min_shrink=1.0)
            h = device_hierarchy(n, xadj, adj, False, threshold=1, min_shrink=1.0)
            assert_same_hierarchy(h, graphs, maps, mults)
            h.free()
    # a clique collapses into one vertex: every entry falls inside the cluster
    pairs = [(i, j) for i in range(6) for j in range(i)]
    xadj, adj = csr_from_pairs(6, pairs)
    h = device_hierarchy(6, xadj, adj, True, threshold=1)
    n1, x1, a1 = h.graph(1)
    assert n1 == 1 and a1.size == 0 and list(x1) == [0, 0]
    h.free()


def test_device_large_matches_host():
    # 2^20 vertices, hub rows far longer than a wavefront: beyond what the oracle does fast
    n = 1 << 20
    c = graphgen.to_csr(n, graphgen.chung_lu(n, 1 << 23, 4), offsets64=True)
    hh = G.gosh_coarsen(n, c.xadj, c.adj, threshold=100, min_shrink=0.8)
    hd = G.gosh_coarsen_device(n, c.xadj, c.adj, threshold=100, min_shrink=0.8)
    assert hh.levels == hd.levels
    for i in range(hh.levels):
        nh, xh, ah = hh.graph(i)
        nd, xd, ad = hd.graph(i)
        assert nh == nd and np.array_equal(xh, xd) and np.array_equal(ah, ad)
        if i > 0:
            assert np.array_equal(hh.mult(i), hd.mult(i))
            assert int(hd.mult(i).sum()) <= c.adj.numel()
        if i + 1 < hh.levels:
            assert np.array_equal(hh.map(i), hd.map(i))
    hh.free()
    hd.free()
