"""gosh_coarsen (host C++) against the oracle's Alg. 4: maps and graphs bit-exact."""
import numpy as np
import pytest
import torch
from hypothesis import given, settings, strategies as st

import graphgen
import paper_2008_12336_amd as G
from oracle import gosh_oracle as O
from tests.util import csr_from_pairs


def product_hierarchy(n, xadj, adj, offsets64, **kw):
    xt = torch.from_numpy(np.asarray(xadj, dtype=np.int64 if offsets64 else np.int32))
    at = torch.from_numpy(np.asarray(adj, dtype=np.int32))
    return G.gosh_coarsen(n, xt, at, **kw)


def assert_same_hierarchy(h, graphs, maps, mults):
    assert h.levels == len(graphs)
    for i, (xo, ao) in enumerate(graphs):
        n, x, a = h.graph(i)
        assert n == xo.size - 1
        assert np.array_equal(np.asarray(x, dtype=np.int64), xo)
        assert np.array_equal(a, ao)
        m = h.mult(i)
        if i == 0:
            assert m is None
        else:
            assert np.array_equal(np.zeros(0, dtype=np.int64) if m is None else m, mults[i])
    for i, mo in enumerate(maps):
        assert np.array_equal(h.map(i), mo)


CASES = {
    "er1024": lambda: (1024, graphgen.er_gnm(1024, 8192, 1)),
    "rmat4096": lambda: (4096, graphgen.rmat(12, 1 << 15, 2)),
    "cl5000": lambda: (5000, graphgen.chung_lu(5000, 40000, 3)),
    "rmat65536": lambda: (1 << 16, graphgen.rmat(16, 1 << 19, 5)),
}


@pytest.mark.parametrize("name", sorted(CASES))
@pytest.mark.parametrize("offsets64", [False, True])
@pytest.mark.parametrize("threads", [1, 5])
def test_hierarchy_matches_oracle(name, offsets64, threads):
    n, edges = CASES[name]()
    c = graphgen.to_csr(n, edges)
    xadj, adj = c.xadj.numpy(), c.adj.numpy()
    for kw in (dict(threshold=100, min_shrink=1.0), dict(threshold=50, min_shrink=0.8),
               dict(threshold=10, min_shrink=1.0, max_levels=3)):
        graphs, maps, mults = O.coarsen(xadj, adj, **kw)
        h = product_hierarchy(n, xadj, adj, offsets64, n_threads=threads, **kw)
        assert_same_hierarchy(h, graphs, maps, mults)
        assert h.levels >= 2
        h.free()


graphs_st = st.integers(min_value=2, max_value=60).flatmap(
    lambda n: st.tuples(st.just(n), st.lists(
        st.tuples(st.integers(0, n - 1), st.integers(0, n - 1)), min_size=0, max_size=5 * n)))


@settings(max_examples=100, deadline=None)
@given(graphs_st)
def test_random_tiny_graphs_match_oracle(g):
    n, pairs = g
    xadj, adj = csr_from_pairs(n, pairs)
    graphs, maps, mults = O.coarsen(xadj, adj, threshold=1, min_shrink=1.0)
    h = product_hierarchy(n, xadj, adj, False, threshold=1, min_shrink=1.0, n_threads=3)
    assert_same_hierarchy(h, graphs, maps, mults)


def test_edge_cases():
    # at or below the threshold: nothing to build
    xadj, adj = csr_from_pairs(5, [(0, 1), (1, 2)])
    h = product_hierarchy(5, xadj, adj, False, threshold=5)
    assert h.levels == 1
    n, x, a = h.graph(0)
    assert n == 5 and np.array_equal(a, adj)
    with pytest.raises(G.GoshError):
        h.map(0)
    # edgeless graph: nothing can merge, so no level is added
    xe = np.zeros(301, dtype=np.int64)
    h = product_hierarchy(300, xe, np.zeros(0, dtype=np.int32), True, threshold=100, min_shrink=0.8)
    assert h.levels == 1
    with pytest.raises(G.GoshError):
        h.map(0)
    # bad arguments
    for kw in (dict(threshold=0), dict(min_shrink=0.0), dict(min_shrink=1.5), dict(max_levels=0)):
        with pytest.raises(G.GoshError):
            product_hierarchy(5, xadj, adj, False, **kw)


def test_csr_validate():
    xadj, adj = csr_from_pairs(6, [(0, 1), (1, 2), (2, 5)])
    xt, at = torch.from_numpy(xadj), torch.from_numpy(adj)
    G.gosh_csr_validate(G.csr_view(6, xt, at))
    bad = at.clone(); bad[0] = 9
    with pytest.raises(G.GoshError, match="out of range"):
        G.gosh_csr_validate(G.csr_view(6, xt, bad))
    bad = at.clone(); bad[0] = 0  # vertex 0 lists itself
    with pytest.raises(G.GoshError, match="self loop"):
        G.gosh_csr_validate(G.csr_view(6, xt, bad))
    bad = at.clone(); bad[1], bad[2] = at[2].item(), at[1].item()  # row of vertex 1 descending
    with pytest.raises(G.GoshError, match="ascending"):
        G.gosh_csr_validate(G.csr_view(6, xt, bad))
    badx = xt.clone(); badx[-1] = xt[-1] + 1
    with pytest.raises(G.GoshError, match="nnz"):
        G.gosh_csr_validate(G.csr_view(6, badx, at))
    badx = xt.clone(); badx[2] = 0
    with pytest.raises(G.GoshError):
        G.gosh_csr_validate(G.csr_view(6, badx, at))


def _ring_lattice(n, reach):
    """Every vertex has the same degree 2*reach: nobody is above the mean degree, so the
    whole marking is decided by the order alone (long dependency chains)."""
    pairs = [(i, (i + r) % n) for i in range(n) for r in range(1, reach + 1)]
    return csr_from_pairs(n, pairs)


@pytest.mark.parametrize("name", ["path", "ring3", "uniform", "mixed"])
def test_marking_with_long_dependency_chains(name):
    """Graphs on which the out-of-order marking needs many rounds or falls back to the
    in-order sweep must still give the sequential result."""
    if name == "path":
        n = 30000
        xadj, adj = csr_from_pairs(n, [(i, i + 1) for i in range(n - 1)])
    elif name == "ring3":
        n = 20000
        xadj, adj = _ring_lattice(n, 3)
    elif name == "uniform":
        n = 60000
        c = graphgen.to_csr(n, graphgen.er_gnm(n, 4 * n, 11))
        xadj, adj = c.xadj.numpy(), c.adj.numpy()
    else:
        n = 50000
        path = [(i, i + 1) for i in range(30000)]
        c = graphgen.chung_lu(n, 120000, 12)
        xadj, adj = csr_from_pairs(n, path + [tuple(e) for e in c.tolist()])
    for threads in (1, 6):
        graphs, maps, mults = O.coarsen(xadj, adj, threshold=n // 2, min_shrink=1.0, max_levels=2)
        h = product_hierarchy(n, xadj, adj, False, threshold=n // 2, min_shrink=1.0, max_levels=2,
                              n_threads=threads)
        assert_same_hierarchy(h, graphs, maps, mults)


def test_release_device_is_a_noop_for_a_host_built_hierarchy():
    c = graphgen.to_csr(1024, graphgen.er_gnm(1024, 8192, 1))
    xadj, adj = c.xadj.numpy(), c.adj.numpy()
    graphs, maps, mults = O.coarsen(xadj, adj, threshold=100, min_shrink=1.0)
    h = product_hierarchy(1024, xadj, adj, False, threshold=100, min_shrink=1.0)
    h.release_device()
    assert_same_hierarchy(h, graphs, maps, mults)
    h.free()


@pytest.mark.skipif(torch.cuda.is_available(), reason="checks the failure without a device")
def test_device_coarsening_fails_loudly_without_a_device():
    c = graphgen.to_csr(1024, graphgen.er_gnm(1024, 8192, 1))
    with pytest.raises(G.GoshError):
        G.gosh_coarsen_device(1024, c.xadj, c.adj, threshold=100)
    # at or below the threshold there is nothing to do on the device
    h = G.gosh_coarsen_device(1024, c.xadj, c.adj, threshold=5000)
    assert h.levels == 1
    h.free()
