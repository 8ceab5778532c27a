"""gosh_coarsen_device (Alg. 4 on the GPU: degree sort, marking rounds, CSR rebuild) against
the oracle and against gosh_coarsen: the hierarchy is unique, so everything is compared
bit for bit."""
import ctypes as C

import numpy as np
import pytest
import torch

import graphgen
import paper_2008_12336_amd as G
from oracle import gosh_oracle as O
from tests.test_coarsen import _ring_lattice, assert_same_hierarchy
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


@pytest.mark.parametrize("name", ["path", "ring3", "uniform", "mixed"])
def test_device_marking_with_long_dependency_chains(name):
    """Graphs whose marking is one long chain (the rounds stall and the host sweep takes
    over) or many short ones (resolved by the rounds) still give the sequential result."""
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
    graphs, maps, mults = O.coarsen(xadj, adj, threshold=n // 2, min_shrink=1.0, max_levels=2)
    h = device_hierarchy(n, xadj, adj, False, threshold=n // 2, min_shrink=1.0, max_levels=2)
    assert_same_hierarchy(h, graphs, maps, mults)
    h.free()


def test_device_isolated_vertices_and_no_progress():
    # only isolated vertices: nothing merges, the hierarchy keeps the one level and no map
    xadj, adj = csr_from_pairs(10, [])
    h = device_hierarchy(10, xadj, adj, False, threshold=1)
    assert h.levels == 1
    h.free()
    # a star plus isolated vertices: one merge level, then no progress
    xadj, adj = csr_from_pairs(12, [(0, i) for i in range(1, 6)])
    graphs, maps, mults = O.coarsen(xadj, adj, threshold=1, min_shrink=1.0)
    h = device_hierarchy(12, xadj, adj, True, threshold=1, min_shrink=1.0)
    assert_same_hierarchy(h, graphs, maps, mults)
    h.free()


def test_release_device_keeps_everything_readable():
    n = 4096
    c = graphgen.to_csr(n, graphgen.rmat(12, 1 << 15, 2))
    xadj, adj = c.xadj.numpy(), c.adj.numpy()
    graphs, maps, mults = O.coarsen(xadj, adj, threshold=100, min_shrink=1.0)
    h = G.gosh_coarsen_device(n, c.xadj, c.adj, threshold=100, min_shrink=1.0)
    h.trim_scratch()  # the levels stay on the device
    h.trim_scratch()
    assert np.array_equal(h.map(0), maps[0])
    h.release_device()
    assert_same_hierarchy(h, graphs, maps, mults)
    # training from the released (host) copies still works and agrees with the oracle's shapes
    M0 = torch.zeros(n, 16, dtype=torch.float32, device="cuda:0")
    stats = G.gosh_embed(h, M0, 3, 12, 0.3, 0.05, 1, flags=G.GOSH_FLAG_SEQUENTIAL)
    torch.cuda.synchronize()
    assert [s["n"] for s in stats] == [g[0].size - 1 for g in graphs]
    assert bool(torch.isfinite(M0).all())
    h.release_device()  # idempotent
    h.free()


def test_device_rejects_malformed_graphs():
    xadj, adj = csr_from_pairs(300, [(i, i + 1) for i in range(299)])
    bad_adj = adj.copy()
    bad_adj[7] = 300  # neighbour id out of range
    with pytest.raises(G.GoshError, match="neighbour"):
        device_hierarchy(300, xadj, bad_adj, False, threshold=10)
    bad_x = xadj.copy()
    bad_x[5] = bad_x[6] + 1  # offsets decrease
    with pytest.raises(G.GoshError, match="xadj"):
        device_hierarchy(300, bad_x, adj, False, threshold=10)
    # the device is still usable afterwards
    h = device_hierarchy(300, xadj, adj, False, threshold=10)
    assert h.levels >= 2
    h.free()


@pytest.mark.parametrize("offsets64", [False, True])
def test_device_resident_input_graph(offsets64):
    """G_0 given as device tensors is used in place (no upload), gives the same hierarchy,
    and its host copy appears on request."""
    n = 4096
    c = graphgen.to_csr(n, graphgen.rmat(12, 1 << 15, 2), offsets64=offsets64)
    xadj, adj = c.xadj.numpy(), c.adj.numpy()
    graphs, maps, mults = O.coarsen(xadj, adj, threshold=100, min_shrink=0.8)
    xd, ad = c.xadj.to("cuda:0"), c.adj.to("cuda:0")
    h = G.gosh_coarsen_device(n, xd, ad, threshold=100, min_shrink=0.8)
    # train first (nothing has been downloaded yet), then read everything back
    want, _, _, _ = O.embed(xadj, adj, 16, 3, 12, 0.3, 0.05, 4, threshold=100, min_shrink=0.8)
    M0 = torch.zeros(n, 16, dtype=torch.float32, device="cuda:0")
    assert h.shape(0) == (n, adj.size) and h.shape(1)[0] == graphs[1][0].size - 1
    stats = G.gosh_embed(h, M0, 3, 12, 0.3, 0.05, 4, flags=G.GOSH_FLAG_SEQUENTIAL)
    torch.cuda.synchronize()
    assert all(s["upload_ms"] < 5.0 for s in stats)
    err = np.abs(M0.cpu().numpy() - want).max() / np.abs(want).max()
    assert err <= 1e-5
    assert_same_hierarchy(h, graphs, maps, mults)
    n0, x0, a0 = h.graph(0)
    assert x0.dtype == (np.int64 if offsets64 else np.int32)
    h.release_device()  # the caller's device tensors stay the caller's
    assert_same_hierarchy(h, graphs, maps, mults)
    h.free()
    assert torch.equal(xd.cpu(), c.xadj) and torch.equal(ad.cpu(), c.adj)
    with pytest.raises(TypeError):
        G.gosh_coarsen_device(n, xd, c.adj, threshold=100)
    with pytest.raises(TypeError):
        G.gosh_coarsen(n, xd, ad, threshold=100)
    # the C entry points that read the graph on the host refuse device memory themselves
    gd = G.csr_view(n, xd, ad)
    out = C.c_void_p()
    assert G.lib().gosh_coarsen(C.byref(gd), 100, 1.0, 64, 0, C.byref(out)) == -1
    assert "host graph" in G.gosh_last_error()
    assert G.lib().gosh_csr_validate(C.byref(gd)) == -1


from hypothesis import given, settings, strategies as st  # noqa: E402

_graphs = st.integers(min_value=2, max_value=90).flatmap(
    lambda n: st.tuples(st.just(n), st.lists(
        st.tuples(st.integers(0, n - 1), st.integers(0, n - 1)), min_size=0, max_size=6 * n)))


@settings(max_examples=60, deadline=None)
@given(_graphs, st.booleans())
def test_device_random_tiny_graphs_match_oracle(g, offsets64):
    n, pairs = g
    xadj, adj = csr_from_pairs(n, pairs)
    graphs, maps, mults = O.coarsen(xadj, adj, threshold=1, min_shrink=1.0)
    h = device_hierarchy(n, xadj, adj, offsets64, threshold=1, min_shrink=1.0)
    assert_same_hierarchy(h, graphs, maps, mults)
    h.free()
