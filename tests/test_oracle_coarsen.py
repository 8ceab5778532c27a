"""Pins for the oracle's MultiEdgeCollapse (Alg. 4), projection and epoch split."""
import os

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import graphgen
from oracle import gosh_oracle as O
from tests.util import csr_from_pairs, dense_from_csr

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _examples():
    out = []
    for line in open(os.path.join(GOLD, "coarsen_examples.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, n, edges, want = [x.strip() for x in line.split("|")]
        pairs = [tuple(map(int, e.split("-"))) for e in edges.split()]
        out.append(pytest.param(int(n), pairs, list(map(int, want.split())), id=name))
    return out


@pytest.mark.parametrize("n,pairs,want", _examples())
def test_worked_examples(n, pairs, want):
    xadj, adj = csr_from_pairs(n, pairs)
    m, nc = O.coarsen_map(xadj, adj)
    assert m.tolist() == want
    assert nc == max(want) + 1


def test_path_quotient_graph():
    xadj, adj = csr_from_pairs(4, [(0, 1), (1, 2), (2, 3)])
    m, nc = O.coarsen_map(xadj, adj)
    xo, ao, mo = O.coarsen_graph(xadj, adj, m, nc)
    assert xo.tolist() == [0, 1, 2] and ao.tolist() == [1, 0] and mo.tolist() == [1, 1]


def dense_reference_map(A):
    """The marking sweep restated on a dense 0/1 matrix (independent data structure)."""
    n = A.shape[0]
    deg = A.sum(1)
    nnz = int(deg.sum())
    order = np.argsort(-deg, kind="stable")
    m = -np.ones(n, dtype=np.int64)
    c = 0
    for v in order:
        if m[v] != -1:
            continue
        m[v] = c
        for u in np.nonzero(A[v])[0]:
            if (deg[v] * n <= nnz or deg[u] * n <= nnz) and m[u] == -1:
                m[u] = c
        c += 1
    return m, c


graphs = st.integers(min_value=2, max_value=40).flatmap(
    lambda n: st.tuples(st.just(n), st.lists(
        st.tuples(st.integers(0, n - 1), st.integers(0, n - 1)), min_size=0, max_size=4 * n)))


@settings(max_examples=150, deadline=None)
@given(graphs)
def test_level_invariants_and_brute_force(g):
    n, pairs = g
    xadj, adj = csr_from_pairs(n, pairs)
    A = dense_from_csr(xadj, adj)
    deg = A.sum(1)
    nnz = int(deg.sum())
    m, nc = O.coarsen_map(xadj, adj)
    ref, refc = dense_reference_map(A)
    assert m.tolist() == ref.tolist() and nc == refc
    # every vertex lands in exactly one cluster id in [0, nc), every id is used
    assert m.min() >= 0 and m.max() == nc - 1 and len(set(m.tolist())) == nc
    # each cluster is a star: one hub, every other member adjacent to it
    big = deg * n > nnz
    for c in range(nc):
        members = np.nonzero(m == c)[0]
        hubs = [h for h in members if all(A[h, u] for u in members if u != h)]
        assert hubs, "cluster is not a star"
        assert big[members].sum() <= 1  # two above-average-degree vertices never merge
    # quotient graph = P^T A P with the diagonal removed
    P = np.zeros((n, nc), dtype=np.int64)
    P[np.arange(n), m] = 1
    Q = P.T @ A @ P
    np.fill_diagonal(Q, 0)
    xo, ao, mo = O.coarsen_graph(xadj, adj, m, nc)
    Qo = np.zeros_like(Q)
    for a in range(nc):
        row = ao[xo[a]:xo[a + 1]]
        assert np.all(np.diff(row) > 0) and a not in row  # sorted, deduped, loop-free
        Qo[a, row] = mo[xo[a]:xo[a + 1]]
    assert np.array_equal(Q, Qo)
    assert np.array_equal(Qo, Qo.T)
    # weight conservation: merged + internal = total
    internal = sum(int(A[np.ix_(m == c, m == c)].sum()) for c in range(nc))
    assert int(mo.sum()) + internal == nnz


def test_hierarchy_stop_rules_and_weight_conservation():
    import graphgen
    edges = graphgen.rmat(11, 1 << 14, seed=3)
    csr = graphgen.to_csr(1 << 11, edges)
    xadj, adj = csr.xadj.numpy().astype(np.int64), csr.adj.numpy()
    graphs, maps, mults = O.coarsen(xadj, adj, threshold=100, min_shrink=1.0)
    sizes = [g[0].size - 1 for g in graphs]
    assert len(maps) == len(graphs) - 1 and len(graphs) >= 3
    # sizes fall strictly until either the threshold is passed or nothing merges any
    # more (isolated vertices can never merge; a level that would repeat the last is dropped)
    assert all(a > b for a, b in zip(sizes, sizes[1:]))
    assert sizes[-2] > 100  # the loop only builds from graphs above the threshold
    if sizes[-1] > 100:
        assert O.coarsen_map(*graphs[-1])[1] == sizes[-1]  # stopped because nothing merges
    tight, _, _ = O.coarsen(xadj, adj, threshold=100, min_shrink=0.8)
    tsz = [g[0].size - 1 for g in tight]
    assert tsz == sizes[:len(tsz)] and tsz[-1] > 0.8 * tsz[-2]
    assert all(b <= 0.8 * a for a, b in zip(tsz[:-2], tsz[1:-1]))
    for i, m in enumerate(maps):
        assert m.size == sizes[i] and m.max() == sizes[i + 1] - 1
        internal = sum(int(mults[i][p]) for v in range(sizes[i])
                       for p in range(graphs[i][0][v], graphs[i][0][v + 1])
                       if m[v] == m[graphs[i][1][p]])
        assert int(mults[i + 1].sum()) + internal == int(mults[i].sum())
    # a graph that cannot shrink (no edges) still terminates
    xe = np.zeros(301, dtype=np.int64)
    g2, m2, _ = O.coarsen(xe, np.zeros(0, dtype=np.int32), threshold=100, min_shrink=0.8)
    assert len(g2) == 1 and m2 == []
    # max_levels is a hard cap
    g3, _, _ = O.coarsen(xadj, adj, threshold=1, min_shrink=1.0, max_levels=2)
    assert len(g3) == 2


def test_projection_copies_super_vertex_rows():
    rng = np.random.default_rng(0)
    Mc = rng.normal(size=(5, 8)).astype(np.float32)
    m = np.array([0, 0, 4, 2, 2, 2, 1, 3, 0], dtype=np.int32)
    Mf = O.project(Mc, m)
    assert Mf.shape == (9, 8)
    for v, c in enumerate(m):
        assert np.array_equal(Mf[v], Mc[c])


def test_epoch_split():
    e = O.epoch_split(1000, 0.3, 5)
    # exact shares 82.58, 105.16, 150.32, 240.65, 421.29: finer levels get half the
    # geometric part of the next coarser one, plus the same uniform part
    assert e.tolist() == [84, 105, 150, 240, 421]
    assert e.sum() == 1000
    for p, D, tot in [(0.1, 8, 600), (0.5, 10, 1400), (0.3, 3, 200), (0.0, 6, 1000)]:
        e = O.epoch_split(tot, p, D)
        assert e.sum() == tot and e.min() >= 1
        assert all(a <= b for a, b in zip(e[1:], e[2:]))  # coarser levels get more
        geo = e[1:] - p * tot / D
        for a, b in zip(geo, geo[1:]):
            assert abs(b - 2 * a) <= 3  # halving, up to flooring
    assert O.epoch_split(1000, 1.0, 4).tolist() == [250, 250, 250, 250]
    assert O.epoch_split(7, 0.3, 1).tolist() == [7]
    with pytest.raises(ValueError):
        O.epoch_split(3, 0.3, 5)


def test_passes_per_epoch_closed_forms():
    """Sec. 4.3: an experiment epoch samples |E| sources, a pass of Alg. 3 |V|."""
    from tests.util import csr_from_pairs
    # complete graph K_n: |E| = n(n-1)/2, so ceil((n-1)/2) passes
    for n in (2, 3, 4, 7, 10, 11):
        x, a = csr_from_pairs(n, [(i, j) for i in range(n) for j in range(i)])
        assert O.passes_per_epoch(x, a) == max(1, -(-(n - 1) // 2))
    # a path has fewer edges than vertices, a cycle exactly as many: one pass
    x, a = csr_from_pairs(9, [(i, i + 1) for i in range(8)])
    assert O.passes_per_epoch(x, a) == 1
    x, a = csr_from_pairs(9, [(i, (i + 1) % 9) for i in range(9)])
    assert O.passes_per_epoch(x, a) == 1
    # no edges: still one pass
    x, a = csr_from_pairs(5, [])
    assert O.passes_per_epoch(x, a) == 1
    # in general: the smallest count that reaches |E| samples
    c = graphgen.to_csr(500, graphgen.er_gnm(500, 4321, 3))
    x, a = c.xadj.numpy(), c.adj.numpy()
    passes, edges = O.passes_per_epoch(x, a), a.size // 2
    assert passes * 500 >= edges > (passes - 1) * 500


def test_embed_with_edge_epochs_runs_enough_samples():
    c = graphgen.to_csr(1024, graphgen.rmat(10, 6000, 4))
    x, a = c.xadj.numpy(), c.adj.numpy()
    _, graphs, _, passes = O.embed(x, a, 8, 2, 6, 0.3, 0.05, 1, threshold=50, min_shrink=0.8,
                                   edge_epochs=True)
    e_i = O.epoch_split(6, 0.3, len(graphs))
    for (gx, ga), run, e in zip(graphs, passes, e_i):
        n, edges = gx.size - 1, ga.size // 2
        assert run % e == 0
        assert run * n >= e * edges and (run // e - 1) * n < max(edges, 1)
