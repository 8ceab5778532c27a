"""Pins for the oracle's single update (Alg. 1), schedule and epoch (Alg. 3)."""
import math
import os

import numpy as np
import pytest

import graphgen
from oracle import gosh_oracle as O
from tests.util import csr_from_pairs

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _examples():
    rows = []
    for line in open(os.path.join(GOLD, "update_examples.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        f = [float(x) for x in line.split()]
        rows.append((int(f[0]), f[1], f[2:4], f[4:6], f[6:8], f[8:10]))
    return rows


@pytest.mark.parametrize("b,lr,eu,ev,eu2,ev2", _examples())
def test_hand_worked_updates(b, lr, eu, ev, eu2, ev2):
    u = np.array(eu, dtype=np.float32)
    v = np.array(ev, dtype=np.float32)
    O.update(u, v, b, lr)
    np.testing.assert_allclose(u, eu2, rtol=2e-7, atol=1e-8)
    np.testing.assert_allclose(v, ev2, rtol=2e-7, atol=1e-8)


def test_sample_row_sees_updated_source_row():
    """The third line of Alg. 1 runs after the second: e_v' = e_v + g * e_u'."""
    u = np.array([0.5, -0.25], dtype=np.float32)
    v = np.array([0.25, 0.5], dtype=np.float32)
    O.update(u, v, 1, 0.1)
    simultaneous = np.array([0.275, 0.4875])
    sequential = np.array([0.275625, 0.48875])
    assert np.abs(v - sequential).max() < 1e-7
    assert np.abs(v - simultaneous).max() > 5e-4


@pytest.mark.parametrize("b", [0, 1])
def test_source_step_is_gradient_of_log_likelihood(b):
    """score * e_v = lr * d/d e_u [ b ln s(x) + (1-b) ln(1 - s(x)) ], x = e_u . e_v."""
    rng = np.random.default_rng(4)
    d, lr = 16, 0.05
    eu = rng.normal(size=d).astype(np.float32) * 0.3
    ev = rng.normal(size=d).astype(np.float32) * 0.3

    def loglik(a):
        x = float(np.dot(a, ev.astype(np.float64)))
        s = 1.0 / (1.0 + math.exp(-x))
        return b * math.log(s) + (1 - b) * math.log(1.0 - s)

    grad = np.zeros(d)
    h = 1e-6
    for c in range(d):
        p = eu.astype(np.float64).copy()
        m = p.copy()
        p[c] += h
        m[c] -= h
        grad[c] = (loglik(p) - loglik(m)) / (2 * h)
    u, v = eu.copy(), ev.copy()
    O.update(u, v, b, lr)
    np.testing.assert_allclose(u.astype(np.float64) - eu, lr * grad, rtol=1e-4, atol=2e-8)
    # and the sample row moves along the *new* source row by the same score
    score = (u.astype(np.float64) - eu)[0] / ev[0]
    np.testing.assert_allclose(v.astype(np.float64) - ev, score * u, rtol=1e-4, atol=2e-8)


def test_update_special_cases():
    rng = np.random.default_rng(5)
    eu = rng.normal(size=8).astype(np.float32)
    ev = rng.normal(size=8).astype(np.float32)
    u, v = eu.copy(), ev.copy()
    O.update(u, v, 1, 0.0)  # lr = 0: nothing moves
    assert np.array_equal(u, eu) and np.array_equal(v, ev)
    # saturated positive: sigmoid -> 1, score -> 0
    u = np.full(8, 3.0, dtype=np.float32)
    v = np.full(8, 3.0, dtype=np.float32)
    O.update(u, v, 1, 0.5)
    assert np.abs(u - 3.0).max() < 1e-6
    # saturated negative with the wrong sign of x: score -> -lr
    u = np.full(8, 3.0, dtype=np.float32)
    v = np.full(8, 3.0, dtype=np.float32)
    O.update(u, v, 0, 0.5)
    np.testing.assert_allclose(u, 3.0 - 0.5 * 3.0, rtol=1e-6)
    # a positive update raises the dot product, a negative one lowers it
    for b, sign in ((1, 1.0), (0, -1.0)):
        u, v = eu.copy() * 0.1, ev.copy() * 0.1
        before = float(np.dot(u, v))
        O.update(u, v, b, 0.1)
        assert sign * (float(np.dot(u, v)) - before) > 0


def test_learning_rate_schedule_closed_form():
    lr0 = 0.045
    assert O.lr(lr0, 0, 600) == pytest.approx(lr0, rel=1e-7)
    assert O.lr(lr0, 599, 600) == pytest.approx(lr0 / 600, rel=1e-6)
    assert O.lr(lr0, 300, 600) == pytest.approx(lr0 / 2, rel=1e-7)
    # the floor only binds for very long runs
    assert O.lr(1.0, 99999, 100000) == pytest.approx(1e-4, rel=1e-6)
    assert O.lr(1.0, 99990, 100000) == pytest.approx(1e-4, rel=1e-6)
    assert O.lr(1.0, 50000, 100000) == pytest.approx(0.5, rel=1e-7)
    vals = [O.lr(lr0, j, 100) for j in range(100)]
    assert all(a > b for a, b in zip(vals, vals[1:]))


def test_single_edge_epoch_by_hand():
    """Graph 0-1, no negatives: the epoch is update(0 -> 1, b=1) then update(1 -> 0, b=1)
    with the rows of the hand-worked example (orthogonal rows, lr = 0.1)."""
    xadj, adj = csr_from_pairs(2, [(0, 1)])
    M = np.array([[0.5, -0.25], [0.25, 0.5]], dtype=np.float32)
    O.train_epoch(xadj, adj, M, 0, 0.1, seed=3, epoch=0, level=0)
    # after source 0: rows (0.5125, -0.225), (0.275625, 0.48875)   [golden case 1]
    # source 1 then updates itself first, and row 0 with its new value:
    a = np.array([0.275625, 0.48875])
    c = np.array([0.5125, -0.225])
    x = float(a @ c)
    g = 0.1 * (1.0 - 1.0 / (1.0 + math.exp(-x)))
    a2 = a + g * c
    c2 = c + g * a2
    np.testing.assert_allclose(M[1], a2, rtol=3e-7)
    np.testing.assert_allclose(M[0], c2, rtol=3e-7)


def test_degenerate_samples():
    # one vertex, no edges: positive is -1, every negative is the source itself
    xadj, adj = csr_from_pairs(1, [])
    M = np.array([[0.3, -0.2, 0.1, 0.4]], dtype=np.float32)
    keep = M.copy()
    s = O.sample_epoch(xadj, adj, 3, 1, 0, 0)
    assert s.tolist() == [[-1, 0, 0, 0]]
    O.train_epoch(xadj, adj, M, 3, 0.5, 1, 0, 0)
    assert np.array_equal(M, keep)
    # isolated vertex in a bigger graph: moves only through negative updates
    n = 6
    xadj, adj = csr_from_pairs(n, [(0, 1), (1, 2), (2, 3), (3, 4)])
    M0 = O.init_embedding(n, 8, 2, 0) * 50
    M = M0.copy()
    O.train_epoch(xadj, adj, M, 0, 0.5, 1, 0, 0)  # no negatives at all
    assert np.array_equal(M[5], M0[5])
    assert not np.array_equal(M[:5], M0[:5])


def test_epoch_is_the_updates_of_its_stream_in_order():
    """Invariant of Alg. 3: replaying the recorded (src, sample, label) stream with
    Alg. 1, sources ascending, reproduces the epoch -- including repeated samples."""
    n, d, k = 24, 8, 5
    pairs = [(i, (i + 1) % n) for i in range(n)] + [(0, 9), (3, 17), (5, 12)]
    xadj, adj = csr_from_pairs(n, pairs)
    M0 = O.init_embedding(n, d, 7, 1) * 30
    stream = O.sample_epoch(xadj, adj, k, 7, 4, 1)
    # the tiny n makes repeated samples and negative == src certain to occur
    assert any(len(set(r.tolist())) < k + 1 for r in stream)
    assert any(src in r[1:].tolist() for src, r in enumerate(stream))
    A = M0.copy()
    O.train_epoch(xadj, adj, A, k, 0.3, 7, 4, 1)
    B = M0.copy()
    for src in range(n):
        for j in range(k + 1):
            v = int(stream[src, j])
            if v < 0 or v == src:
                continue
            O.update(B[src], B[v], 1 if j == 0 else 0, 0.3)
    assert np.array_equal(A, B)


def test_init_embedding_distribution():
    n, d = 512, 32
    M = O.init_embedding(n, d, 1, 0)
    assert M.dtype == np.float32 and M.shape == (n, d)
    assert M.min() >= -0.5 / d and M.max() < 0.5 / d
    u = (M.astype(np.float64) * d + 0.5).ravel()
    import scipy.stats
    assert scipy.stats.kstest(u, "uniform").pvalue > 1e-3
    assert abs(np.corrcoef(M[:, 0], M[:, 1])[0, 1]) < 0.15
    assert not np.array_equal(M, O.init_embedding(n, d, 2, 0))
    assert not np.array_equal(M, O.init_embedding(n, d, 1, 1))
    assert len(np.unique(M)) > 0.9 * 0.5 * M.size  # 24-bit grid, few collisions


def test_training_separates_two_cliques():
    """End-to-end sign check: after training, vertices of the same clique have a larger
    dot product than vertices of different cliques."""
    import graphgen
    size = 12
    edges = graphgen.two_cliques(size, bridges=1)
    csr = graphgen.to_csr(2 * size, edges)
    xadj, adj = csr.xadj.numpy().astype(np.int64), csr.adj.numpy()
    M = O.init_embedding(2 * size, 16, 1, 0)
    O.train_level(xadj, adj, M, 3, 0.05, 300, 1, 0)
    G = M.astype(np.float64) @ M.T.astype(np.float64)
    intra = (G[:size, :size].sum() - np.trace(G[:size, :size])) / (size * (size - 1))
    inter = G[:size, size:].mean()
    assert intra > inter + 0.5, (intra, inter)


def test_hogwild_slice_is_the_sequential_slice_on_one_thread_and_sane_on_many():
    """The multi-threaded slice exists for timing the paper's multi-core CPU baseline: at
    one thread it must be the sequential slice bit for bit; at several it must still
    learn (two cliques separate) although its values depend on the interleaving."""
    n, edges = 64, graphgen.two_cliques(32)
    c = graphgen.to_csr(n, edges)
    xadj, adj = c.xadj.numpy().astype(np.int64), c.adj.numpy()
    a = O.init_embedding(n, 16, 3, 0)
    b = a.copy()
    O.train_sources(xadj, adj, a, 3, 0.05, 3, 0, 0, 5, 40)
    O.train_sources_hogwild(xadj, adj, b, 3, 0.05, 3, 0, 0, 5, 40, 1)
    assert np.array_equal(a, b)
    M = O.init_embedding(n, 16, 3, 0)
    for j in range(300):
        O.train_sources_hogwild(xadj, adj, M, 3, float(O.lr(0.05, j, 300)), 3, j, 0, 0, n, 4)
    assert np.isfinite(M).all()
    inside = np.mean([M[i] @ M[j] for i in range(0, 32, 3) for j in range(1, 32, 5) if i != j])
    across = np.mean([M[i] @ M[32 + j] for i in range(0, 32, 3) for j in range(1, 32, 5)])
    assert inside > across + 0.5
