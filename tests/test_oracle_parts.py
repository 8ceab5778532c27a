"""Pins for the oracle's large-graph rotation (Sec. 3.3, Alg. 5)."""
import numpy as np
import pytest

import graphgen
from oracle import gosh_oracle as O
from tests.util import csr_from_pairs


def test_pair_order_closed_form():
    assert O.pair_order(1) == [(0, 0)]
    assert O.pair_order(3) == [(0, 0), (1, 0), (1, 1), (2, 0), (2, 1), (2, 2)]
    for K in range(1, 12):
        order = O.pair_order(K)
        assert len(order) == K * (K + 1) // 2
        assert len(set(order)) == len(order)
        assert all(a >= b for a, b in order)  # every unordered pair exactly once
        # the printed recurrence
        assert order[0] == (0, 0)
        for (a0, b0), (a1, b1) in zip(order, order[1:]):
            assert (a1, b1) == ((a0, b0 + 1) if a0 > b0 else (a0 + 1, 0))


def test_rotation_count():
    assert O.rotations(200, 5, 4) == 10  # e_i / (B K)
    assert O.rotations(201, 5, 4) == 11
    assert O.rotations(3, 5, 4) == 1


@pytest.mark.parametrize("K,pa,pb", [(3, 1, 0), (3, 2, 2), (4, 3, 1), (5, 4, 0)])
def test_pair_stream_invariants(K, pa, pb):
    n, k, B, d = 50, 3, 4, 8
    edges = graphgen.er_gnm(n, 200, 5)
    csr = graphgen.to_csr(n, edges)
    xadj, adj = csr.xadj.numpy().astype(np.int64), csr.adj.numpy()
    M = O.init_embedding(n, d, 1, 0)
    stream = O.train_pair(xadj, adj, M, k, B, K, pa, pb, 0.0, 1, 0, 0, 2, want_stream=True)
    ps = -(-n // K)
    rng_of = lambda p: (min(n, p * ps), min(n, p * ps + ps))
    sides = [(pa, pb)] if pa == pb else [(pa, pb), (pb, pa)]
    pos = 0
    for own, other in sides:
        lo, hi = rng_of(own)
        olo, ohi = rng_of(other)
        for src in range(lo, hi):
            nb = [u for u in adj[xadj[src]:xadj[src + 1]] if olo <= u < ohi]
            for r in range(B):
                row = stream[pos:pos + k + 1]
                pos += k + 1
                if nb:
                    assert row[0] in nb  # positives: neighbours inside the partner part
                else:
                    assert row[0] == -1  # none there: no positive update for this pair
                assert all(olo <= x < ohi for x in row[1:])  # negatives: partner part
    assert pos == stream.size
    assert np.array_equal(M, O.init_embedding(n, d, 1, 0))  # lr = 0 moves nothing


def test_pair_touches_only_its_two_parts_and_replays_as_updates():
    n, k, B, d, K = 40, 2, 3, 8, 4
    xadj, adj = csr_from_pairs(n, [(i, (i * 7 + 3) % n) for i in range(n)] +
                               [(i, (i + 1) % n) for i in range(n)])
    M0 = O.init_embedding(n, d, 2, 0) * 20
    M = M0.copy()
    stream = O.train_pair(xadj, adj, M, k, B, K, 2, 1, 0.2, 9, 3, 0, 4, want_stream=True)
    ps = n // K
    untouched = np.r_[0:ps, 3 * ps:n]
    assert np.array_equal(M[untouched], M0[untouched])
    assert not np.array_equal(M[ps:3 * ps], M0[ps:3 * ps])
    R = M0.copy()
    pos = 0
    for own in (2, 1):
        for src in range(own * ps, own * ps + ps):
            for r in range(B):
                for j in range(k + 1):
                    v = int(stream[pos]); pos += 1
                    if v < 0 or v == src:
                        continue
                    O.update(R[src], R[v], 1 if j == 0 else 0, 0.2)
    assert np.array_equal(R, M)


def test_parts_training_separates_two_cliques():
    size = 12
    edges = graphgen.two_cliques(size, bridges=1)
    csr = graphgen.to_csr(2 * size, edges)
    xadj, adj = csr.xadj.numpy().astype(np.int64), csr.adj.numpy()
    M = O.init_embedding(2 * size, 16, 1, 0)
    O.train_parts(xadj, adj, M, 3, 300, 0.05, 1, 0, K=3, B=5)
    G = M.astype(np.float64) @ M.T.astype(np.float64)
    intra = (G[:size, :size].sum() - np.trace(G[:size, :size])) / (size * (size - 1))
    inter = G[:size, size:].mean()
    assert intra > inter + 0.5, (intra, inter)


def _loads_with_optimal_cache(order, slots):
    """Part loads a cache of `slots` parts needs for the visiting order `order` when it
    evicts the part whose next use is farthest (brute force, independent of the library)."""
    resident, loads = set(), 0
    for t, pair in enumerate(order):
        for p in set(pair):
            if p in resident:
                continue
            loads += 1
            if len(resident) >= slots:
                def next_use(q):
                    for u in range(t, len(order)):
                        if q in order[u]:
                            return u
                    return len(order)
                victims = [q for q in resident if q not in pair]
                resident.remove(max(victims, key=next_use))
            resident.add(p)
    return loads


def test_blocked_pair_order():
    """The blocked order (not the paper's): every pair once, the paper's order when one block
    holds all parts, the hand-written sequence for K = 5, R = 2, and fewer part loads than
    the paper's order on a device with R + 2 slots."""
    assert O.pair_order_blocked(5, 2) == [(0, 0), (1, 0), (1, 1), (2, 0), (2, 1), (3, 0), (3, 1), (4, 0),
                                          (4, 1), (2, 2), (3, 2), (3, 3), (4, 2), (4, 3), (4, 4)]
    assert O.pair_order_blocked(4, 1) == [(0, 0), (1, 0), (2, 0), (3, 0), (1, 1), (2, 1), (3, 1), (2, 2),
                                          (3, 2), (3, 3)]
    for K in range(1, 12):
        assert O.pair_order_blocked(K, K) == O.pair_order(K) == O.pair_order_blocked(K, K + 3)
        for R in range(1, K + 1):
            order = O.pair_order_blocked(K, R)
            assert sorted(order) == sorted((a, b) for a in range(K) for b in range(a + 1))
            assert all(a >= b for a, b in order)
    for K, R in [(13, 2), (17, 2), (21, 3), (9, 1)]:
        blocked, paper = O.pair_order_blocked(K, R), O.pair_order(K)
        starts = range(0, K, R)
        closed_form = sum(min(R, K - s) + max(0, K - (s + R)) for s in starts)
        # the closed form is what "keep the block, stream the rest" needs; an optimal cache can
        # also carry a few parts over from one block to the next
        loads = _loads_with_optimal_cache(blocked, R + 2)
        assert K <= loads <= closed_form
        if R > 1:
            assert loads < 0.75 * _loads_with_optimal_cache(paper, R + 2)
    assert O.blocked_block_size(3, 13) == 1 and O.blocked_block_size(5, 21) == 3
    assert O.blocked_block_size(4, 2) == 1


def test_blocked_rotation_differs_only_in_order():
    """With one block the blocked rotation is the paper's, bit for bit; with small blocks it
    applies the same multiset of updates in another order (same sample ids per pair)."""
    n = 60
    c = graphgen.to_csr(n, graphgen.er_gnm(n, 300, 5))
    xadj, adj = c.xadj.numpy().astype(np.int64), c.adj.numpy()
    a = O.init_embedding(n, 8, 2, 0)
    b, c2 = a.copy(), a.copy()
    O.train_parts(xadj, adj, a, 2, 40, 0.05, 2, 0, 4, 5)
    O.train_parts(xadj, adj, b, 2, 40, 0.05, 2, 0, 4, 5, block=4)
    O.train_parts(xadj, adj, c2, 2, 40, 0.05, 2, 0, 4, 5, block=2)
    assert np.array_equal(a, b)
    assert not np.array_equal(a, c2) and np.isfinite(c2).all()
