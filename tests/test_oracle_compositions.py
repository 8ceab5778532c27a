"""Pins for the oracle's compositions: the epoch loop of Alg. 3, the rotation loop and the
sampling rule of Alg. 5, the initial matrix, and the level loop of Alg. 2 with and without
its "fits into the GPU" branch.  Each composition is rebuilt here from pieces that have
pins of their own (Philox against ATen's engine, the multiply-high index, single updates
of Alg. 1, the coarsening maps, the projection) plus numbers written out by hand, so that
a slip in a loop index, a counter word or a schedule argument shows up as a bit difference.
"""
import numpy as np
import pytest
import scipy.stats

import graphgen
from oracle import gosh_oracle as O
from tests.util import csr_from_pairs


def f32(x):
    return float(np.float32(x))


def lr_by_hand(lr0, j, e):
    """lr * max(1 - j / e, 1e-4) of the fp32 value of lr0, in fp64, rounded once (Sec. 3)."""
    return f32(f32(lr0) * max(1.0 - j / e, 1e-4))


def replay_alg3_epoch(xadj, adj, M, k, lr, seed, epoch, level):
    """One epoch of Alg. 3 as single updates of Alg. 1 over the recorded sample stream."""
    stream = O.sample_epoch(xadj, adj, k, seed, epoch, level)
    for src in range(M.shape[0]):
        for j in range(k + 1):
            v = int(stream[src, j])
            if v < 0 or v == src:
                continue
            O.update(M[src], M[v], 1 if j == 0 else 0, lr)


def ring_with_chords(n):
    return csr_from_pairs(n, [(i, (i + 1) % n) for i in range(n)] + [(i, (i * 7 + 3) % n) for i in range(0, n, 3)])


def test_train_level_is_the_epoch_loop_of_alg3():
    """Alg. 3: for j = 0..e_i-1, one epoch with learning rate lr*max(1 - j/e_i, 1e-4), the
    draws of epoch j keyed by j and by the level."""
    n, d, k, e, lr0, seed, level = 30, 8, 2, 7, 0.05, 11, 3
    xadj, adj = ring_with_chords(n)
    M0 = O.init_embedding(n, d, seed, level) * np.float32(25)
    got = M0.copy()
    O.train_level(xadj, adj, got, k, lr0, e, seed, level)
    want = M0.copy()
    for j in range(e):
        replay_alg3_epoch(xadj, adj, want, k, lr_by_hand(lr0, j, e), seed, j, level)
    assert np.array_equal(got, want)
    # the pieces that a slip would change do change the result
    for bad in ("epoch word", "level word", "schedule length", "schedule index"):
        other = M0.copy()
        for j in range(e):
            lr = lr_by_hand(lr0, j + (bad == "schedule index"), e + (bad == "schedule length"))
            replay_alg3_epoch(xadj, adj, other, k, lr, seed, j + (bad == "epoch word"),
                              level + (bad == "level word"))
        assert not np.array_equal(other, want), bad


def pair_stream_by_hand(xadj, adj, k, B, K, pa, pb, seed, rotation, level, pair_index):
    """The sample ids of one visit of the pair (pa, pb), Sec. 3.3: for every vertex of part
    pa, B rounds of (one positive among its neighbours inside part pb, k negatives uniform in
    part pb), then the same with the roles swapped.  Draw (side, round, j) of a source is
    Philox counter (src, side*B*(k+1) + round*(k+1) + j, rotation, level | (pair_index+1) << 8)."""
    n = xadj.size - 1
    ps = -(-n // K)
    bounds = lambda p: (min(n, p * ps), min(n, p * ps + ps))
    out = []
    for side, (own, other) in enumerate([(pa, pb)] if pa == pb else [(pa, pb), (pb, pa)]):
        lo, hi = bounds(own)
        olo, ohi = bounds(other)
        for src in range(lo, hi):
            inside = [int(u) for u in adj[xadj[src]:xadj[src + 1]] if olo <= u < ohi]
            for rnd in range(B):
                for j in range(k + 1):
                    slot = side * B * (k + 1) + rnd * (k + 1) + j
                    r = O.draw(seed, src, slot, rotation, (level & 255) | ((pair_index + 1) << 8))
                    if j == 0:
                        v = inside[O.bounded(r, len(inside))] if inside else -1
                    else:
                        v = olo + O.bounded(r, ohi - olo) if ohi > olo else -1
                    out.append((src, v, 1 if j == 0 else 0))
    return out


@pytest.mark.parametrize("K,pa,pb", [(3, 1, 0), (3, 2, 2), (4, 3, 1), (7, 6, 2)])
def test_pair_visit_stream_and_updates_by_hand(K, pa, pb):
    n, d, k, B = 45, 8, 2, 3
    xadj, adj = csr_from_pairs(n, [(i, (i * 5 + 2) % n) for i in range(n)] + [(i, (i + 1) % n) for i in range(n)] +
                               [(i, (i + 11) % n) for i in range(0, n, 2)])
    seed, rotation, level, q = 2 ** 40 + 5, 6, 258, 4  # only the low 8 bits of the level reach the counter
    M0 = O.init_embedding(n, d, 3, 0) * np.float32(20)
    got = M0.copy()
    stream = O.train_pair(xadj, adj, got, k, B, K, pa, pb, 0.2, seed, rotation, level, q, want_stream=True)
    by_hand = pair_stream_by_hand(xadj, adj, k, B, K, pa, pb, seed, rotation, level, q)
    assert stream.tolist() == [v for _, v, _ in by_hand]
    assert any(v >= 0 and b == 1 for _, v, b in by_hand)
    want = M0.copy()
    for src, v, b in by_hand:
        if v >= 0 and v != src:
            O.update(want[src], want[v], b, 0.2)
    assert np.array_equal(got, want)
    # level 258 and level 2 share their low 8 bits, another pair index or rotation does not
    same = O.train_pair(xadj, adj, M0.copy(), k, B, K, pa, pb, 0.0, seed, rotation, 2, q, want_stream=True)
    assert np.array_equal(same, stream)
    for kw in (dict(rotation=rotation + 1), dict(pair_index=q + 1), dict(level=level + 1)):
        args = dict(rotation=rotation, level=level, pair_index=q)
        args.update(kw)
        other = O.train_pair(xadj, adj, M0.copy(), k, B, K, pa, pb, 0.0, seed, args["rotation"], args["level"],
                             args["pair_index"], want_stream=True)
        assert not np.array_equal(other, stream), kw


def test_positive_inside_the_partner_part_is_uniform():
    """Sec. 3.3: the positive of a vertex for a pair is a uniform member of its neighbours
    inside the partner part -- chi-square over six candidates (and over three on the
    diagonal pair), with neighbours outside the part never drawn."""
    n, K = 20, 2  # parts 0..9 and 10..19
    xadj, adj = csr_from_pairs(n, [(0, u) for u in (1, 2, 3, 10, 11, 12, 13, 14, 15)] + [(5, 19), (7, 8)])
    M = np.zeros((n, 4), dtype=np.float32)
    cross = np.zeros(n)
    diag = np.zeros(n)
    k, B = 1, 2
    for rotation in range(1500):
        s = O.train_pair(xadj, adj, M, k, B, K, 1, 0, 0.0, 9, rotation, 0, 1, want_stream=True)
        side1 = s[10 * B * (k + 1):]          # sources 0..9 follow the ten sources of part 1
        for rnd in range(B):
            cross[side1[rnd * (k + 1)]] += 1  # source 0, positive of round rnd
        s = O.train_pair(xadj, adj, M, k, B, K, 0, 0, 0.0, 9, rotation, 0, 0, want_stream=True)
        for rnd in range(B):
            diag[s[rnd * (k + 1)]] += 1
    assert cross.sum() == 3000 and cross[10:16].sum() == 3000 and cross[:10].sum() == 0
    assert scipy.stats.chisquare(cross[10:16]).pvalue > 1e-3
    assert diag.sum() == 3000 and diag[1:4].sum() == 3000
    assert scipy.stats.chisquare(diag[1:4]).pvalue > 1e-3
    assert not M.any()


@pytest.mark.parametrize("block", [0, 2])
def test_train_parts_is_the_rotation_loop_of_alg5(block):
    """Alg. 5: ceil(e_i / (B*K)) rotations; in rotation r every pair of the visiting order
    once, with lr*max(1 - r/rotations, 1e-4), the draws keyed by r and by the pair's position
    q in the order.  K = 3 in the paper's order (Sec. 3.3.1) written out."""
    n, d, k, B, K, e, lr0, seed, level = 33, 8, 2, 2, 3, 13, 0.05, 21, 1
    xadj, adj = ring_with_chords(n)
    order = {0: [(0, 0), (1, 0), (1, 1), (2, 0), (2, 1), (2, 2)],
             2: [(0, 0), (1, 0), (1, 1), (2, 0), (2, 1), (2, 2)]}[block]  # blocks {0,1},{2}: same sequence at K = 3
    if block:
        assert O.pair_order_blocked(K, block) == order
    rotations = 3  # ceil(13 / 6)
    M0 = O.init_embedding(n, d, seed, level) * np.float32(25)
    got = M0.copy()
    O.train_parts(xadj, adj, got, k, e, lr0, seed, level, K, B, block=block)
    want = M0.copy()
    for r in range(rotations):
        for q, (a, b) in enumerate(order):
            for src, v, label in pair_stream_by_hand(xadj, adj, k, B, K, a, b, seed, r, level, q):
                if v >= 0 and v != src:
                    O.update(want[src], want[v], label, lr_by_hand(lr0, r, rotations))
    assert np.array_equal(got, want)
    for bad in ("rotation word", "pair word", "schedule index", "schedule length"):
        other = M0.copy()
        for r in range(rotations):
            lr = lr_by_hand(lr0, r + (bad == "schedule index"), rotations + (bad == "schedule length"))
            for q, (a, b) in enumerate(order):
                for src, v, label in pair_stream_by_hand(xadj, adj, k, B, K, a, b, seed, r + (bad == "rotation word"),
                                                         level, q + (bad == "pair word")):
                    if v >= 0 and v != src:
                        O.update(other[src], other[v], label, lr)
        assert not np.array_equal(other, want), bad


def test_blocked_rotation_visits_its_own_order():
    """K = 4 in blocks of 1 -- (0,0),(1,0),(2,0),(3,0),(1,1),... -- replayed pair by pair."""
    n, d, k, B, K, e, lr0, seed, level = 32, 4, 1, 2, 4, 8, 0.1, 4, 0
    xadj, adj = ring_with_chords(n)
    order = [(0, 0), (1, 0), (2, 0), (3, 0), (1, 1), (2, 1), (3, 1), (2, 2), (3, 2), (3, 3)]
    M0 = O.init_embedding(n, d, seed, level) * np.float32(25)
    got = M0.copy()
    O.train_parts(xadj, adj, got, k, e, lr0, seed, level, K, B, block=1)
    want = M0.copy()
    for q, (a, b) in enumerate(order):  # 8 epochs = one rotation of 2 * 4
        O.train_pair(xadj, adj, want, k, B, K, a, b, lr_by_hand(lr0, 0, 1), seed, 0, level, q)
    assert np.array_equal(got, want)


def test_init_rows_entries_by_hand(aten_philox):
    """Entry (v, c) of the initial matrix of a level: word c % 4 of the Philox block with
    counter (v, c / 4, 0xFFFFFFFF, level), its top 24 bits as a fraction in [0, 1), centred
    and divided by d -- worked out here from the words of an independent Philox."""
    d, seed, level, first = 12, 2 ** 33 + 7, 5, 1000
    rows = O.init_rows(first, 3, d, seed, level)
    cases = [(0, 0), (0, 3), (1, 4), (2, 11), (2, 6)]
    blocks = aten_philox([(seed, 0xFFFFFFFF | (level << 32), (first + r) | ((c // 4) << 32)) for r, c in cases])
    for (r, c), words in zip(cases, blocks):
        w = words[c % 4]
        want = np.float32(((w >> 8) / 16777216.0 - 0.5) / d)
        assert rows[r, c] == want, (r, c)
        assert rows[r, c] != np.float32(((w >> 9) / 16777216.0 - 0.5) / d) or (w >> 8) == 0
    # a slice is a window of the whole matrix, and the range is the full [-0.5/d, 0.5/d)
    whole = O.init_embedding(first + 3, d, seed, level)
    assert np.array_equal(whole[first:], rows)
    big = O.init_embedding(4096, 8, 1, 0).astype(np.float64) * 8
    assert big.min() < -0.499 and big.max() > 0.499 and big.min() >= -0.5 and big.max() < 0.5


def toy_hierarchy():
    n = 400
    c = graphgen.to_csr(n, graphgen.chung_lu(n, 2400, 3))
    xadj, adj = c.xadj.numpy().astype(np.int64), c.adj.numpy()
    graphs, maps, _ = O.coarsen(xadj, adj, threshold=40, min_shrink=1.0, max_levels=3)
    assert len(graphs) == 3, [g[0].size - 1 for g in graphs]
    return xadj, adj, graphs, maps


def test_embed_is_the_level_loop_of_alg2():
    """Alg. 2 on three levels: initialise M_2 with the level word 2, train levels 2, 1, 0 with
    their own level word and epoch budget, project after levels 2 and 1.  Budget written out:
    e = 20, p = 0.5, D = 3: 10/3 + 10 * 2^i / 7 = 9.05, 6.19 -> 9, 6, and level 0 the rest, 5."""
    xadj, adj, graphs, maps = toy_hierarchy()
    d, k, lr0, seed = 8, 2, 0.05, 7
    got, graphs2, maps2, e_i = O.embed(xadj, adj, d, k, 20, 0.5, lr0, seed, threshold=40, min_shrink=1.0,
                                       max_levels=3)
    assert e_i.tolist() == [5, 6, 9]
    assert all(np.array_equal(a, b) for a, b in zip(maps, maps2))
    M = O.init_rows(0, graphs[2][0].size - 1, d, seed, 2)
    for level, e in ((2, 9), (1, 6), (0, 5)):
        x, a = graphs[level]
        for j in range(e):
            replay_alg3_epoch(x, a, M, k, lr_by_hand(lr0, j, e), seed, j, level)
        if level > 0:
            M = np.ascontiguousarray(M[maps[level - 1]])
    assert np.array_equal(got, M)
    assert got.shape == (400, d)


def test_embed_with_given_part_counts_runs_alg5_on_those_levels():
    xadj, adj, graphs, maps = toy_hierarchy()
    d, k, lr0, seed = 8, 2, 0.05, 7
    got, *_ = O.embed(xadj, adj, d, k, 20, 0.5, lr0, seed, threshold=40, min_shrink=1.0, max_levels=3,
                      parts_K=[2, 0, 1])
    M = O.init_rows(0, graphs[2][0].size - 1, d, seed, 2)
    O.train_parts(graphs[2][0], graphs[2][1], M, k, 9, lr0, seed, 2, 1, 5)
    M = O.project(M, maps[1])
    O.train_level(graphs[1][0], graphs[1][1], M, k, lr0, 6, seed, 1)
    M = O.project(M, maps[0])
    O.train_parts(graphs[0][0], graphs[0][1], M, k, 5, lr0, seed, 0, 2, 5)
    assert np.array_equal(got, M)


def test_edge_epochs_multiply_the_passes():
    """Sec. 4.3 counts |E| sampled sources as an epoch: ceil(|E_i| / |V_i|) passes of Alg. 3
    each.  Path of 4 vertices: 3 edges, 4 vertices -> 1 pass; K_5: 10 edges, 5 vertices -> 2;
    star with 9 leaves plus a triangle among leaves: 12 edges, 10 vertices -> 2."""
    assert O.passes_per_epoch(*csr_from_pairs(4, [(0, 1), (1, 2), (2, 3)])) == 1
    assert O.passes_per_epoch(*csr_from_pairs(5, [(i, j) for i in range(5) for j in range(i)])) == 2
    star = [(0, i) for i in range(1, 10)] + [(1, 2), (2, 3), (1, 3)]
    assert O.passes_per_epoch(*csr_from_pairs(10, star)) == 2
    assert O.passes_per_epoch(*csr_from_pairs(3, [])) == 1


def test_parts_split_cases_by_hand():
    """Smallest K whose min(P, K) slots of ceil(n/K) rows, S pools of 2*ceil(n/K)*B ids and
    n bits (in 64-bit words) fit: n = 1000, d = 128 (512-byte rows), P = 3, S = 4, B = 5.
      K = 1: 1*1000*512 + 4*2*1000*5*4 + 128 = 672,128
      K = 2: 2* 500*512 + 4*2* 500*5*4 + 128 = 592,128
      K = 3: 3* 334*512 + 4*2* 334*5*4 + 128 = 566,592
      K = 4: 3* 250*512 + 4*2* 250*5*4 + 128 = 424,128
      K = 5: 3* 200*512 + 4*2* 200*5*4 + 128 = 339,328"""
    for budget, K in [(672128, 1), (672127, 2), (592128, 2), (592127, 3), (566592, 3), (566591, 4),
                      (424128, 4), (424127, 5), (10 ** 9, 1)]:
        assert O.parts_split(1000, 128, budget, 3, 4, 5) == K, budget
    assert O.parts_split(1000, 128, 424128, 2, 4, 5) == 3   # two slots only: 2*334*512 + 53,440 + 128
    with pytest.raises(ValueError):
        O.parts_split(10, 128, 100, 3, 4, 5)


def test_embed_budget_puts_the_levels_that_do_not_fit_through_alg5():
    """Alg. 2's "fits into the GPU" branch: graph (offsets + neighbours) plus matrix against
    the budget, level by level; the level that does not fit is split by parts_split and
    trained with Alg. 5, the others with Alg. 3."""
    xadj, adj, graphs, maps = toy_hierarchy()
    d, k, lr0, seed, P, S, B = 8, 2, 0.05, 7, 3, 4, 2
    n0, nnz0 = 400, adj.size
    level0_bytes = 401 * 4 + nnz0 * 4 + 400 * 8 * 4          # 32-bit offsets at level 0
    n1, nnz1 = graphs[1][0].size - 1, graphs[1][1].size
    level1_bytes = (n1 + 1) * 8 + nnz1 * 4 + n1 * 8 * 4      # coarse levels: 64-bit offsets
    assert level1_bytes < level0_bytes
    budget = level0_bytes - 1
    # parts for 400 rows of 32 bytes, P = 3, S = 4, B = 2, 7 bitmap words: need(K) by hand
    need = lambda K: min(P, K) * -(-n0 // K) * 32 + S * 2 * -(-n0 // K) * B * 4 + 56
    assert need(1) == 12800 + 25600 + 56  # slot: 400*32; pools: 4 pools * 2 sides * 400 * 2 rounds * 4 bytes
    assert need(2) == 12800 + 12800 + 56 and need(1) > budget >= need(2)
    K0 = next(K for K in range(1, 50) if need(K) <= budget)
    got, modes = O.embed_budget(xadj, adj, d, k, 20, 0.5, lr0, seed, budget, P, S, B, threshold=40,
                                min_shrink=1.0, max_levels=3)
    assert K0 == 2 and len(modes) == 3 and modes == [K0, 0, 0] and K0 == O.parts_split(n0, d, budget, P, S, B)
    M = O.init_rows(0, graphs[2][0].size - 1, d, seed, 2)
    O.train_level(graphs[2][0], graphs[2][1], M, k, lr0, 9, seed, 2)
    M = O.project(M, maps[1])
    O.train_level(graphs[1][0], graphs[1][1], M, k, lr0, 6, seed, 1)
    M = O.project(M, maps[0])
    O.train_parts(graphs[0][0], graphs[0][1], M, k, 5, lr0, seed, 0, K0, B)
    assert np.array_equal(got, M)
    # one byte more and level 0 fits: everything is Alg. 3
    _, modes = O.embed_budget(xadj, adj, d, k, 20, 0.5, lr0, seed, budget + 1, P, S, B, threshold=40,
                              min_shrink=1.0, max_levels=3)
    assert modes == [0, 0, 0]
    # with 64-bit offsets at level 0 it is 4 * 401 bytes larger
    _, modes = O.embed_budget(xadj, adj, d, k, 20, 0.5, lr0, seed, budget + 1, P, S, B, threshold=40,
                              min_shrink=1.0, max_levels=3, offsets64=True)
    assert modes[0] > 0
