"""The kernels as they are shipped and benchmarked, held to the sequential-order bar.

GOSH_FLAG_SEQUENTIAL | GOSH_FLAG_CONCURRENT_LAYOUT runs the concurrent template itself --
its lane-to-column layout (32-bit interleaved units for d > 64, 64-bit units for d <= 64,
128-bit units for d <= 64 when every row is written with plain stores),
its device-scope row accesses, the hot-row bitmap with the atomic-add and the plain-store
write paths, the source's own atomic delta, the forwarding inside a chunk of four samples --
on one lane group that walks the sources in ascending id.  Every address is then touched
by one lane in program order, so the result is the sequential one and is compared with the
oracle's epoch (Alg. 3 order, Alg. 1 per update) at 1e-5 relative, three epochs in a row.
"""
import sys

import numpy as np
import pytest
import torch

import graphgen
import paper_2008_12336_amd as G
from oracle import gosh_oracle as O
from tests.util import csr_from_pairs, rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = 1e-5
SEQ_LAYOUT = G.GOSH_FLAG_SEQUENTIAL | G.GOSH_FLAG_CONCURRENT_LAYOUT


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def hub_graph(n, m, seed):
    """Chung-Lu power law: a few vertices with hundreds of neighbours, most with a handful."""
    c = graphgen.to_csr(n, graphgen.chung_lu(n, m, seed))
    return c.xadj.numpy().astype(np.int64), c.adj.numpy()


@pytest.fixture
def hot_degree():
    """Sets the hot-row rule to 'degree >= value' for one test (the default rule would call
    every row of a graph this small hot)."""
    def set_(value):
        G.gosh_set_tuning(hot_min_degree=value)
    yield set_
    G.gosh_set_tuning()


def start_matrix(n, d, seed, scale):
    return (O.init_embedding(n, d, seed, 0).astype(np.float64) * d * scale).astype(np.float32)


def upload(n, xadj, adj, offsets64):
    xt = torch.from_numpy(np.asarray(xadj, dtype=np.int64 if offsets64 else np.int32)).to(DEV)
    at = torch.from_numpy(np.asarray(adj, dtype=np.int32)).to(DEV)
    return G.csr_view(n, xt, at), (xt, at)


MIX, ALL_ATOMIC, ALL_STORES = "mix", "atomic", "stores"

CASES = [
    # d, k, offsets64, scale, write paths
    (8, 3, False, 2.0, MIX),
    (16, 5, True, 1.5, MIX),
    (32, 3, False, 1.0, MIX),
    (64, 3, False, 0.8, MIX),
    (100, 4, False, 0.6, MIX),      # LPG = 32, last unit of the row masked
    (128, 3, True, 0.6, MIX),       # the benchmarked instantiation
    (128, 3, False, 0.6, ALL_ATOMIC),
    (128, 3, False, 0.6, ALL_STORES),
    (128, 9, False, 0.5, MIX),      # samples cross chunk boundaries: 10 = 4 + 4 + 2
    (256, 3, False, 0.4, MIX),
    (260, 1, False, 0.4, MIX),      # 64 lanes x 8 units, most of the last masked
    (512, 3, True, 0.3, MIX),
    (32, 3, False, 1.0, ALL_ATOMIC),
    (4, 15, False, 2.0, MIX),
    # store-only and all-atomic launches of the 128-bit units of d <= 64
    (32, 3, False, 1.0, ALL_STORES),
    (64, 5, True, 0.8, ALL_STORES),
    (8, 3, False, 2.0, ALL_STORES),
    (4, 9, False, 2.0, ALL_STORES),
    (36, 2, False, 1.0, ALL_STORES),
    (64, 3, False, 0.8, ALL_ATOMIC),
    (8, 5, True, 2.0, ALL_ATOMIC),
    (36, 4, False, 1.0, MIX),
]


@pytest.mark.parametrize("d,k,offsets64,scale,paths", CASES)
def test_shipped_kernel_in_sequential_order(d, k, offsets64, scale, paths, hot_degree):
    n = 3001
    xadj, adj = hub_graph(n, 20000, 3)
    deg = np.diff(xadj)
    min_degree = 12
    hot = deg >= min_degree
    assert 0.05 < hot.mean() < 0.6 and deg.max() > 100  # both kinds of row, real hubs
    say(f"[layout] d={d} k={k} offsets64={offsets64} paths={paths} hot rows {hot.mean():.2f}")
    flags = SEQ_LAYOUT | {MIX: 0, ALL_ATOMIC: G.GOSH_FLAG_ATOMIC_ADDS, ALL_STORES: G.GOSH_FLAG_PLAIN_STORES}[paths]
    hot_degree(min_degree)
    g, keep = upload(n, xadj, adj, offsets64)
    M0 = start_matrix(n, d, 5, scale)
    want = M0.copy()
    M = torch.from_numpy(M0).to(DEV)
    worst = 0.0
    for epoch in range(3):
        lr = G.gosh_lr(0.2, epoch, 3)
        if epoch == 0 and paths == MIX:
            # the epoch really takes both write paths, for samples and for sources
            stream = O.sample_epoch(xadj, adj, k, 77, epoch, 1)
            used = stream[stream >= 0]
            assert hot[used].any() and (~hot[used]).any()
        G.gosh_train_epoch(g, M, k, lr, 77, epoch, 1, flags)
        torch.cuda.synchronize()
        O.train_epoch(xadj, adj, want, k, lr, 77, epoch, 1)
        worst = max(worst, rel_err(M.cpu().numpy(), want))
        assert worst <= TOL, (epoch, worst)
    assert rel_err(M0, want) > 1e-3
    say(f"         worst relative error {worst:.2e}")


def test_layout_mode_on_tiny_and_degenerate_graphs(hot_degree):
    """Repeated samples inside a chunk (forwarded through registers, then added or stored),
    negatives equal to the source, isolated sources, a single vertex."""
    hot_degree(3)
    ring = csr_from_pairs(24, [(i, (i + 1) % 24) for i in range(24)] + [(0, 9), (3, 17), (0, 5), (0, 13)])
    for (xadj, adj), d, k in [(ring, 8, 15), (ring, 128, 7), (ring, 64, 6), (csr_from_pairs(1, []), 32, 3),
                              (csr_from_pairs(5, []), 16, 3), (csr_from_pairs(5, [(0, 1)]), 256, 5)]:
        n = xadj.size - 1
        g, keep = upload(n, xadj, adj, False)
        M0 = start_matrix(n, d, 6, 1.5)
        want = M0.copy()
        M = torch.from_numpy(M0).to(DEV)
        for epoch in range(3):
            G.gosh_train_epoch(g, M, k, 0.2, 5, epoch, 0, SEQ_LAYOUT)
            torch.cuda.synchronize()
            O.train_epoch(xadj, adj, want, k, 0.2, 5, epoch, 0)
            assert rel_err(M.cpu().numpy(), want) <= TOL, (n, d, k, epoch)


def test_layout_flag_alone_changes_nothing_and_the_default_rule_is_used_without_tuning():
    """Without GOSH_FLAG_SEQUENTIAL the flag has no effect; with it and the default tuning
    every row of a small graph is hot (all-atomic), which must still be the sequential result."""
    n, d, k = 2000, 128, 3
    xadj, adj = hub_graph(n, 12000, 9)
    g, keep = upload(n, xadj, adj, False)
    M0 = start_matrix(n, d, 2, 0.6)
    want = M0.copy()
    O.train_epoch(xadj, adj, want, k, 0.1, 4, 0, 0)
    M = torch.from_numpy(M0).to(DEV)
    G.gosh_train_epoch(g, M, k, 0.1, 4, 0, 0, SEQ_LAYOUT)
    torch.cuda.synchronize()
    assert rel_err(M.cpu().numpy(), want) <= TOL
    M = torch.from_numpy(M0).to(DEV)
    G.gosh_train_epoch(g, M, k, 0.0, 4, 0, 0, G.GOSH_FLAG_CONCURRENT_LAYOUT)  # concurrent, lr = 0
    torch.cuda.synchronize()
    assert np.array_equal(M.cpu().numpy(), M0)


@pytest.mark.parametrize("stores_only", [False, True])
@pytest.mark.parametrize("d,K,B,k", [(128, 3, 5, 3), (32, 4, 2, 3), (256, 2, 3, 2), (8, 5, 4, 5), (512, 9, 4, 9)])
def test_shipped_pair_kernel_in_sequential_order(d, K, B, k, stores_only, hot_degree):
    """The same for the pair kernel of Alg. 5 (rotation on a device-resident matrix and on a
    host matrix): concurrent layout and write paths, sequential order, against the oracle's
    rotation."""
    n, epochs = 1200, 2 * B * K
    xadj, adj = hub_graph(n, 9000, 8)
    hot_degree(10)
    say(f"[layout pair] d={d} K={K} B={B} k={k} stores_only={stores_only}")
    M0 = (O.init_embedding(n, d, 3, 0).astype(np.float64) * d * 0.8).astype(np.float32)
    want = M0.copy()
    O.train_parts(xadj, adj, want, k, epochs, 0.1, 7, 2, K, B)
    xt, at = torch.from_numpy(xadj), torch.from_numpy(adj)
    for where in ("device", "host"):
        M = torch.from_numpy(M0.copy()).to(DEV) if where == "device" else torch.from_numpy(M0.copy()).pin_memory()
        gx, ga = (xt.to(DEV), at.to(DEV)) if where == "device" else (xt, at)
        st = G.gosh_train_parts(n, gx, ga, M, k, epochs, 0.1, 7, level=2, force_K=K, B=B,
                                flags=SEQ_LAYOUT | (G.GOSH_FLAG_PLAIN_STORES if stores_only else 0))
        torch.cuda.synchronize()
        err = rel_err(M.cpu().numpy(), want)
        say(f"              {where}: err={err:.2e}")
        assert st["K"] == K and st["nonfinite"] == 0
        assert err <= TOL
