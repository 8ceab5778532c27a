"""GPU parity tests of the training path against the oracle, through the C ABI.

Bars: sample streams, initial matrices and projections bit-exact; sequential-order
epochs within 1e-5 relative (max |diff| / max |M|); Hogwild training judged by
link-prediction AUCROC within 0.01 of the oracle.
"""
import sys

import numpy as np
import pytest
import torch

import graphgen
import paper_2008_12336_amd as G
from oracle import gosh_oracle as O
from tests.linkpred import aucroc, make_eval_sets
from tests.util import corrupt, csr_from_pairs, rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = 1e-5


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def validate_csr(n, xadj, adj):
    """Host-side check that a kernel launched on these arrays stays in bounds."""
    xadj = np.asarray(xadj)
    adj = np.asarray(adj)
    assert xadj.size == n + 1 and xadj[0] == 0 and xadj[-1] == adj.size
    assert np.all(np.diff(xadj) >= 0)
    if adj.size:
        assert adj.min() >= 0 and adj.max() < n


def upload(n, xadj, adj, offsets64):
    validate_csr(n, xadj, adj)
    xt = torch.from_numpy(np.asarray(xadj, dtype=np.int64 if offsets64 else np.int32)).to(DEV)
    at = torch.from_numpy(np.asarray(adj, dtype=np.int32)).to(DEV)
    return G.csr_view(n, xt, at), (xt, at)


def small_graphs():
    out = {}
    e = graphgen.er_gnm(1024, 8192, 1)
    c = graphgen.to_csr(1024, e)
    out["er1024"] = (1024, c.xadj.numpy(), c.adj.numpy())
    e = graphgen.rmat(12, 1 << 15, 2)  # has isolated vertices and hubs
    c = graphgen.to_csr(1 << 12, e)
    out["rmat4096"] = (1 << 12, c.xadj.numpy(), c.adj.numpy())
    e = graphgen.chung_lu(3001, 20000, 3)  # ragged vertex count
    c = graphgen.to_csr(3001, e)
    out["cl3001"] = (3001, c.xadj.numpy(), c.adj.numpy())
    x, a = csr_from_pairs(24, [(i, (i + 1) % 24) for i in range(24)] + [(0, 9), (3, 17)])
    out["ring24"] = (24, x, a)  # tiny: repeated samples and negative == source abound
    x, a = csr_from_pairs(1, [])
    out["single"] = (1, x, a)
    x, a = csr_from_pairs(5, [])
    out["edgeless5"] = (5, x, a)
    return out


GRAPHS = small_graphs()


@pytest.mark.parametrize("name", sorted(GRAPHS))
@pytest.mark.parametrize("offsets64", [False, True])
@pytest.mark.parametrize("k", [0, 3, 5, 15])
def test_sample_stream_bit_exact(name, offsets64, k):
    n, xadj, adj = GRAPHS[name]
    say(f"[sample] graph={name} n={n} k={k} offsets64={offsets64}")
    g, keep = upload(n, xadj, adj, offsets64)
    for seed, epoch, level in [(1, 0, 0), (0xDEADBEEF12345678, 599, 7), (2 ** 64 - 1, 2 ** 31 - 1, 255)]:
        out = torch.full((n, k + 1), -7, dtype=torch.int32, device=DEV)
        G.gosh_sample_epoch(g, k, seed, epoch, level, out)
        torch.cuda.synchronize()
        want = O.sample_epoch(xadj, adj, k, seed, epoch, level)
        assert np.array_equal(out.cpu().numpy(), want)


@pytest.mark.parametrize("n,d", [(1000, 4), (777, 8), (513, 32), (300, 100), (1025, 128), (64, 512)])
def test_init_embedding_bit_exact(n, d):
    say(f"[init] n={n} d={d}")
    for seed, level in [(1, 0), (2 ** 63 + 11, 9)]:
        M = torch.zeros(n, d, dtype=torch.float32, device=DEV)
        G.gosh_init_embedding(M, seed, level)
        torch.cuda.synchronize()
        assert np.array_equal(M.cpu().numpy(), O.init_embedding(n, d, seed, level))


def start_matrix(n, d, seed, scale):
    """Initial rows scaled up so that dot products span the sigmoid's curved range."""
    return (O.init_embedding(n, d, seed, 0).astype(np.float64) * d * scale).astype(np.float32)


SEQ_CASES = [
    # graph, d, k, offsets64, scale
    ("ring24", 8, 15, False, 2.0),
    ("ring24", 128, 7, True, 0.6),
    ("single", 32, 3, False, 1.0),
    ("edgeless5", 16, 3, False, 1.5),
    ("er1024", 32, 3, False, 1.0),
    ("er1024", 4, 3, True, 2.0),
    ("er1024", 8, 0, False, 2.0),
    ("er1024", 16, 5, False, 1.5),
    ("er1024", 64, 3, False, 0.8),
    ("cl3001", 128, 3, True, 0.6),
    ("cl3001", 100, 4, False, 0.6),
    ("rmat4096", 128, 3, False, 0.6),
    ("rmat4096", 256, 2, True, 0.4),
    ("er1024", 512, 3, False, 0.3),
    ("er1024", 260, 1, False, 0.4),
]


@pytest.mark.parametrize("name,d,k,offsets64,scale", SEQ_CASES)
def test_sequential_epoch_parity(name, d, k, offsets64, scale):
    n, xadj, adj = GRAPHS[name]
    say(f"[seq] graph={name} n={n} d={d} k={k} offsets64={offsets64}")
    g, keep = upload(n, xadj, adj, offsets64)
    M0 = start_matrix(n, d, 5, scale)
    want = M0.copy()
    M = torch.from_numpy(M0).to(DEV)
    worst = 0.0
    for epoch in range(3):
        lr = G.gosh_lr(0.2, epoch, 3)
        G.gosh_train_epoch(g, M, k, lr, 77, epoch, 1, G.GOSH_FLAG_SEQUENTIAL)
        torch.cuda.synchronize()
        O.train_epoch(xadj, adj, want, k, lr, 77, epoch, 1)
        got = M.cpu().numpy()
        worst = max(worst, rel_err(got, want))
        assert worst <= TOL, (epoch, worst)
    if n > 5:
        assert rel_err(M0, want) > 1e-3  # the epochs did move the matrix
    say(f"      worst relative error {worst:.2e}")


@pytest.mark.parametrize("flags", [0, G.GOSH_FLAG_PLAIN_STORES, G.GOSH_FLAG_ATOMIC_ADDS])
@pytest.mark.parametrize("name,d,k", [("cl3001", 128, 3), ("er1024", 32, 3), ("rmat4096", 64, 5),
                                      ("ring24", 8, 15), ("er1024", 512, 1), ("cl3001", 100, 2)])
def test_parallel_epoch_with_zero_lr_moves_nothing(name, d, k, flags):
    """With lr = 0 every update writes back exactly what it read (or adds a zero step), so
    any row stored to the wrong place by the parallel launch would show."""
    n, xadj, adj = GRAPHS[name]
    say(f"[lr0] graph={name} n={n} d={d} k={k} flags={flags}")
    g, keep = upload(n, xadj, adj, False)
    M0 = start_matrix(n, d, 6, 1.0)
    M = torch.from_numpy(M0).to(DEV)
    G.gosh_train_epoch(g, M, k, 0.0, 3, 0, 0, flags)
    torch.cuda.synchronize()
    assert np.array_equal(M.cpu().numpy(), M0)


@pytest.mark.parametrize("name,d,k", [("cl3001", 128, 3), ("er1024", 32, 3), ("ring24", 8, 15),
                                      ("rmat4096", 100, 4)])
def test_atomic_epoch_matches_first_order_sum(name, d, k):
    """With atomic adds no update is lost, and for a small learning rate the order of
    updates matters only at second order: every row must end within a small fraction of
    its own movement from the sequential-order result, however the updates interleave."""
    n, xadj, adj = GRAPHS[name]
    lr = 1e-3
    say(f"[atomic] graph={name} n={n} d={d} k={k}")
    g, keep = upload(n, xadj, adj, False)
    M0 = start_matrix(n, d, 9, 0.5)
    want = M0.copy()
    O.train_epoch(xadj, adj, want, k, lr, 21, 2, 0)
    M = torch.from_numpy(M0).to(DEV)
    G.gosh_train_epoch(g, M, k, lr, 21, 2, 0, G.GOSH_FLAG_ATOMIC_ADDS)
    torch.cuda.synchronize()
    got = M.cpu().numpy().astype(np.float64)
    step = np.abs(want.astype(np.float64) - M0).max(axis=1)
    err = np.abs(got - want).max(axis=1)
    # second-order terms: each of the h touches of a row sees partners that moved by
    # about lr; allow 2% of the row's own movement plus rounding
    ok = err <= 0.02 * step + 2e-7 * np.abs(M0).max()
    say(f"      rows agreeing: {ok.mean():.4f}, worst err/step {np.max(err / np.maximum(step, 1e-30)):.3e}")
    assert ok.all()


@pytest.fixture
def tuning():
    yield G.gosh_set_tuning
    G.gosh_set_tuning()


@pytest.mark.parametrize("name,d,k,max_waves", [("cl3001", 128, 3, 1), ("cl3001", 128, 3, 7), ("er1024", 32, 3, 5),
                                                ("rmat4096", 64, 4, 100), ("ring24", 8, 15, 2),
                                                ("cl3001", 512, 2, 1000), ("er1024", 16, 3, 3)])
def test_few_wavefronts_walk_every_source_once(name, d, k, max_waves, tuning):
    """When the launch is capped to fewer wavefronts than there are sources to hand out, each
    wavefront walks a block of consecutive sources (ragged at the end of the graph).  With
    atomic adds and a small learning rate the result is the sequential one to first order, so a
    source that was skipped or taken twice shows as an error of the size of its own step; with
    lr = 0 nothing may move."""
    n, xadj, adj = GRAPHS[name]
    lr = 1e-3
    say(f"[blocks] graph={name} n={n} d={d} k={k} max_waves={max_waves}")
    tuning(max_waves=max_waves)
    g, keep = upload(n, xadj, adj, False)
    M0 = start_matrix(n, d, 9, 0.5)
    M = torch.from_numpy(M0).to(DEV)
    G.gosh_train_epoch(g, M, k, 0.0, 21, 2, 0, 0)
    torch.cuda.synchronize()
    assert np.array_equal(M.cpu().numpy(), M0)
    want = M0.copy()
    O.train_epoch(xadj, adj, want, k, lr, 21, 2, 0)
    G.gosh_train_epoch(g, M, k, lr, 21, 2, 0, G.GOSH_FLAG_ATOMIC_ADDS)
    torch.cuda.synchronize()
    got = M.cpu().numpy().astype(np.float64)
    step = np.abs(want.astype(np.float64) - M0).max(axis=1)
    err = np.abs(got - want).max(axis=1)
    ok = err <= 0.02 * step + 2e-7 * np.abs(M0).max()
    say(f"      rows agreeing: {ok.mean():.4f}, worst err/step {np.max(err / np.maximum(step, 1e-30)):.3e}")
    assert ok.all()


def test_parallel_epoch_stays_within_the_reach_of_its_updates():
    """A Hogwild epoch on a small graph races on nearly every row (all sources are in
    flight at once), so rows cannot be compared one by one; what must hold is that no
    row moves further than all updates that touch it could move it, and that rows do move.
    Row-by-row agreement with the sequential order is checked at full size, where races
    are rare (test_gpu_fullsize.py)."""
    n = 1 << 15
    d, k, lr = 128, 3, 1e-3
    edges = graphgen.rmat(15, 1 << 18, 4)
    c = graphgen.to_csr(n, edges)
    xadj, adj = c.xadj.numpy(), c.adj.numpy()
    say(f"[bounded] n={n} nnz={adj.size}")
    g, keep = upload(n, xadj, adj, False)
    M0 = start_matrix(n, d, 8, 0.5)
    stream = O.sample_epoch(xadj, adj, k, 5, 0, 0)
    touches = np.bincount(stream[stream >= 0].ravel(), minlength=n) + (k + 1)
    M = torch.from_numpy(M0).to(DEV)
    G.gosh_train_epoch(g, M, k, lr, 5, 0, 0, 0)
    torch.cuda.synchronize()
    got = M.cpu().numpy().astype(np.float64)
    step = np.abs(got - M0).max(axis=1)
    # one update moves a row by at most lr * max|other row| (|score| <= lr)
    assert np.all(step <= 1.01 * touches * lr * np.abs(M0).max() * 1.1)
    assert (step > 0).mean() > 0.99


def hogwild_train(n, xadj, adj, d, k, lr0, epochs, seed):
    g, keep = upload(n, xadj, adj, False)
    M = torch.empty(n, d, dtype=torch.float32, device=DEV)
    G.gosh_init_embedding(M, seed, 0)
    for j in range(epochs):
        G.gosh_train_epoch(g, M, k, G.gosh_lr(lr0, j, epochs), seed, j, 0, 0)
    torch.cuda.synchronize()
    return M.cpu().numpy()


def test_hogwild_aucroc_config1():
    """Config 1: 1,024 vertices, 8,192 uniform-endpoint edges, d = 32, k = 3,
    lr 0.025 -> 0, 100 epochs, seed 1, 10 % of edges held out."""
    n = 1024
    edges = graphgen.er_gnm(n, 8192, 1)
    train, test = graphgen.holdout_split(edges, 0.1, 1001)
    c = graphgen.to_csr(n, train)
    xadj, adj = c.xadj.numpy(), c.adj.numpy()
    sets = make_eval_sets(n, train.numpy(), test.numpy(), seed=1)
    Mo = O.init_embedding(n, 32, 1, 0)
    O.train_level(xadj, adj, Mo, 3, 0.025, 100, 1, 0)
    Mg = hogwild_train(n, xadj, adj, 32, 3, 0.025, 100, 1)
    ho, fo = aucroc(Mo, sets)
    hg, fg = aucroc(Mg, sets)
    say(f"[auc cfg1] oracle held-out {ho:.4f} fit {fo:.4f} | gpu held-out {hg:.4f} fit {fg:.4f}")
    assert np.isfinite(Mg).all()
    assert abs(hg - ho) <= 0.01
    assert abs(fg - fo) <= 0.01


def test_hogwild_aucroc_rmat():
    """A graph with structure (R-MAT, 4,096 vertices): held-out AUCROC far above chance
    and within 0.01 of the oracle's."""
    n = 1 << 12
    edges = graphgen.rmat(12, 1 << 16, 2)
    train, test = graphgen.holdout_split(edges, 0.1, 1002)
    c = graphgen.to_csr(n, train)
    xadj, adj = c.xadj.numpy(), c.adj.numpy()
    sets = make_eval_sets(n, train.numpy(), test.numpy(), seed=1)
    Mo = O.init_embedding(n, 32, 1, 0)
    O.train_level(xadj, adj, Mo, 3, 0.045, 300, 1, 0)
    Mg = hogwild_train(n, xadj, adj, 32, 3, 0.045, 300, 1)
    ho, fo = aucroc(Mo, sets)
    hg, fg = aucroc(Mg, sets)
    say(f"[auc rmat] oracle held-out {ho:.4f} fit {fo:.4f} | gpu held-out {hg:.4f} fit {fg:.4f}")
    assert hg > 0.75
    assert abs(hg - ho) <= 0.01
    assert abs(fg - fo) <= 0.01


@pytest.mark.parametrize("nc,nf,d", [(5, 9, 8), (300, 1000, 128), (1, 17, 4), (700, 701, 100)])
def test_project_bit_exact(nc, nf, d):
    say(f"[project] nc={nc} nf={nf} d={d}")
    rng = np.random.default_rng(nc)
    Mc = rng.normal(size=(nc, d)).astype(np.float32)
    m = rng.integers(0, nc, size=nf).astype(np.int32)
    m[:nc] = np.arange(nc)
    out = torch.zeros(nf, d, dtype=torch.float32, device=DEV)
    G.gosh_project(torch.from_numpy(Mc).to(DEV), torch.from_numpy(m).to(DEV), out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), O.project(Mc, m))


def test_operands_a_kernel_cannot_reach_are_refused():
    """Pageable host memory, or a span that runs past its device allocation, would make a
    kernel fault: the entry points check where their operands live and refuse with
    GOSH_EINVAL instead of launching."""
    import ctypes as C

    n, d, k = 1000, 32, 3
    c = graphgen.to_csr(n, graphgen.er_gnm(n, 4000, 1))
    dev = c.to(DEV)
    lib = G.lib()
    M_host = torch.zeros(n, d, dtype=torch.float32)
    M_dev = torch.zeros(n, d, dtype=torch.float32, device=DEV)
    g_dev = G.csr_view(n, dev.xadj, dev.adj)
    g_host = G.csr_view(n, c.xadj, c.adj)
    # the matrix in pageable host memory
    assert lib.gosh_train_epoch(C.byref(g_dev), M_host.data_ptr(), d, k, 0.1, 1, 0, 0, 0, None) == -1
    assert "reach" in G.gosh_last_error()
    # the graph in pageable host memory
    assert lib.gosh_train_epoch(C.byref(g_host), M_dev.data_ptr(), d, k, 0.1, 1, 0, 0, 0, None) == -1
    assert lib.gosh_sample_epoch(C.byref(g_host), k, 1, 0, 0, M_dev.data_ptr(), None) == -1
    assert lib.gosh_init_embedding(M_host.data_ptr(), n, d, 1, 0, None) == -1
    # a matrix far smaller than n x d: its own allocation of 64 rows, asked to hold 2^22
    small = torch.empty(1 << 22, dtype=torch.uint8, device=DEV)  # a 4 MiB block of its own
    assert lib.gosh_init_embedding(small.data_ptr(), 1 << 22, d, 1, 0, None) == -1
    assert "do not fit" in G.gosh_last_error()
    # and the device still works
    G.gosh_train_epoch(g_dev, M_dev, k, 0.1, 1, 0, 0, G.GOSH_FLAG_SEQUENTIAL)
    torch.cuda.synchronize()


@pytest.mark.parametrize("offsets64", [False, True])
def test_malformed_graph_keeps_the_kernels_inside_their_operands(offsets64):
    """The training kernels trust no graph content: a row whose offsets leave adj counts as
    empty, an entry that names no vertex is no sample.  Every other source draws what the
    oracle draws on the intact graph, and training leaves a finite matrix."""
    n, d, k = 3000, 32, 3
    c = graphgen.to_csr(n, graphgen.chung_lu(n, 24000, 5))
    good_xadj, good_adj = c.xadj.numpy().astype(np.int64), c.adj.numpy()
    xadj, adj, touched = corrupt(c, offsets64, 1)
    nnz = adj.size
    # what the guards must decide, row by row, computed here on the host
    lo, hi = xadj[:-1].astype(np.int64), xadj[1:].astype(np.int64)
    row_ok = (lo >= 0) & (lo <= hi) & (hi <= nnz)
    assert (~row_ok).sum() >= 12 and all(not row_ok[v] for v in touched)
    want = O.sample_epoch(good_xadj, good_adj, k, 9, 2, 1)
    # the intact rows: the same entry index is drawn; the entry itself may have been replaced
    for v in range(n):
        if v in touched or want[v, 0] < 0:
            continue
        j = good_xadj[v] + np.searchsorted(good_adj[good_xadj[v]:good_xadj[v + 1]], want[v, 0])
        want[v, 0] = adj[j] if 0 <= adj[j] < n else -1
    xadj_dev, adj_dev = torch.from_numpy(xadj).to(DEV), torch.from_numpy(adj).to(DEV)
    g = G.csr_view(n, xadj_dev, adj_dev)
    assert g.nnz == nnz
    out = torch.empty(n, k + 1, dtype=torch.int32, device=DEV)
    say(f"malformed graph, offsets64={offsets64}: sample stream")
    G.gosh_sample_epoch(g, k, 9, 2, 1, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    rows = np.array([v not in touched for v in range(n)])
    assert np.array_equal(got[rows], want[rows])
    assert np.array_equal(got[:, 1:], want[:, 1:])
    assert np.all(got[~rows, 0] == -1)
    for flags in (G.GOSH_FLAG_SEQUENTIAL, 0):
        say(f"malformed graph, offsets64={offsets64}: epoch with flags {flags}")
        M = torch.from_numpy(O.init_embedding(n, d, 1, 0)).to(DEV)
        G.gosh_train_epoch(g, M, k, 0.05, 9, 2, 1, flags)
        torch.cuda.synchronize()
        assert torch.isfinite(M).all()


def test_projection_through_a_map_with_invalid_entries():
    """A map entry that names no coarse vertex gives a row of zeros; the others are copied."""
    n_fine, n_coarse, d = 500, 40, 16
    rng = np.random.default_rng(3)
    m = rng.integers(0, n_coarse, size=n_fine, dtype=np.int32)
    bad = rng.choice(n_fine, size=20, replace=False)
    m[bad] = np.resize(np.array([n_coarse, -1, 2**31 - 1, -2**31], dtype=np.int32), 20)
    Mc = rng.standard_normal((n_coarse, d)).astype(np.float32)
    out = torch.full((n_fine, d), 7.0, dtype=torch.float32, device=DEV)
    G.gosh_project(torch.from_numpy(Mc).to(DEV), torch.from_numpy(m).to(DEV), out)
    torch.cuda.synchronize()
    want = np.zeros((n_fine, d), dtype=np.float32)
    valid = (m >= 0) & (m < n_coarse)
    want[valid] = Mc[m[valid]]
    assert np.array_equal(out.cpu().numpy(), want)


def test_matrix_place_gives_usable_memory_and_takes_it_back():
    """gosh_matrix_place: the matrix is an ordinary n x d device array to every entry point
    (training on it gives bit for bit what training on a plain tensor gives), only the pieces
    under it stay allocated, release returns them, and a second release is refused."""
    n, d, k = 1 << 16, 128, 3
    c = graphgen.to_csr(n, graphgen.chung_lu(n, 1 << 19, 2))
    xd, ad = c.xadj.to(DEV), c.adj.to(DEV)
    g = G.csr_view(n, xd, ad)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    M, info = G.gosh_matrix_place(n, d, arena_bytes=6 << 30)
    assert M.shape == (n, d) and M.dtype == torch.float32 and M.is_cuda and M.is_contiguous()
    assert info["arena_bytes"] == 6 << 30 and info["probes"] >= 3
    assert n * d * 4 <= info["kept_bytes"] <= n * d * 4 + (2 << 30)
    assert free_before - torch.cuda.mem_get_info()[0] <= info["kept_bytes"] + (64 << 20)
    plain = torch.empty(n, d, dtype=torch.float32, device=DEV)
    for X in (M, plain):
        G.gosh_init_embedding(X, 5, 0)
        G.gosh_train_epoch(g, X, k, 0.05, 5, 0, 0, G.GOSH_FLAG_SEQUENTIAL)
        G.gosh_row_probe(X, 1000)
    torch.cuda.synchronize()
    assert torch.equal(M, plain)
    # the rotation in place and the projection take it too
    G.gosh_train_parts(n, xd, ad, M, k, 10, 0.0, 1, force_K=4)
    out = torch.empty(100, d, dtype=torch.float32, device=DEV)
    G.gosh_project(M, torch.arange(100, dtype=torch.int32, device=DEV), out)
    torch.cuda.synchronize()
    assert torch.equal(out, plain[:100])
    G.gosh_matrix_release(M)
    with pytest.raises(G.GoshError):
        G.gosh_matrix_release(M)
    del M
    # too little room for an arena of three times the matrix: refused, and the helper falls back
    with pytest.raises(G.GoshError):
        G.gosh_matrix_place(n, d, arena_bytes=1 << 30)
    from paper_2008_12336_amd.placement import place_matrix

    P, info2 = place_matrix(n, d, arena_bytes=1 << 30)
    assert info2["mode"].startswith("plain") and P.shape == (n, d)
    Q, info3 = place_matrix(n, d, arena_bytes=6 << 30)
    assert info3["mode"] == "search"
    G.gosh_matrix_release(Q)


def test_row_probe_leaves_the_matrix_as_it_is():
    """gosh_row_probe reads random rows and writes them back with zero added: the values stay,
    for every d (a lane group per row, one or two passes over it) and with rows hit many
    times; the read-only mode and the epoch mix leave them too; the write mode zeroes the
    rows it visits and nothing else."""
    for n, d in ((1000, 128), (37, 512), (5000, 4), (300, 260), (4097, 8), (513, 32), (100, 100)):
        M0 = torch.randn(n, d, dtype=torch.float32, device=DEV)
        M = M0.clone()
        for mode in (G.GOSH_PROBE_READ_WRITE, G.GOSH_PROBE_READ, G.GOSH_PROBE_EPOCH_MIX):
            G.gosh_row_probe(M, 8 * n, seed=3, mode=mode)
        torch.cuda.synchronize()
        assert torch.equal(M, M0), (n, d)
        G.gosh_row_probe(M, n // 4, seed=4, mode=G.GOSH_PROBE_WRITE)
        torch.cuda.synchronize()
        zeroed = (M == 0).all(dim=1)
        kept = (M == M0).all(dim=1)
        assert (zeroed | kept).all() and 0 < int(zeroed.sum()) <= max(1, n // 4), (n, d)
    G.gosh_row_probe(M, 0)  # nothing to do
    with pytest.raises(G.GoshError):
        G.gosh_row_probe(M, 10, mode=7)
