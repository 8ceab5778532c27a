"""Parity at the benchmark's full size and launch configuration (workload 4,
level 0: Chung-Lu graph, 2^24 vertices, 2^28 edge draws, int64 offsets, d = 128, k = 3).

The oracle cannot replay a racing Hogwild epoch, so the checks are:
  * the sample stream of a whole epoch, bit-exact against the oracle (all 2^26 ids);
  * sampled rows of the initial matrix, bit-exact;
  * a Hogwild epoch with lr = 0 leaves sampled rows untouched;
  * a Hogwild epoch with a small learning rate: for sampled rows, the oracle applies,
    one by one and in sequential order, exactly the updates that touch the row (taking
    the other row of each update from the matrix before the epoch).  The order of
    updates matters only at second order in lr, so the kernel's row must agree to a
    small fraction of the row's own movement; a row that lost an update to a race
    (tolerated by the method) is the rare exception that is counted, not hidden.
"""
import sys
import time

import numpy as np
import pytest
import torch

import graphgen
import paper_2008_12336_amd as G
from oracle import gosh_oracle as O

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]
DEV = "cuda:0"
LOG2N, LOG2M, D, K = 24, 28, 128, 3


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def big():
    t = time.time()
    n = 1 << LOG2N
    edges = graphgen.chung_lu(n, 1 << LOG2M, 1, gamma=2.1, device=DEV)
    csr = graphgen.to_csr(n, edges, offsets64=True)
    del edges
    torch.cuda.synchronize()
    say(f"[full] graph on device: n={n} nnz={csr.nnz} in {time.time() - t:.1f}s")
    xadj = csr.xadj.cpu().numpy()
    adj = csr.adj.cpu().numpy()
    assert xadj[0] == 0 and xadj[-1] == adj.size and np.all(np.diff(xadj) >= 0)
    assert adj.min() >= 0 and adj.max() < n
    return n, csr, xadj, adj


def test_full_size_sample_stream_bit_exact(big):
    n, csr, xadj, adj = big
    g = G.csr_view(n, csr.xadj, csr.adj)
    out = torch.empty(n, K + 1, dtype=torch.int32, device=DEV)
    say("[full] sample stream on device")
    G.gosh_sample_epoch(g, K, 1, 17, 0, out)
    torch.cuda.synchronize()
    t = time.time()
    want = O.sample_epoch(xadj, adj, K, 1, 17, 0)
    say(f"[full] oracle stream in {time.time() - t:.1f}s")
    assert np.array_equal(out.cpu().numpy(), want)


@pytest.mark.parametrize("D", [128, 32])  # the benchmark's kernel, and the 128-bit small-dimension one
def test_full_size_hogwild_epoch_rows(big, D):
    n, csr, xadj, adj = big
    g = G.csr_view(n, csr.xadj, csr.adj)
    seed, epoch, lr, scale = 1, 3, 1e-3, 48.0 * D / 128
    M = torch.empty(n, D, dtype=torch.float32, device=DEV)
    G.gosh_init_embedding(M, seed, 0)
    torch.cuda.synchronize()
    rng = np.random.default_rng(0)
    rows = np.unique(np.concatenate((rng.integers(0, n, 3000), [0, 1, n - 2, n - 1])))
    first = int(rows[len(rows) // 2])
    blk = M[first:first + 64].cpu().numpy()
    assert np.array_equal(blk, O.init_rows(first, blk.shape[0], D, seed, 0))
    say("[full] initial rows bit-exact")
    M.mul_(scale)  # spread the dot products over the curved part of the sigmoid

    rows_t = torch.from_numpy(rows).to(DEV)
    before = M[rows_t].cpu().numpy()
    G.gosh_train_epoch(g, M, K, 0.0, seed, epoch, 0, 0)
    torch.cuda.synchronize()
    assert np.array_equal(M[rows_t].cpu().numpy(), before)
    say("[full] lr = 0 epoch leaves the sampled rows untouched")

    # who touches the sampled rows in this epoch
    stream = O.sample_epoch(xadj, adj, K, seed, epoch, 0)
    flat = stream.ravel()
    hit = np.nonzero(np.isin(flat, rows))[0]
    hit_src, hit_j = hit // (K + 1), hit % (K + 1)
    partners = np.unique(np.concatenate((hit_src, stream[rows].ravel().clip(min=0), rows)))
    part_t = torch.from_numpy(partners).to(DEV)
    M0 = dict(zip(partners.tolist(), M[part_t].cpu().numpy()))
    by_row = {}
    for s, j in zip(hit_src.tolist(), hit_j.tolist()):
        by_row.setdefault(int(stream[s, j]), []).append((s, j))

    say(f"[full] hogwild epoch, lr={lr}, {len(rows)} rows sampled, {len(hit)} incoming updates")
    G.gosh_train_epoch(g, M, K, lr, seed, epoch, 0, 0)
    torch.cuda.synchronize()
    got = M[rows_t].cpu().numpy().astype(np.float64)

    bad = 0
    worst_ok = 0.0
    for i, r in enumerate(rows.tolist()):
        row = M0[r].copy()
        events = sorted(by_row.get(r, []) + [(r, -1)])  # sequential order: by source id
        for s, j in events:
            if j == -1:  # r's own turn as a source
                for jj in range(K + 1):
                    v = int(stream[r, jj])
                    if v < 0 or v == r:
                        continue
                    O.update(row, M0[v].copy(), 1 if jj == 0 else 0, lr)
            elif s != r:
                O.update(M0[s].copy(), row, 1 if j == 0 else 0, lr)
        step = np.abs(row.astype(np.float64) - M0[r]).max()
        err = np.abs(got[i] - row).max()
        if err <= 0.02 * step + 1e-7 * np.abs(row).max():
            worst_ok = max(worst_ok, err / max(step, 1e-30))
        else:
            bad += 1
    frac_bad = bad / len(rows)
    say(f"[full] rows off by more than 2% of their own step: {bad}/{len(rows)} "
        f"(worst agreeing row: {worst_ok:.2e} of its step)")
    # Rows that miss are rows that lost an update to a race, which the method tolerates: two
    # sources in flight at once that touch the same cold row.  Their share follows the rows in
    # flight -- resident wavefronts x sources per wavefront (2 at d = 128, 8 at d = 32) x K + 2
    # rows each, out of n: about 0.5 % and 2 % here (observed 0.8 % and 2.2 %).
    assert frac_bad <= (0.03 if D == 128 else 0.05)


def test_full_size_coarsening(big):
    """Alg. 4 at the benchmark's size: the first map against the oracle's marking sweep
    (bit-exact, 2^24 entries), the whole device-built hierarchy against the host-built one
    (every graph, map and multiplicity), and weight conservation from level to level."""
    n, csr, xadj, adj = big
    xh, ah = csr.xadj.cpu(), csr.adj.cpu()
    say("[full] coarsening on the device")
    t = time.time()
    hd = G.gosh_coarsen_device(n, xh, ah, threshold=100, min_shrink=0.8)
    say(f"[full] device hierarchy: {hd.levels} levels in {time.time() - t:.2f}s")
    t = time.time()
    want_map, n_coarse = O.coarsen_map(xadj, adj)
    say(f"[full] oracle marking sweep in {time.time() - t:.1f}s: {n_coarse} clusters")
    assert hd.graph(1)[0] == n_coarse
    assert np.array_equal(hd.map(0), want_map)
    del want_map
    t = time.time()
    hh = G.gosh_coarsen(n, xh, ah, threshold=100, min_shrink=0.8)
    say(f"[full] host hierarchy in {time.time() - t:.1f}s")
    assert hh.levels == hd.levels >= 4
    total = adj.size
    for i in range(hh.levels):
        nh, xa, aa = hh.graph(i)
        nd, xb, ab = hd.graph(i)
        assert nh == nd and np.array_equal(xa, xb) and np.array_equal(aa, ab), f"graph {i}"
        if i > 0:
            mult = hd.mult(i)
            assert np.array_equal(hh.mult(i), mult), f"multiplicities {i}"
            # entries swallowed by clusters only ever reduce the total weight
            assert 0 < int(mult.sum()) <= total
            total = int(mult.sum())
        if i + 1 < hh.levels:
            assert np.array_equal(hh.map(i), hd.map(i)), f"map {i}"
    say(f"[full] device hierarchy == host hierarchy, sizes {[hd.graph(i)[0] for i in range(hd.levels)]}")
    hh.free()
    hd.free()
