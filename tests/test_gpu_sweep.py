"""Randomised parity sweep over the whole C ABI (valid inputs only, fixed seeds): for every
drawn case the sample stream (bit-exact), one sequential-order epoch, the device coarsening
(maps bit-exact), the sequential V-cycle and a sequential rotation are compared with the
oracle.  Shapes are drawn around the tile edges of the kernels (63/64/65 vertices, d = 4 ..
512 including non-powers of two, k = 0 .. 15, both offset widths, every pair order)."""
import numpy as np
import pytest
import torch

import graphgen
import paper_2008_12336_amd as G
from oracle import gosh_oracle as O
from tests.util import conditioned_bar, oracle_sensitivity, rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def draw_graph(rng):
    n = int(rng.choice([1, 2, 3, 17, 63, 64, 65, 255, 257, 1000, 2049]))
    m = int(rng.integers(0, 8 * n + 1))
    kind = str(rng.choice(["er", "cl", "rmat"]))
    gseed = int(rng.integers(0, 1000))
    if kind == "rmat":
        lg = max(1, int(np.ceil(np.log2(max(n, 2)))))
        n = 1 << lg
        e = graphgen.rmat(lg, max(m, 1), gseed)
    elif kind == "cl" and n >= 3:
        e = graphgen.chung_lu(n, max(m, 1), gseed)
    else:
        kind = "er"
        e = graphgen.er_gnm(n, min(m, n * (n - 1) // 2), gseed)
    return kind, n, graphgen.to_csr(n, e, offsets64=bool(rng.integers(0, 2)))


@pytest.mark.parametrize("sweep_seed", [11, 12, 13])
def test_random_cases_match_the_oracle(sweep_seed):
    rng = np.random.default_rng(sweep_seed)
    for case in range(25):
        kind, n, c = draw_graph(rng)
        xadj, adj = c.xadj.numpy(), c.adj.numpy()
        d = int(rng.choice([4, 8, 12, 16, 32, 36, 64, 100, 128, 132, 256, 260, 512]))
        k = int(rng.integers(0, 16))
        seed = int(rng.integers(1, 2 ** 62))
        epoch, level = int(rng.integers(0, 2 ** 31)), int(rng.integers(0, 256))
        print(f"sweep {sweep_seed}/{case}: {kind} n={n} nnz={adj.size} xadj={c.xadj.dtype} d={d} k={k} "
              f"seed={seed} epoch={epoch} level={level}", flush=True)
        xd, ad = c.xadj.to(DEV), c.adj.to(DEV)
        g = G.csr_view(n, xd, ad)
        out = torch.empty(n, k + 1, dtype=torch.int32, device=DEV)
        G.gosh_sample_epoch(g, k, seed, epoch, level, out)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), O.sample_epoch(xadj, adj, k, seed, epoch, level))

        # one epoch in sequential order, from rows large enough to bend the sigmoid
        scale = float(rng.choice([0.3, 0.6, 1.0, 2.0]))
        lr = float(rng.choice([0.01, 0.05, 0.2]))
        M0 = (O.init_embedding(n, d, seed, 0).astype(np.float64) * d * scale).astype(np.float32)
        M = torch.from_numpy(M0.copy()).to(DEV)
        G.gosh_train_epoch(g, M, k, lr, seed, epoch, level, G.GOSH_FLAG_SEQUENTIAL)
        torch.cuda.synchronize()
        # (rows this long can make the epoch ill-conditioned in the oracle itself, as in the
        # rotation below: the bar follows the oracle's measured sensitivity there, 1e-5 elsewhere)
        want, sens = oracle_sensitivity(lambda X: O.train_epoch(xadj, adj, X, k, lr, seed, epoch, level), M0)
        err, bar = rel_err(M.cpu().numpy(), want), conditioned_bar(sens)
        assert err <= bar, (err, bar, sens, scale, lr)
        # the concurrent kernels (default mix, plain stores, atomic adds) move nothing at lr = 0
        for flags in (0, G.GOSH_FLAG_PLAIN_STORES, G.GOSH_FLAG_ATOMIC_ADDS):
            M = torch.from_numpy(M0.copy()).to(DEV)
            G.gosh_train_epoch(g, M, k, 0.0, seed, epoch, level, flags)
            torch.cuda.synchronize()
            assert np.array_equal(M.cpu().numpy(), M0)

        # Alg. 4 on the device and the sequential V-cycle of Alg. 2
        thr, shrink = int(rng.choice([1, 10, 100])), float(rng.choice([0.5, 0.8, 0.95]))
        epochs, dd, kk = int(rng.integers(20, 60)), int(rng.choice([8, 32, 64])), min(k, 5)
        try:
            want_m0, graphs, maps, _ = O.embed(xadj, adj, dd, kk, epochs, 0.3, 0.05, seed, threshold=thr,
                                               min_shrink=shrink)
        except Exception:  # more levels than epochs: refused by both sides, not a parity case
            want_m0 = None
        if want_m0 is not None:
            h = G.gosh_coarsen_device(n, xd, ad, threshold=thr, min_shrink=shrink)
            assert h.levels == len(graphs)
            for i in range(h.levels - 1):
                got_map = h.map(i)
                if got_map.shape != maps[i].shape or not np.array_equal(got_map, maps[i]):
                    # say which side moved: the oracle asked again, and the host coarsening
                    again = O.coarsen(xadj, adj, thr, shrink)[1]
                    host = G.gosh_coarsen(n, c.xadj, c.adj, threshold=thr, min_shrink=shrink)
                    raise AssertionError(
                        f"map {i} of {h.levels - 1} differs (threshold {thr}, shrink {shrink}):\n device {got_map.tolist()}\n"
                        f" oracle {maps[i].tolist()}\n oracle asked again {again[i].tolist()}\n"
                        f" host coarsening {host.map(i).tolist()}")
            Mv = torch.zeros(n, dd, dtype=torch.float32, device=DEV)
            G.gosh_embed(h, Mv, kk, epochs, 0.3, 0.05, seed, flags=G.GOSH_FLAG_SEQUENTIAL)
            torch.cuda.synchronize()
            assert rel_err(Mv.cpu().numpy(), want_m0) <= 1e-5
            h.free()

        # Alg. 5: a sequential rotation from rows of the full range of magnitudes.  Where the
        # drawn rows are so long that the run is ill-conditioned in the oracle itself (it
        # cannot repeat its own result from an input one ulp away), the bar follows that
        # measured sensitivity; everywhere else it is 1e-5.
        if n >= 2:
            K, P, S = int(rng.integers(1, min(n, 9) + 1)), int(rng.integers(2, 7)), int(rng.integers(1, 4))
            B = int(rng.integers(1, 5))
            ep = int(rng.integers(1, 3 * B * K + 1))
            blocked, on_device = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
            R0 = (O.init_embedding(n, d, seed, 1).astype(np.float64) * d * scale).astype(np.float32)
            block = O.blocked_block_size(P, K) if blocked else 0
            want, sens = oracle_sensitivity(
                lambda X: O.train_parts(xadj, adj, X, kk, ep, 0.1, seed, level, K, B, block=block), R0)
            bar = conditioned_bar(sens)
            print(f"   rotation K={K} P={P} S={S} B={B} epochs={ep} blocked={blocked} device_graph={on_device} "
                  f"scale={scale} oracle sensitivity={sens:.1e} bar={bar:.1e}", flush=True)
            Mp = torch.from_numpy(R0.copy()).pin_memory()
            G.gosh_train_parts(n, xd if on_device else c.xadj, ad if on_device else c.adj, Mp, kk, ep, 0.1, seed,
                               level=level, P_gpu=P, S_gpu=S, B=B, force_K=K,
                               flags=G.GOSH_FLAG_SEQUENTIAL | (G.GOSH_FLAG_BLOCKED_ORDER if blocked else 0))
            err = rel_err(Mp.numpy(), want)
            assert err <= bar, (err, bar, sens)
