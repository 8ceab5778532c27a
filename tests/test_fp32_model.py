"""Where the sequential-order bar comes from, shown on the CPU.  The kernel computes an
update of Alg. 1 in fp32 (tree-ordered dot product, fp32 sigmoid, fused axpys), the oracle
in fp64 on the same fp32-stored rows.  tests/fp32_model.py models the former.  Per update
the two agree to a few units of 2^-24.  Whether such differences stay that small over a run
is a property of the run, not of the implementation: a randomised rotation case (Chung-Lu,
1,000 vertices, d = 512, k = 5, K = 9, B = 4, 76 epochs, rows of magnitude 1) ended 4.8e-4
from the oracle on the GPU, and here the oracle itself, started one ulp away, ends 2.5e-4
from its own result -- rows that long make the SGD step exceed what the curvature of the
logistic loss allows, and every difference is amplified."""
import numpy as np

import graphgen
from oracle import gosh_oracle as O
from tests import fp32_model as F
from tests.util import oracle_sensitivity, rel_err


def test_single_updates_agree_to_a_few_ulps():
    rng = np.random.default_rng(1)
    for d in (8, 100, 128, 512):
        lanes, upl = F.lanes_for(d)
        for scale in (0.05, 0.3, 1.0):
            for label in (0, 1):
                s = (rng.standard_normal(d) * scale).astype(np.float32)
                r = (rng.standard_normal(d) * scale).astype(np.float32)
                a, b = s.copy(), r.copy()
                F.update_fp32(a, b, label, 0.1, lanes, upl)
                O.update(s, r, label, 0.1)
                top = max(np.abs(s).max(), np.abs(r).max())
                assert np.abs(a - s).max() <= 4 * 2.0 ** -24 * top + 1e-12
                assert np.abs(b - r).max() <= 4 * 2.0 ** -24 * top + 1e-12


def test_dot_tree_is_a_dot_product():
    rng = np.random.default_rng(2)
    for d in (4, 12, 36, 128, 260, 512):
        lanes, upl = F.lanes_for(d)
        s = rng.standard_normal(d).astype(np.float32)
        r = rng.standard_normal(d).astype(np.float32)
        exact = float(s.astype(np.float64) @ r.astype(np.float64))
        mass = float(np.abs(s.astype(np.float64) * r.astype(np.float64)).sum())
        assert abs(float(F.dot_tree(s, r, lanes, upl)) - exact) <= 12 * 2.0 ** -24 * mass


def case_445():
    """The randomised rotation case that missed 1e-5 on the GPU (4.8e-4): Chung-Lu graph of
    1,000 vertices, d = 512, k = 5, K = 9 parts, B = 4, 76 epochs = 3 rotations, starting rows
    uniform in [-scale/2, scale/2) with scale = 2."""
    n = 1000
    c = graphgen.to_csr(n, graphgen.chung_lu(n, 5690, 26))
    xadj, adj = c.xadj.numpy().astype(np.int64), c.adj.numpy()
    assert adj.size == 11026
    return dict(n=n, xadj=xadj, adj=adj, d=512, k=5, K=9, B=4, epochs=76, seed=779413867887070026, level=244)


def test_the_rotation_case_that_missed_the_bar_is_ill_conditioned_in_the_oracle_itself():
    """With rows of magnitude 1 at d = 512, lr * |row|^2 / 4 is about 4 at the start (40 at
    the end): every update near the sigmoid's centre multiplies an existing difference by up
    to 1 + lr * |row|^2 / 4.  The fp64 oracle, run twice from inputs one ulp apart, ends 2.5e-4
    apart -- the size of the GPU's and of the fp32 model's distance from it.  With the same
    rows scaled to 1, 0.6 or 0.3 the same run repeats to about 1e-6."""
    c = case_445()
    for scale, lo, hi in ((2.0, 5e-5, 5e-3), (1.0, 0, 5e-6), (0.3, 0, 5e-6)):
        R0 = (O.init_embedding(c["n"], c["d"], c["seed"], 1).astype(np.float64) * c["d"] * scale).astype(np.float32)
        run = lambda M: O.train_parts(c["xadj"], c["adj"], M, c["k"], c["epochs"], 0.1, c["seed"], c["level"],
                                      c["K"], c["B"])
        _, sens = oracle_sensitivity(run, R0)
        step = 0.1 * float((R0.astype(np.float64) ** 2).sum(axis=1).mean()) / 4
        assert lo <= sens <= hi, (scale, sens)
        assert (step > 2) == (scale == 2.0)  # 4.3 at scale 2; 1.1 and 0.1 for the others


def test_model_tracks_the_oracle_where_the_run_is_well_conditioned():
    """One rotation of a small well-conditioned case: the fp32 model (tree dot, fp32 sigmoid,
    fused axpys) stays within 1e-5 of the fp64 oracle, as the kernel does."""
    n, d, k, B, K, seed, level = 120, 128, 3, 2, 3, 5, 1
    c = graphgen.to_csr(n, graphgen.chung_lu(n, 700, 4))
    xadj, adj = c.xadj.numpy().astype(np.int64), c.adj.numpy()
    R0 = (O.init_embedding(n, d, seed, 1).astype(np.float64) * d * 0.8).astype(np.float32)
    want, model = R0.copy(), R0.copy()
    dummy = np.zeros((n, 4), dtype=np.float32)
    ps = -(-n // K)
    for q, (a, b) in enumerate(O.pair_order(K)):
        stream = O.train_pair(xadj, adj, dummy, k, B, K, a, b, 0.0, seed, 0, level, q, want_stream=True)
        O.train_pair(xadj, adj, want, k, B, K, a, b, 0.1, seed, 0, level, q)
        srcs = [v for p in ([a] if a == b else [a, b]) for v in range(min(n, p * ps), min(n, p * ps + ps))]
        per = B * (k + 1)
        F.replay(model, [(srcs[i // per], int(v), 1 if i % (k + 1) == 0 else 0) for i, v in enumerate(stream)], 0.1)
    assert rel_err(R0, want) > 1e-3
    assert rel_err(model, want) <= 1e-5
