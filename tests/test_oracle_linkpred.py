"""The oracle's embedding carries link-prediction signal (end-to-end pin of signs,
sampling and schedule): AUCROC far above chance on a graph with structure."""
import numpy as np

import graphgen
from oracle import gosh_oracle as O
from tests.linkpred import aucroc, make_eval_sets


def test_oracle_embedding_predicts_links_on_rmat():
    n = 1 << 12
    edges = graphgen.rmat(12, 1 << 16, seed=2)
    train, test = graphgen.holdout_split(edges, 0.1, 1002)
    csr = graphgen.to_csr(n, train)
    xadj, adj = csr.xadj.numpy().astype(np.int64), csr.adj.numpy()
    sets = make_eval_sets(n, train.numpy(), test.numpy(), seed=1)
    M = O.init_embedding(n, 32, 1, 0)
    held0, fit0 = aucroc(M, sets)
    O.train_level(xadj, adj, M, 3, 0.045, 300, 1, 0)
    held, fit = aucroc(M, sets)
    assert abs(held0 - 0.5) < 0.06  # the random initialisation knows nothing
    assert held > 0.75 and fit > 0.9, (held, fit)


def test_uniform_random_graph_has_no_held_out_signal():
    """On config 1 (uniform random endpoints) held-out edges are independent of the
    training edges, so held-out AUCROC stays at chance for any embedding; what
    training does show is that the embedding separates training edges from non-edges."""
    n = 1024
    edges = graphgen.er_gnm(n, 8192, 1)
    train, test = graphgen.holdout_split(edges, 0.1, 1001)
    csr = graphgen.to_csr(n, train)
    xadj, adj = csr.xadj.numpy().astype(np.int64), csr.adj.numpy()
    sets = make_eval_sets(n, train.numpy(), test.numpy(), seed=1)
    M = O.init_embedding(n, 32, 1, 0)
    O.train_level(xadj, adj, M, 3, 0.025, 100, 1, 0)
    held, fit = aucroc(M, sets)
    assert abs(held - 0.5) < 0.05
    assert fit > 0.68, fit
