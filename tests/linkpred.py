"""Link-prediction evaluation of an embedding (Sec. 4.1 of the paper), used by the tests.

Train and test edge sets come from ``graphgen.holdout_split``.  Test edges with an
endpoint that is isolated in the training graph are dropped; each positive set is
balanced with as many non-edges; features are element-wise products of the two
endpoint rows; a logistic-regression classifier is fitted on the training pairs
and AUCROC is reported on the test pairs.
"""
from __future__ import annotations

import numpy as np
from sklearn.linear_model import LogisticRegression
from sklearn.metrics import roc_auc_score


def _non_edges(n, forbidden, count, rng, vertices):
    out = []
    while len(out) < count:
        u = vertices[rng.integers(0, vertices.size, size=2 * count)]
        v = vertices[rng.integers(0, vertices.size, size=2 * count)]
        for a, b in zip(u.tolist(), v.tolist()):
            if a == b:
                continue
            key = (min(a, b), max(a, b))
            if key in forbidden:
                continue
            out.append(key)
            if len(out) == count:
                break
    return np.asarray(out, dtype=np.int64)


def make_eval_sets(n, train_edges, test_edges, seed=0):
    """Positive/negative vertex pairs for classifier training and testing."""
    train = np.asarray(train_edges, dtype=np.int64)
    test = np.asarray(test_edges, dtype=np.int64)
    deg = np.bincount(train.ravel(), minlength=n)
    test = test[(deg[test[:, 0]] > 0) & (deg[test[:, 1]] > 0)]
    vertices = np.nonzero(deg > 0)[0]
    forbidden = {(int(a), int(b)) for a, b in train} | {(int(a), int(b)) for a, b in test}
    rng = np.random.default_rng(seed)
    neg_train = _non_edges(n, forbidden, len(train), rng, vertices)
    neg_test = _non_edges(n, forbidden, len(test), rng, vertices)
    return dict(pos_train=train, neg_train=neg_train, pos_test=test, neg_test=neg_test)


def _features(M, pairs):
    return M[pairs[:, 0]].astype(np.float64) * M[pairs[:, 1]].astype(np.float64)


def aucroc(M, sets, max_train=200000, seed=0):
    """(held-out AUCROC, AUCROC on the training pairs themselves)."""
    rng = np.random.default_rng(seed)
    pt, nt = sets["pos_train"], sets["neg_train"]
    if len(pt) > max_train:
        pt = pt[rng.choice(len(pt), max_train, replace=False)]
        nt = nt[rng.choice(len(nt), max_train, replace=False)]
    Xtr = np.vstack((_features(M, pt), _features(M, nt)))
    ytr = np.concatenate((np.ones(len(pt)), np.zeros(len(nt))))
    # Hub rows of a power-law graph can be orders of magnitude longer than the rest, so
    # the features are standardised per column (statistics of the training pairs) and
    # clipped; otherwise a handful of pairs sets the scale and the classifier sees zeros.
    mean = Xtr.mean(axis=0)
    std = np.maximum(Xtr.std(axis=0), 1e-30)
    prep = lambda X: np.clip((X - mean) / std, -10.0, 10.0)
    clf = LogisticRegression(max_iter=500, C=1.0)
    clf.fit(prep(Xtr), ytr)
    Xte = np.vstack((_features(M, sets["pos_test"]), _features(M, sets["neg_test"])))
    yte = np.concatenate((np.ones(len(sets["pos_test"])), np.zeros(len(sets["neg_test"]))))
    held = roc_auc_score(yte, clf.decision_function(prep(Xte)))
    fit = roc_auc_score(ytr, clf.decision_function(prep(Xtr)))
    return float(held), float(fit)
