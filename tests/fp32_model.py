"""A CPU model of the ARITHMETIC of the sequential-order kernel, for tests that reason about
rounding: fp32 rows, the dot product as per-lane fused multiply-add chains joined by a
butterfly tree over the lanes, the sigmoid in fp32, the two axpys as fused multiply-adds.
It is not the oracle (which does every update in fp64 on the fp32-stored rows) and not the
kernel (it shares no code with it): it exists to tell accumulated fp32 rounding, which it
reproduces in kind and size, from an ordering or indexing mistake, which it cannot make.
numpy only; slow (tens of microseconds per update)."""
from __future__ import annotations

import numpy as np

F32 = np.float32


def _fma(a, b, c):
    """round32(a * b + c): the product of two fp32 values is exact in fp64."""
    return (a.astype(np.float64) * b.astype(np.float64) + c.astype(np.float64)).astype(F32)


def lanes_for(d):
    """Plain 128-bit layout of the sequential-order mode: lanes, units per lane."""
    units = d // 4
    lanes = 1
    while lanes < units and lanes < 64:
        lanes *= 2
    return lanes, (2 if d > 256 else 1)


def dot_tree(s, r, lanes, upl):
    """The kernel's dot product: lane g owns floats (g + i*lanes)*4 .. +4 for i < upl, chains
    them with fused multiply-adds, then the lanes are summed pairwise (lane ^ 1, ^ 2, ...)."""
    d = s.size
    pad = lanes * upl * 4
    a = np.zeros(pad, dtype=F32)
    b = np.zeros(pad, dtype=F32)
    a[:d] = s
    b[:d] = r
    a = a.reshape(upl, lanes, 4)
    b = b.reshape(upl, lanes, 4)
    partial = np.zeros(lanes, dtype=F32)
    for i in range(upl):
        for c in range(4):
            partial = _fma(a[i, :, c], b[i, :, c], partial)
    step = 1
    idx = np.arange(lanes)
    while step < lanes:
        partial = (partial + partial[idx ^ step]).astype(F32)
        step *= 2
    return partial[0]


def update_fp32(s, r, label, lr, lanes, upl):
    """Alg. 1 in the kernel's precision, in place on two fp32 rows."""
    x = dot_tree(s, r, lanes, upl)
    with np.errstate(over="ignore"):  # exp overflows to inf for x << 0: the sigmoid is then 0, as on the device
        sig = F32(1.0) / (F32(1.0) + np.exp(-x, dtype=F32))
    g = F32(lr) * (F32(label) - sig)
    gv = np.full(s.size, g, dtype=F32)
    s[:] = _fma(gv, r, s)
    r[:] = _fma(gv, s, r)


def replay(M, triples, lr):
    """Applies (src, sample, label) triples in order to the fp32 matrix M."""
    lanes, upl = lanes_for(M.shape[1])
    for src, v, label in triples:
        if v < 0 or v == src:
            continue
        update_fp32(M[src], M[v], label, lr, lanes, upl)
