"""ctypes access to the C++ oracle (numpy arrays in, numpy arrays out).

Test infrastructure: see the header of gosh_oracle.cpp.  The library is built by
``oracle/build.py``; it is loaded lazily and built on first use if missing.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build()
        L = C.CDLL(path)
        u32p, i32p, i64p, f32p = (C.POINTER(C.c_uint32), C.POINTER(C.c_int32),
                                  C.POINTER(C.c_int64), C.POINTER(C.c_float))
        L.orc_philox4x32_10.argtypes = [u32p, u32p, u32p]
        L.orc_philox4x32_10.restype = None
        L.orc_draw.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32]
        L.orc_draw.restype = C.c_uint64
        L.orc_bounded.argtypes = [C.c_uint64, C.c_uint64]
        L.orc_bounded.restype = C.c_uint64
        L.orc_sample_epoch.argtypes = [C.c_int64, i64p, i32p, C.c_int32, C.c_uint64,
                                       C.c_uint32, C.c_uint32, i32p]
        L.orc_sample_epoch.restype = None
        L.orc_sample_source.argtypes = [C.c_int64, i64p, i32p, C.c_int32, C.c_uint64,
                                        C.c_uint32, C.c_uint32, C.c_int64, i32p]
        L.orc_sample_source.restype = None
        L.orc_update.argtypes = [f32p, f32p, C.c_int32, C.c_int32, C.c_float]
        L.orc_update.restype = None
        L.orc_lr.argtypes = [C.c_float, C.c_int64, C.c_int64]
        L.orc_lr.restype = C.c_float
        L.orc_train_epoch.argtypes = [C.c_int64, i64p, i32p, f32p, C.c_int32, C.c_int32,
                                      C.c_float, C.c_uint64, C.c_uint32, C.c_uint32]
        L.orc_train_epoch.restype = None
        L.orc_train_sources.argtypes = [C.c_int64, i64p, i32p, f32p, C.c_int32, C.c_int32,
                                        C.c_float, C.c_uint64, C.c_uint32, C.c_uint32,
                                        C.c_int64, C.c_int64]
        L.orc_train_sources.restype = None
        L.orc_train_sources_hogwild.argtypes = [C.c_int64, i64p, i32p, f32p, C.c_int32, C.c_int32,
                                                C.c_float, C.c_uint64, C.c_uint32, C.c_uint32,
                                                C.c_int64, C.c_int64, C.c_int32]
        L.orc_train_sources_hogwild.restype = None
        L.orc_init_rows.argtypes = [f32p, C.c_int64, C.c_int64, C.c_int32, C.c_uint64,
                                    C.c_uint32]
        L.orc_init_rows.restype = None
        L.orc_train_level.argtypes = [C.c_int64, i64p, i32p, f32p, C.c_int32, C.c_int32,
                                      C.c_float, C.c_int64, C.c_uint64, C.c_uint32]
        L.orc_train_level.restype = None
        L.orc_init_embedding.argtypes = [f32p, C.c_int64, C.c_int32, C.c_uint64, C.c_uint32]
        L.orc_init_embedding.restype = None
        L.orc_project.argtypes = [f32p, i32p, C.c_int64, C.c_int32, f32p]
        L.orc_project.restype = None
        L.orc_epoch_split.argtypes = [C.c_int64, C.c_double, C.c_int32, i64p]
        L.orc_epoch_split.restype = C.c_int
        L.orc_coarsen_map.argtypes = [C.c_int64, i64p, i32p, i32p]
        L.orc_coarsen_map.restype = C.c_int64
        L.orc_coarsen_graph.argtypes = [C.c_int64, i64p, i32p, i64p, i32p, C.c_int64,
                                        i64p, i32p, i64p]
        L.orc_coarsen_graph.restype = C.c_int64
        L.orc_pair_order.argtypes = [C.c_int32, i32p, i32p]
        L.orc_pair_order.restype = C.c_int64
        L.orc_pair_order_blocked.argtypes = [C.c_int32, C.c_int32, i32p, i32p]
        L.orc_pair_order_blocked.restype = C.c_int64
        L.orc_train_pair.argtypes = [C.c_int64, i64p, i32p, f32p, C.c_int32, C.c_int32,
                                     C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_float,
                                     C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, i32p]
        L.orc_train_pair.restype = None
        L.orc_rotations.argtypes = [C.c_int64, C.c_int32, C.c_int32]
        L.orc_rotations.restype = C.c_int64
        L.orc_train_parts.argtypes = [C.c_int64, i64p, i32p, f32p, C.c_int32, C.c_int32,
                                      C.c_int64, C.c_float, C.c_uint64, C.c_uint32, C.c_int32,
                                      C.c_int32, C.c_int32]
        L.orc_train_parts.restype = None
        _lib = L
    return _lib


def _p(a, ctype):
    return a.ctypes.data_as(C.POINTER(ctype)) if a is not None else None


def _csr(xadj, adj):
    xadj = np.ascontiguousarray(np.asarray(xadj), dtype=np.int64)
    adj = np.ascontiguousarray(np.asarray(adj), dtype=np.int32)
    return xadj, adj


def philox(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_p(c, C.c_uint32), _p(k, C.c_uint32), _p(out, C.c_uint32))
    return out


def draw(seed, src, j, epoch, level):
    return int(lib().orc_draw(seed, src, j, epoch, level))


def bounded(r, bound):
    return int(lib().orc_bounded(r, bound))


def sample_epoch(xadj, adj, k, seed, epoch, level):
    xadj, adj = _csr(xadj, adj)
    n = xadj.size - 1
    out = np.empty((n, k + 1), dtype=np.int32)
    lib().orc_sample_epoch(n, _p(xadj, C.c_int64), _p(adj, C.c_int32), k, seed, epoch, level,
                           _p(out, C.c_int32))
    return out


def sample_source(xadj, adj, k, seed, epoch, level, src):
    xadj, adj = _csr(xadj, adj)
    out = np.empty(k + 1, dtype=np.int32)
    lib().orc_sample_source(xadj.size - 1, _p(xadj, C.c_int64), _p(adj, C.c_int32), k, seed,
                            epoch, level, src, _p(out, C.c_int32))
    return out


def update(m_v, m_sample, b, lr):
    """Apply Alg. 1 in place to two fp32 rows (numpy arrays)."""
    assert m_v.dtype == np.float32 and m_sample.dtype == np.float32
    lib().orc_update(_p(m_v, C.c_float), _p(m_sample, C.c_float), m_v.size, b, lr)


def lr(lr0, j, e_i):
    return float(lib().orc_lr(lr0, j, e_i))


def train_epoch(xadj, adj, M, k, lr_epoch, seed, epoch, level):
    """One sequential epoch, in place on the fp32 matrix M (n x d, C-contiguous)."""
    xadj, adj = _csr(xadj, adj)
    assert M.dtype == np.float32 and M.flags.c_contiguous
    n, d = M.shape
    assert n == xadj.size - 1
    lib().orc_train_epoch(n, _p(xadj, C.c_int64), _p(adj, C.c_int32), _p(M, C.c_float), d, k,
                          lr_epoch, seed, epoch, level)


def train_sources(xadj, adj, M, k, lr_epoch, seed, epoch, level, first, count):
    """Sources first..first+count-1 of one sequential epoch, in place on M."""
    xadj, adj = _csr(xadj, adj)
    assert M.dtype == np.float32 and M.flags.c_contiguous
    n, d = M.shape
    lib().orc_train_sources(n, _p(xadj, C.c_int64), _p(adj, C.c_int32), _p(M, C.c_float), d, k,
                            lr_epoch, seed, epoch, level, first, count)


def train_sources_hogwild(xadj, adj, M, k, lr_epoch, seed, epoch, level, first, count, threads):
    """The same slice spread lock-free over `threads` threads (the paper's multi-core CPU
    baseline): for timing and quality checks only, its result depends on the interleaving."""
    xadj, adj = _csr(xadj, adj)
    assert M.dtype == np.float32 and M.flags.c_contiguous
    n, d = M.shape
    lib().orc_train_sources_hogwild(n, _p(xadj, C.c_int64), _p(adj, C.c_int32), _p(M, C.c_float), d,
                                    k, lr_epoch, seed, epoch, level, first, count, threads)


def init_rows(first, count, d, seed, level):
    out = np.empty((count, d), dtype=np.float32)
    lib().orc_init_rows(_p(out, C.c_float), first, count, d, seed, level)
    return out


def train_level(xadj, adj, M, k, lr0, e_i, seed, level):
    xadj, adj = _csr(xadj, adj)
    assert M.dtype == np.float32 and M.flags.c_contiguous
    n, d = M.shape
    lib().orc_train_level(n, _p(xadj, C.c_int64), _p(adj, C.c_int32), _p(M, C.c_float), d, k,
                          lr0, e_i, seed, level)


def init_embedding(n, d, seed, level):
    M = np.empty((n, d), dtype=np.float32)
    lib().orc_init_embedding(_p(M, C.c_float), n, d, seed, level)
    return M


def project(M_coarse, map_):
    map_ = np.ascontiguousarray(map_, dtype=np.int32)
    assert M_coarse.dtype == np.float32 and M_coarse.flags.c_contiguous
    out = np.empty((map_.size, M_coarse.shape[1]), dtype=np.float32)
    lib().orc_project(_p(M_coarse, C.c_float), _p(map_, C.c_int32), map_.size,
                      M_coarse.shape[1], _p(out, C.c_float))
    return out


def epoch_split(e, p, D):
    out = np.zeros(D, dtype=np.int64)
    rc = lib().orc_epoch_split(e, p, D, _p(out, C.c_int64))
    if rc != 0:
        raise ValueError("epoch budget cannot cover every level")
    return out


def coarsen_map(xadj, adj):
    xadj, adj = _csr(xadj, adj)
    n = xadj.size - 1
    m = np.empty(n, dtype=np.int32)
    nc = lib().orc_coarsen_map(n, _p(xadj, C.c_int64), _p(adj, C.c_int32), _p(m, C.c_int32))
    return m, int(nc)


def coarsen_graph(xadj, adj, map_, n_coarse, mult=None):
    xadj, adj = _csr(xadj, adj)
    n = xadj.size - 1
    map_ = np.ascontiguousarray(map_, dtype=np.int32)
    if mult is not None:
        mult = np.ascontiguousarray(mult, dtype=np.int64)
    nnz = lib().orc_coarsen_graph(n, _p(xadj, C.c_int64), _p(adj, C.c_int32),
                                  _p(mult, C.c_int64), _p(map_, C.c_int32), n_coarse,
                                  None, None, None)
    xo = np.zeros(n_coarse + 1, dtype=np.int64)
    ao = np.zeros(nnz, dtype=np.int32)
    mo = np.zeros(nnz, dtype=np.int64)
    lib().orc_coarsen_graph(n, _p(xadj, C.c_int64), _p(adj, C.c_int32), _p(mult, C.c_int64),
                            _p(map_, C.c_int32), n_coarse, _p(xo, C.c_int64),
                            _p(ao, C.c_int32), _p(mo, C.c_int64))
    return xo, ao, mo


def coarsen(xadj, adj, threshold=100, min_shrink=0.8, max_levels=64):
    """Alg. 4 outer loop.  READING (stop rule): build G_{i+1} while |V_i| > threshold;
    after building it, stop if |V_{i+1}| > min_shrink * |V_i| (the level barely
    shrank; it is still kept as the last one).  A level that merged nothing
    (|V_{i+1}| == |V_i|, e.g. only isolated vertices are left) would repeat G_i and is
    not kept.  max_levels caps the number of graphs.
    Returns (graphs, maps, mults): graphs[i] = (xadj, adj) of G_i, maps[i]: V_i -> V_{i+1}."""
    xadj, adj = _csr(xadj, adj)
    graphs, maps, mults = [(xadj, adj)], [], [np.ones(adj.size, dtype=np.int64)]
    while graphs[-1][0].size - 1 > threshold and len(graphs) < max_levels:
        x, a = graphs[-1]
        n = x.size - 1
        m, nc = coarsen_map(x, a)
        if nc == n:
            break
        xo, ao, mo = coarsen_graph(x, a, m, nc, mults[-1])
        graphs.append((xo, ao))
        maps.append(m)
        mults.append(mo)
        if nc > min_shrink * n:
            break
    return graphs, maps, mults


def passes_per_epoch(xadj, adj):
    """Sec. 4.3 (experimental setup): the experiments call |E| sampled sources one epoch,
    while one pass of Alg. 3 samples |V|.  READING: the smallest whole number of passes
    that samples at least |E| = nnz/2 sources (at least one)."""
    n = xadj.size - 1
    edges = adj.size // 2
    passes = 1
    while passes * n < edges:
        passes += 1
    return passes


def embed(xadj, adj, d, k, epochs, p, lr0, seed, threshold=100, min_shrink=1.0, max_levels=64,
          edge_epochs=False, parts_K=None):
    """Alg. 2: coarsen, initialise M_{D-1}, then for i = D-1..0 train e_i epochs on G_i and
    (i > 0) project to G_{i-1}.  READING: the printed loop bound "D-1 to 1" would never
    train G_0; the text trains until M_0 is obtained.  With edge_epochs an epoch is the
    experiments' (Sec. 4.3): level i runs e_i * passes_per_epoch(G_i) passes of Alg. 3.
    parts_K (not the paper's: Alg. 2 trains a level that fits with Alg. 3): one entry per
    level, given by the caller; level i runs Alg. 5 on parts_K[i] parts with B = 5 where the
    entry is non-zero, Alg. 3 otherwise.
    Returns (M_0, graphs, maps, passes run per level)."""
    graphs, maps, _ = coarsen(xadj, adj, threshold, min_shrink, max_levels)
    D = len(graphs)
    e_i = epoch_split(epochs, p, D)
    if edge_epochs:
        e_i = np.array([int(e_i[i]) * passes_per_epoch(*graphs[i]) for i in range(D)], dtype=np.int64)
    M = init_embedding(graphs[-1][0].size - 1, d, seed, D - 1)
    for i in range(D - 1, -1, -1):
        K = int(parts_K[i]) if parts_K is not None else 0
        if K:
            train_parts(graphs[i][0], graphs[i][1], M, k, int(e_i[i]), lr0, seed, i, K, 5)
        else:
            train_level(graphs[i][0], graphs[i][1], M, k, lr0, int(e_i[i]), seed, i)
        if i > 0:
            M = project(M, maps[i - 1])
    return M, graphs, maps, e_i


def parts_split(n, d, budget, P_gpu, S_gpu, B):
    """READING (number of parts; the paper leaves GetEmbeddingPartInfo open): the smallest
    K for which min(P_gpu, K) part slots of ceil(n/K) rows, S_gpu pools of 2*ceil(n/K)*B
    ids and one bit per vertex fit the budget."""
    K = 1
    while True:
        ps = -(-n // K)
        need = min(P_gpu, K) * ps * d * 4 + S_gpu * 2 * ps * B * 4 + ((n + 63) // 64) * 8
        if need <= budget:
            return K
        K += 1
        if K > n:
            raise ValueError("budget too small")


def embed_budget(xadj, adj, d, k, epochs, p, lr0, seed, budget, P_gpu=3, S_gpu=4, B=5,
                 threshold=100, min_shrink=1.0, offsets64=False, blocked=False, max_levels=64):
    """Alg. 2 with its "fits into GPU" test: a level whose graph (offsets + adj) and matrix
    exceed `budget` bytes is trained with the rotation of Alg. 5, the others with Alg. 3.
    Coarse levels have 64-bit offsets; level 0 as given.  Returns (M_0, modes) where
    modes[i] is 0 or the K used."""
    graphs, maps, _ = coarsen(xadj, adj, threshold, min_shrink, max_levels)
    D = len(graphs)
    e_i = epoch_split(epochs, p, D)
    M = init_embedding(graphs[-1][0].size - 1, d, seed, D - 1)
    modes = [0] * D
    for i in range(D - 1, -1, -1):
        x, a = graphs[i]
        n = x.size - 1
        off = 8 if (i > 0 or offsets64) else 4
        size = (n + 1) * off + a.size * 4 + n * d * 4
        if size <= budget:
            train_level(x, a, M, k, lr0, int(e_i[i]), seed, i)
        else:
            K = parts_split(n, d, budget, P_gpu, S_gpu, B)
            modes[i] = K
            train_parts(x, a, M, k, int(e_i[i]), lr0, seed, i, K, B,
                        block=blocked_block_size(P_gpu, K) if blocked else 0)
        if i > 0:
            M = project(M, maps[i - 1])
    return M, modes


def pair_order(K):
    npairs = K * (K + 1) // 2
    a = np.zeros(npairs, dtype=np.int32)
    b = np.zeros(npairs, dtype=np.int32)
    cnt = lib().orc_pair_order(K, _p(a, C.c_int32), _p(b, C.c_int32))
    assert cnt == npairs
    return list(zip(a.tolist(), b.tolist()))


def blocked_block_size(P_gpu, K):
    """Block size of the blocked order for a device with P_gpu part slots: all slots but two
    (the two take turns receiving the streamed parts), at least one."""
    return max(1, min(P_gpu, K) - 2)


def pair_order_blocked(K, R):
    npairs = K * (K + 1) // 2
    a = np.zeros(npairs, dtype=np.int32)
    b = np.zeros(npairs, dtype=np.int32)
    cnt = lib().orc_pair_order_blocked(K, R, _p(a, C.c_int32), _p(b, C.c_int32))
    assert cnt == npairs
    return list(zip(a.tolist(), b.tolist()))


def rotations(e_i, B, K):
    return int(lib().orc_rotations(e_i, B, K))


def train_pair(xadj, adj, M, k, B, K, pa, pb, lr_, seed, rotation, level, pair_index,
               want_stream=False):
    xadj, adj = _csr(xadj, adj)
    n, d = M.shape
    stream = None
    if want_stream:
        ps = (n + K - 1) // K
        cnt = 0
        for part in ([pa] if pa == pb else [pa, pb]):
            lo = min(n, part * ps)
            cnt += min(n, lo + ps) - lo
        stream = np.full(cnt * B * (k + 1), -2, dtype=np.int32)
    lib().orc_train_pair(n, _p(xadj, C.c_int64), _p(adj, C.c_int32), _p(M, C.c_float), d, k, B,
                         K, pa, pb, lr_, seed, rotation, level, pair_index,
                         _p(stream, C.c_int32))
    return stream


def train_parts(xadj, adj, M, k, e_i, lr0, seed, level, K, B, block=0):
    """Alg. 5, sequentially.  block = 0: the paper's visiting order; block = R > 0: the
    blocked order with blocks of R parts."""
    xadj, adj = _csr(xadj, adj)
    n, d = M.shape
    lib().orc_train_parts(n, _p(xadj, C.c_int64), _p(adj, C.c_int32), _p(M, C.c_float), d, k,
                          e_i, lr0, seed, level, K, B, block)
