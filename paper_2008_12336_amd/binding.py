"""Thin ctypes binding of libgosh: same names as the C ABI, argument marshalling only.

Tensors are torch tensors used purely as handles to device (or host) memory; every
step of the training path runs inside the library's HIP kernels.  There is no CPU
fallback: if the shared library is missing, loading fails with an error.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgosh.so")

GOSH_FLAG_SEQUENTIAL = 1
GOSH_FLAG_PLAIN_STORES = 2
GOSH_FLAG_ATOMIC_ADDS = 4
GOSH_FLAG_EDGE_EPOCHS = 8
GOSH_FLAG_BLOCKED_ORDER = 16
GOSH_FLAG_PAIR_LEVELS = 32
GOSH_FLAG_CONCURRENT_LAYOUT = 64
GOSH_EDIVERGED = -5
GOSH_MAX_DIM = 512
GOSH_MAX_NEG = 15
GOSH_STATIC_MAX_N = 1 << 26


class GoshError(RuntimeError):
    """A negative status of the library.  `stats` carries the statistics the call filled in
    before it failed (GOSH_EDIVERGED: all of them), else None."""

    def __init__(self, code: int, message: str, stats=None):
        super().__init__(f"libgosh error {code}: {message}")
        self.code = code
        self.stats = stats


class gosh_csr(C.Structure):
    _fields_ = [("n", C.c_int64), ("nnz", C.c_int64), ("xadj", C.c_void_p),
                ("adj", C.c_void_p), ("xadj_is64", C.c_int32)]


class gosh_level_stats(C.Structure):
    _fields_ = [("level", C.c_int32), ("n", C.c_int64), ("nnz", C.c_int64), ("epochs", C.c_int64),
                ("upload_ms", C.c_double), ("train_ms", C.c_double), ("project_ms", C.c_double),
                ("parts_K", C.c_int32), ("max_abs", C.c_float), ("nonfinite", C.c_int64)]


class gosh_parts_stats(C.Structure):
    _fields_ = [("K", C.c_int32), ("rotations", C.c_int64), ("pair_visits", C.c_int64),
                ("updates", C.c_int64), ("device_bytes", C.c_uint64), ("bytes_h2d", C.c_uint64),
                ("bytes_d2h", C.c_uint64), ("kernel_ms", C.c_double), ("wall_ms", C.c_double),
                ("sampler_ms", C.c_double), ("sampler_wait_ms", C.c_double), ("max_abs", C.c_float),
                ("nonfinite", C.c_int64)]


class gosh_tuning(C.Structure):
    _fields_ = [("plain_rows", C.c_int32), ("max_waves", C.c_int64), ("hot_inv_eps", C.c_int64),
                ("hot_all_inv_eps", C.c_int64), ("hot_min_degree", C.c_int64),
                ("pair_level_min_n", C.c_int64)]


class gosh_placement_info(C.Structure):
    _fields_ = [("arena_bytes", C.c_uint64), ("window_offset_bytes", C.c_uint64), ("kept_bytes", C.c_uint64),
                ("probes", C.c_int32), ("probe_ms_best", C.c_float), ("probe_ms_median", C.c_float),
                ("search_ms", C.c_double)]


EXPORTS = {
    "gosh_last_error": (C.c_char_p, []),
    "gosh_tuning_defaults": (None, [C.POINTER(gosh_tuning)]),
    "gosh_set_tuning": (C.c_int, [C.POINTER(gosh_tuning)]),
    "gosh_get_tuning": (C.c_int, [C.POINTER(gosh_tuning)]),
    "gosh_pair_level_parts": (C.c_int32, [C.c_int64, C.c_int64, C.c_int64, C.c_int32]),
    "gosh_matrix_check": (C.c_int, [C.c_void_p, C.c_int64, C.c_int32, C.POINTER(C.c_float),
                                    C.POINTER(C.c_int64), C.c_void_p]),
    "gosh_lr": (C.c_float, [C.c_float, C.c_int64, C.c_int64]),
    "gosh_epoch_split": (C.c_int, [C.c_int64, C.c_double, C.c_int32, C.POINTER(C.c_int64)]),
    "gosh_csr_validate": (C.c_int, [C.POINTER(gosh_csr)]),
    "gosh_coarsen": (C.c_int, [C.POINTER(gosh_csr), C.c_int64, C.c_double, C.c_int32, C.c_int32,
                               C.POINTER(C.c_void_p)]),
    "gosh_coarsen_device": (C.c_int, [C.POINTER(gosh_csr), C.c_int64, C.c_double, C.c_int32,
                                      C.c_int32, C.POINTER(C.c_void_p)]),
    "gosh_hierarchy_release_device": (C.c_int, [C.c_void_p]),
    "gosh_hierarchy_trim_scratch": (C.c_int, [C.c_void_p]),
    "gosh_hierarchy_levels": (C.c_int, [C.c_void_p]),
    "gosh_hierarchy_shape": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_int64),
                                       C.POINTER(C.c_int64)]),
    "gosh_hierarchy_graph": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(gosh_csr)]),
    "gosh_hierarchy_map": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.POINTER(C.c_int32)),
                                     C.POINTER(C.c_int64)]),
    "gosh_hierarchy_mult": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.POINTER(C.c_int64)),
                                      C.POINTER(C.c_int64)]),
    "gosh_hierarchy_times": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_double)]),
    "gosh_hierarchy_free": (None, [C.c_void_p]),
    "gosh_init_embedding": (C.c_int, [C.c_void_p, C.c_int64, C.c_int32, C.c_uint64, C.c_uint32,
                                      C.c_void_p]),
    "gosh_sample_epoch": (C.c_int, [C.POINTER(gosh_csr), C.c_int32, C.c_uint64, C.c_uint32,
                                    C.c_uint32, C.c_void_p, C.c_void_p]),
    "gosh_train_epoch": (C.c_int, [C.POINTER(gosh_csr), C.c_void_p, C.c_int32, C.c_int32,
                                   C.c_float, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32,
                                   C.c_void_p]),
    "gosh_train_epoch_static": (C.c_int, [C.POINTER(gosh_csr), C.c_void_p, C.c_int32, C.c_int32,
                                          C.c_float, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32,
                                          C.c_void_p]),
    "gosh_embed": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int64, C.c_double, C.c_float,
                             C.c_uint64, C.c_uint32, C.c_uint64, C.c_void_p,
                             C.POINTER(gosh_level_stats), C.c_void_p]),
    "gosh_pair_order": (C.c_int, [C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "gosh_pair_order_blocked": (C.c_int, [C.c_int32, C.c_int32, C.POINTER(C.c_int32),
                                          C.POINTER(C.c_int32)]),
    "gosh_parts_plan": (C.c_int, [C.c_int64, C.c_int32, C.c_int64, C.c_uint64, C.c_int32, C.c_int32,
                                  C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int64),
                                  C.POINTER(C.c_uint64)]),
    "gosh_parts_sample_pair": (C.c_int, [C.POINTER(gosh_csr), C.c_int32, C.c_int32, C.c_int32,
                                         C.c_int32, C.c_int32, C.c_uint64, C.c_uint32, C.c_uint32,
                                         C.c_uint32, C.c_void_p]),
    "gosh_train_parts": (C.c_int, [C.POINTER(gosh_csr), C.c_void_p, C.c_int32, C.c_int32, C.c_int64,
                                   C.c_float, C.c_uint64, C.c_uint32, C.c_uint64, C.c_int32,
                                   C.c_int32, C.c_int32, C.c_int32, C.c_uint32,
                                   C.POINTER(gosh_parts_stats)]),
    "gosh_embed_host": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int64, C.c_double, C.c_float,
                                  C.c_uint64, C.c_uint32, C.c_uint64, C.c_int32, C.c_int32, C.c_int32,
                                  C.c_void_p, C.POINTER(gosh_level_stats), C.c_void_p]),
    "gosh_project": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int32,
                               C.c_void_p, C.c_void_p]),
    "gosh_row_probe": (C.c_int, [C.c_void_p, C.c_int64, C.c_int32, C.c_int64, C.c_uint64, C.c_int32,
                                 C.c_void_p]),
    "gosh_matrix_place": (C.c_int, [C.c_int64, C.c_int32, C.c_uint64, C.POINTER(C.c_void_p),
                                    C.POINTER(gosh_placement_info)]),
    "gosh_matrix_release": (C.c_int, [C.c_void_p]),
}

_lib = None


def lib() -> C.CDLL:
    """Load libgosh.so (built by ``paper_2008_12336_amd.build``); fail loudly if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2008_12336_amd.build` "
                "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def _check(rc: int, stats=None) -> None:
    if rc != 0:
        raise GoshError(rc, lib().gosh_last_error().decode(), stats() if (stats and rc == GOSH_EDIVERGED) else None)


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def csr_view(n: int, xadj: torch.Tensor, adj: torch.Tensor) -> gosh_csr:
    """Describe CSR tensors (both on the same device, contiguous) to the library."""
    if xadj.dtype not in (torch.int32, torch.int64) or adj.dtype != torch.int32:
        raise TypeError("xadj must be int32/int64 and adj int32")
    if xadj.numel() != n + 1 or not xadj.is_contiguous() or not adj.is_contiguous():
        raise ValueError("xadj must hold n+1 contiguous offsets, adj must be contiguous")
    view = gosh_csr(n, adj.numel(), xadj.data_ptr(), adj.data_ptr() if adj.numel() else None,
                    1 if xadj.dtype == torch.int64 else 0)
    view._tensors = (xadj, adj)  # the view holds raw pointers: keep their memory alive with it
    return view


def _matrix(M: torch.Tensor, name: str):
    if M.dtype != torch.float32 or M.dim() != 2 or not M.is_contiguous():
        raise TypeError(f"{name} must be a contiguous 2-D float32 tensor")
    return M.data_ptr(), M.shape[0], M.shape[1]


def gosh_last_error() -> str:
    return lib().gosh_last_error().decode()


def gosh_tuning_defaults() -> dict:
    t = gosh_tuning()
    lib().gosh_tuning_defaults(C.byref(t))
    return {name: getattr(t, name) for name, _ in gosh_tuning._fields_}


def gosh_get_tuning() -> dict:
    t = gosh_tuning()
    _check(lib().gosh_get_tuning(C.byref(t)))
    return {name: getattr(t, name) for name, _ in gosh_tuning._fields_}


def gosh_set_tuning(**fields) -> None:
    """Set the named fields of the process-wide tuning record; the others return to their
    defaults.  No arguments: everything back to the defaults."""
    if not fields:
        _check(lib().gosh_set_tuning(None))
        return
    t = gosh_tuning()
    lib().gosh_tuning_defaults(C.byref(t))
    for name, value in fields.items():
        if name not in dict(gosh_tuning._fields_):
            raise TypeError(f"gosh_tuning has no field {name!r}")
        setattr(t, name, value)
    _check(lib().gosh_set_tuning(C.byref(t)))


def gosh_pair_level_parts(epochs: int, n: int, min_n: int, B: int = 5) -> int:
    return int(lib().gosh_pair_level_parts(epochs, n, min_n, B))


def gosh_matrix_check(M: torch.Tensor, stream=None):
    """(largest finite |entry|, number of non-finite entries) of a device matrix."""
    ptr, n, d = _matrix(M, "M")
    top, bad = C.c_float(), C.c_int64()
    _check(lib().gosh_matrix_check(ptr, n, d, C.byref(top), C.byref(bad), _stream(stream)))
    return float(top.value), int(bad.value)


def gosh_lr(lr0: float, j: int, e_i: int) -> float:
    return float(lib().gosh_lr(lr0, j, e_i))


def gosh_epoch_split(e: int, p: float, D: int):
    out = (C.c_int64 * max(D, 1))()
    _check(lib().gosh_epoch_split(e, p, D, out))
    return [int(x) for x in out[:D]]


def gosh_init_embedding(M: torch.Tensor, seed: int, level: int = 0, stream=None) -> None:
    ptr, n, d = _matrix(M, "M")
    _check(lib().gosh_init_embedding(ptr, n, d, seed, level, _stream(stream)))


def gosh_sample_epoch(g: gosh_csr, k_neg: int, seed: int, epoch: int, level: int,
                      out: torch.Tensor, stream=None) -> None:
    if out.dtype != torch.int32 or not out.is_contiguous() or out.numel() != g.n * (k_neg + 1):
        raise TypeError("out must be a contiguous int32 tensor of n*(k_neg+1) entries")
    _check(lib().gosh_sample_epoch(C.byref(g), k_neg, seed, epoch, level, out.data_ptr(),
                                   _stream(stream)))


def gosh_train_epoch(g: gosh_csr, M: torch.Tensor, k_neg: int, lr_epoch: float, seed: int,
                     epoch: int, level: int = 0, flags: int = 0, stream=None) -> None:
    ptr, n, d = _matrix(M, "M")
    if n != g.n:
        raise ValueError("M must have one row per vertex")
    _check(lib().gosh_train_epoch(C.byref(g), ptr, d, k_neg, lr_epoch, seed, epoch, level, flags,
                                  _stream(stream)))


def gosh_train_epoch_static(g: gosh_csr, M: torch.Tensor, k_neg: int, lr_epoch: float, seed: int,
                            epoch: int, level: int = 0, flags: int = 0, stream=None) -> None:
    """gosh_train_epoch without any allocation (fixed in-library bitmap, n <= 2^26)."""
    ptr, n, d = _matrix(M, "M")
    if n != g.n:
        raise ValueError("M must have one row per vertex")
    _check(lib().gosh_train_epoch_static(C.byref(g), ptr, d, k_neg, lr_epoch, seed, epoch, level, flags,
                                         _stream(stream)))


def gosh_project(M_coarse: torch.Tensor, map_: torch.Tensor, M_fine: torch.Tensor,
                 stream=None) -> None:
    cptr, nc, d = _matrix(M_coarse, "M_coarse")
    fptr, nf, d2 = _matrix(M_fine, "M_fine")
    if d != d2 or map_.dtype != torch.int32 or map_.numel() != nf or not map_.is_contiguous():
        raise TypeError("map must be int32 with one entry per fine vertex; dims must agree")
    _check(lib().gosh_project(cptr, nc, map_.data_ptr(), nf, d, fptr, _stream(stream)))


GOSH_PROBE_READ_WRITE, GOSH_PROBE_READ, GOSH_PROBE_WRITE, GOSH_PROBE_EPOCH_MIX = 0, 1, 2, 3


def gosh_row_probe(M: torch.Tensor, accesses: int, seed: int = 1, mode: int = GOSH_PROBE_READ_WRITE,
                   stream=None) -> None:
    """Random row traffic over M without arithmetic (values unchanged except in write mode);
    time it to compare locations or to measure what the memory system allows."""
    ptr, n, d = _matrix(M, "M")
    _check(lib().gosh_row_probe(ptr, n, d, accesses, seed, mode, _stream(stream)))


class _DeviceArray:
    """A raw device pointer presented through __cuda_array_interface__ (no ownership)."""

    def __init__(self, ptr: int, rows: int, cols: int):
        self.__cuda_array_interface__ = {"shape": (rows, cols), "typestr": "<f4", "data": (ptr, False),
                                         "version": 2, "strides": None}


def gosh_matrix_place(n: int, d: int, arena_bytes: int = 0):
    """An n x d float32 CUDA tensor placed where random row traffic is fastest, and what the
    search found.  The memory belongs to the library: call gosh_matrix_release(tensor) when
    nothing uses the tensor any more (not before), or leave it to the end of the process."""
    ptr = C.c_void_p()
    info = gosh_placement_info()
    _check(lib().gosh_matrix_place(n, d, arena_bytes, C.byref(ptr), C.byref(info)))
    M = torch.as_tensor(_DeviceArray(ptr.value, n, d), device="cuda")
    if M.data_ptr() != ptr.value:  # a copy would defeat the purpose
        lib().gosh_matrix_release(ptr)
        raise RuntimeError("torch copied the placed matrix instead of wrapping it")
    return M, {name: getattr(info, name) for name, _ in gosh_placement_info._fields_}


def gosh_matrix_release(M: torch.Tensor) -> None:
    _check(lib().gosh_matrix_release(M.data_ptr()))


def gosh_csr_validate(g: gosh_csr) -> None:
    """Raise GoshError unless the HOST graph follows the CSR conventions."""
    _check(lib().gosh_csr_validate(C.byref(g)))


class Hierarchy:
    """Handle of a library-owned coarsening hierarchy.  Arrays are exposed as numpy
    views of the library's host memory (level 0 is the caller's own graph)."""

    def __init__(self, handle, keep_alive):
        self._h = handle
        self._keep = keep_alive  # the level-0 tensors must outlive the hierarchy

    def __del__(self):
        self.free()

    def free(self) -> None:
        if getattr(self, "_h", None):
            lib().gosh_hierarchy_free(self._h)
            self._h = None

    def trim_scratch(self) -> None:
        """Return the device scratch blocks kept from the construction of the hierarchy."""
        _check(lib().gosh_hierarchy_trim_scratch(self._h))

    def release_device(self) -> None:
        """Bring a device-built hierarchy to the host and free its device copies."""
        _check(lib().gosh_hierarchy_release_device(self._h))

    @property
    def handle(self):
        return self._h

    @property
    def levels(self) -> int:
        return int(lib().gosh_hierarchy_levels(self._h))

    def shape(self, i: int):
        """(n, nnz) of G_i; never triggers a download."""
        n, nnz = C.c_int64(), C.c_int64()
        _check(lib().gosh_hierarchy_shape(self._h, i, C.byref(n), C.byref(nnz)))
        return int(n.value), int(nnz.value)

    def graph_view(self, i: int) -> gosh_csr:
        v = gosh_csr()
        _check(lib().gosh_hierarchy_graph(self._h, i, C.byref(v)))
        return v

    def graph(self, i: int):
        """(n, xadj, adj) of G_i as numpy arrays (views, do not write)."""
        import numpy as np

        v = self.graph_view(i)
        off_t = C.c_int64 if v.xadj_is64 else C.c_int32
        xadj = np.ctypeslib.as_array(C.cast(v.xadj, C.POINTER(off_t)), shape=(v.n + 1,))
        if v.nnz:
            adj = np.ctypeslib.as_array(C.cast(v.adj, C.POINTER(C.c_int32)), shape=(v.nnz,))
        else:
            adj = np.zeros(0, dtype=np.int32)
        return int(v.n), xadj, adj

    def map(self, i: int):
        import numpy as np

        ptr = C.POINTER(C.c_int32)()
        n = C.c_int64()
        _check(lib().gosh_hierarchy_map(self._h, i, C.byref(ptr), C.byref(n)))
        return np.ctypeslib.as_array(ptr, shape=(n.value,))

    def times(self, i: int):
        """{sort_ms, mark_ms, build_ms} of coarsening level i."""
        ms = (C.c_double * 3)()
        _check(lib().gosh_hierarchy_times(self._h, i, ms))
        return dict(sort_ms=ms[0], mark_ms=ms[1], build_ms=ms[2])

    def mult(self, i: int):
        import numpy as np

        ptr = C.POINTER(C.c_int64)()
        n = C.c_int64()
        _check(lib().gosh_hierarchy_mult(self._h, i, C.byref(ptr), C.byref(n)))
        if n.value == 0:
            return None
        return np.ctypeslib.as_array(ptr, shape=(n.value,))


def _coarsen(fn, n, xadj, adj, threshold, min_shrink, max_levels, n_threads,
             device_ok=False) -> Hierarchy:
    if xadj.is_cuda != adj.is_cuda:
        raise TypeError("xadj and adj must live on the same side")
    if xadj.is_cuda and not device_ok:
        raise TypeError("gosh_coarsen takes host (CPU) tensors")
    g = csr_view(n, xadj, adj)
    out = C.c_void_p()
    _check(fn(C.byref(g), threshold, min_shrink, max_levels, n_threads, C.byref(out)))
    return Hierarchy(out, (xadj, adj))


def gosh_coarsen(n: int, xadj: torch.Tensor, adj: torch.Tensor, threshold: int = 100,
                 min_shrink: float = 1.0, max_levels: int = 64, n_threads: int = 0) -> Hierarchy:
    """Coarsen a HOST graph (CPU tensors).  The tensors are kept alive by the result."""
    return _coarsen(lib().gosh_coarsen, n, xadj, adj, threshold, min_shrink, max_levels, n_threads)


def gosh_coarsen_device(n: int, xadj: torch.Tensor, adj: torch.Tensor, threshold: int = 100,
                        min_shrink: float = 1.0, max_levels: int = 64,
                        n_threads: int = 0) -> Hierarchy:
    """Same hierarchy, built on the current device, where every level then stays.  The
    graph may be given as CPU tensors (uploaded once) or as tensors on that device."""
    return _coarsen(lib().gosh_coarsen_device, n, xadj, adj, threshold, min_shrink, max_levels,
                    n_threads, device_ok=True)


def gosh_hierarchy_levels(h: Hierarchy) -> int:
    return h.levels


def gosh_hierarchy_shape(h: Hierarchy, i: int):
    return h.shape(i)


def gosh_hierarchy_graph(h: Hierarchy, i: int):
    return h.graph(i)


def gosh_hierarchy_map(h: Hierarchy, i: int):
    return h.map(i)


def gosh_hierarchy_mult(h: Hierarchy, i: int):
    return h.mult(i)


def gosh_hierarchy_times(h: Hierarchy, i: int):
    return h.times(i)


def gosh_hierarchy_trim_scratch(h: Hierarchy) -> None:
    h.trim_scratch()


def gosh_hierarchy_release_device(h: Hierarchy) -> None:
    h.release_device()


def gosh_hierarchy_free(h: Hierarchy) -> None:
    h.free()


def gosh_embed(h: Hierarchy, M0: torch.Tensor, k_neg: int, epochs: int, p: float, lr0: float,
               seed: int, flags: int = 0, device_budget_bytes: int = 0, stream=None):
    """Multilevel training into the device matrix M0 (n_0 x d); returns per-level stats."""
    ptr, n0, d = _matrix(M0, "M0")
    if n0 != h.shape(0)[0]:
        raise ValueError("M0 must have one row per vertex of G_0")
    D = h.levels
    stats = (gosh_level_stats * D)()
    _check(lib().gosh_embed(h.handle, d, k_neg, epochs, p, lr0, seed, flags, device_budget_bytes,
                            ptr, stats, _stream(stream)), lambda: _level_stats(stats))
    return _level_stats(stats)


def _level_stats(stats):
    return [dict(level=s.level, n=s.n, nnz=s.nnz, epochs=s.epochs, upload_ms=s.upload_ms,
                 train_ms=s.train_ms, project_ms=s.project_ms, parts_K=s.parts_K, max_abs=s.max_abs,
                 nonfinite=s.nonfinite) for s in stats]


def gosh_embed_host(h: Hierarchy, M0_host: torch.Tensor, k_neg: int, epochs: int, p: float,
                    lr0: float, seed: int, flags: int = 0, device_budget_bytes: int = 0,
                    P_gpu: int = 3, S_gpu: int = 4, B: int = 5, stream=None):
    """Multilevel training into the HOST matrix M0_host; levels above the budget use the
    part-pair rotation.  Returns per-level stats."""
    if M0_host.is_cuda:
        raise TypeError("M0_host must be a host tensor")
    ptr, n0, d = _matrix(M0_host, "M0_host")
    if n0 != h.shape(0)[0]:
        raise ValueError("M0_host must have one row per vertex of G_0")
    D = h.levels
    stats = (gosh_level_stats * D)()
    _check(lib().gosh_embed_host(h.handle, d, k_neg, epochs, p, lr0, seed, flags,
                                 device_budget_bytes, P_gpu, S_gpu, B, ptr, stats, _stream(stream)),
           lambda: _level_stats(stats))
    return _level_stats(stats)


def gosh_pair_order(K: int):
    """[(a_0, b_0), (a_1, b_1), ...]: the order in which part pairs are visited."""
    npairs = K * (K + 1) // 2 if K > 0 else 1
    a = (C.c_int32 * npairs)()
    b = (C.c_int32 * npairs)()
    _check(lib().gosh_pair_order(K, a, b))
    return list(zip(list(a), list(b)))


def gosh_pair_order_blocked(K: int, R: int):
    """The blocked visiting order with blocks of R parts (not the paper's order)."""
    npairs = K * (K + 1) // 2 if K > 0 else 1
    a = (C.c_int32 * npairs)()
    b = (C.c_int32 * npairs)()
    _check(lib().gosh_pair_order_blocked(K, R, a, b))
    return list(zip(list(a), list(b)))


def gosh_parts_plan(n: int, d: int, epochs: int, device_budget_bytes: int, P_gpu: int = 3,
                    S_gpu: int = 4, B: int = 5):
    K = C.c_int32()
    rot = C.c_int64()
    nbytes = C.c_uint64()
    _check(lib().gosh_parts_plan(n, d, epochs, device_budget_bytes, P_gpu, S_gpu, B, C.byref(K),
                                 C.byref(rot), C.byref(nbytes)))
    return dict(K=K.value, rotations=rot.value, device_bytes=nbytes.value)


def _host_csr(n, xadj, adj):
    if xadj.is_cuda or adj.is_cuda:
        raise TypeError("this entry point takes host (CPU) graph tensors")
    return csr_view(n, xadj, adj)


def gosh_parts_sample_pair(n: int, xadj: torch.Tensor, adj: torch.Tensor, K: int, pa: int, pb: int,
                           B: int, k_neg: int, seed: int, rotation: int, level: int,
                           pair_index: int) -> torch.Tensor:
    g = _host_csr(n, xadj, adj)
    ps = -(-n // K)
    size = lambda p: max(0, min(n, (p + 1) * ps) - min(n, p * ps))
    sources = size(pa) + (size(pb) if pa != pb else 0)
    out = torch.full((sources * B * (k_neg + 1),), -2, dtype=torch.int32)
    _check(lib().gosh_parts_sample_pair(C.byref(g), K, pa, pb, B, k_neg, seed, rotation, level,
                                        pair_index, out.data_ptr()))
    return out


def gosh_train_parts(n: int, xadj: torch.Tensor, adj: torch.Tensor, M_host: torch.Tensor,
                     k_neg: int, epochs: int, lr0: float, seed: int, level: int = 0,
                     device_budget_bytes: int = 0, P_gpu: int = 3, S_gpu: int = 4, B: int = 5,
                     force_K: int = 0, flags: int = 0):
    """Train a matrix in place with the part-pair rotation: a HOST matrix (ideally pinned),
    whose parts rotate through the device, or a matrix on the current device, whose parts are
    trained where they are.  The graph may be CPU tensors (positives are drawn by a host
    sampler) or tensors on the current device (positives are drawn there)."""
    if xadj.is_cuda != adj.is_cuda:
        raise TypeError("xadj and adj must live on the same side")
    g = csr_view(n, xadj, adj) if xadj.is_cuda else _host_csr(n, xadj, adj)
    ptr, rows, d = _matrix(M_host, "M_host")
    if rows != n:
        raise ValueError("M_host must have one row per vertex")
    st = gosh_parts_stats()
    as_dict = lambda: {name: getattr(st, name) for name, _ in gosh_parts_stats._fields_}
    _check(lib().gosh_train_parts(C.byref(g), ptr, d, k_neg, epochs, lr0, seed, level,
                                  device_budget_bytes, P_gpu, S_gpu, B, force_K, flags, C.byref(st)), as_dict)
    return as_dict()
