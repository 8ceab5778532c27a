"""CPU-only checks of the C ABI: the library loads, exports every declared symbol,
rejects bad arguments before touching a device, and its host helpers agree with the
oracle."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2008_12336_amd as G
from oracle import gosh_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if fn.endswith(".h"):
            text = open(os.path.join(ROOT, "include", fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(gosh_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    lib = G.lib()
    names = declared_symbols()
    assert "gosh_train_epoch" in names and len(names) >= 6
    for name in names:
        assert hasattr(lib, name), f"{name} declared in include/ but not exported"
    assert sorted(G.binding.EXPORTS) == names, "binding and header disagree"
    for name in names:
        assert hasattr(G.binding, name), f"binding lacks {name}"


def test_lr_matches_oracle_bit_for_bit():
    for lr0 in (0.025, 0.035, 0.045, 0.05, 1.0):
        for e in (1, 7, 100, 600, 1400, 100000):
            for j in sorted({0, 1, e // 3, e // 2, e - 1}):
                if j < e:
                    assert G.gosh_lr(lr0, j, e) == O.lr(lr0, j, e)
    assert G.gosh_lr(0.1, 0, 0) == 0.0


def test_epoch_split_matches_oracle():
    for e in (5, 64, 200, 600, 1000, 1400, 99991):
        for p in (0.0, 0.1, 0.3, 0.5, 0.77, 1.0):
            for D in (1, 2, 5, 8, 12):
                try:
                    want = O.epoch_split(e, p, D).tolist()
                except ValueError:
                    with pytest.raises(G.GoshError):
                        G.gosh_epoch_split(e, p, D)
                    continue
                assert G.gosh_epoch_split(e, p, D) == want


def _fake_csr(n=8, nnz=8, is64=0):
    return G.gosh_csr(n, nnz, 0x1000, 0x2000, is64)


def test_bad_arguments_are_rejected_on_the_host():
    """Each call fails in the argument checks, before any HIP call, so this runs
    without a GPU (the pointers are never dereferenced)."""
    lib = G.lib()
    g = _fake_csr()
    ok_ptr = 0x10000

    def train(gv=g, ptr=ok_ptr, d=128, k=3, lr=0.1, flags=0):
        return lib.gosh_train_epoch(C.byref(gv), ptr, d, k, lr, 1, 0, 0, flags, None)

    for kwargs, frag in [
        (dict(d=6), "multiple of 4"),
        (dict(d=0), "multiple of 4"),
        (dict(d=516), "multiple of 4"),
        (dict(k=16), "k_neg"),
        (dict(k=-1), "k_neg"),
        (dict(ptr=ok_ptr + 4), "aligned"),
        (dict(ptr=0), "null"),
        (dict(flags=8), "flags"),
        (dict(flags=2 | 4), "flags"),
        (dict(lr=float("nan")), "NaN"),
        (dict(gv=G.gosh_csr(0, 0, 0x1000, 0x2000, 0)), "n = 0"),
        (dict(gv=G.gosh_csr(2 ** 31, 0, 0x1000, 0x2000, 1)), "n ="),
        (dict(gv=G.gosh_csr(8, 8, 0, 0x2000, 0)), "xadj"),
        (dict(gv=G.gosh_csr(8, 8, 0x1000, 0, 0)), "adj"),
        (dict(gv=G.gosh_csr(8, 2 ** 31 + 5, 0x1000, 0x2000, 0)), "64-bit"),
    ]:
        assert train(**kwargs) == -1, kwargs
        assert frag in G.gosh_last_error(), (kwargs, G.gosh_last_error())

    assert lib.gosh_sample_epoch(C.byref(g), 16, 1, 0, 0, ok_ptr, None) == -1
    assert lib.gosh_sample_epoch(C.byref(g), 3, 1, 0, 0, 0, None) == -1
    assert lib.gosh_init_embedding(ok_ptr, 0, 32, 1, 0, None) == -1
    assert lib.gosh_init_embedding(ok_ptr, 10, 30, 1, 0, None) == -1
    assert lib.gosh_project(ok_ptr, 0, 0x3000, 5, 32, ok_ptr * 2, None) == -1  # empty coarse level
    assert lib.gosh_project(ok_ptr, 5, 0, 10, 32, ok_ptr * 2, None) == -1
    assert lib.gosh_epoch_split(10, 0.5, 3, None) == -1
    # the placement entry points check their arguments before they touch the device too
    out = C.c_void_p()
    assert lib.gosh_matrix_place(10, 6, 0, C.byref(out), None) == -1 and out.value is None
    assert lib.gosh_matrix_place(0, 32, 0, C.byref(out), None) == -1
    assert lib.gosh_matrix_place(10, 32, 0, None, None) == -1
    assert lib.gosh_row_probe(ok_ptr, 10, 30, 5, 1, 0, None) == -1
    assert lib.gosh_row_probe(ok_ptr + 4, 10, 32, 5, 1, 0, None) == -1
    assert lib.gosh_row_probe(ok_ptr, 0, 32, 5, 1, 0, None) == -1
    assert lib.gosh_row_probe(ok_ptr, 10, 32, -1, 1, 0, None) == -1
    assert lib.gosh_row_probe(ok_ptr, 10, 32, 5, 1, 4, None) == -1 and "mode" in G.gosh_last_error()
    assert lib.gosh_matrix_check(ok_ptr, 10, 30, None, None, None) == -1
    assert lib.gosh_matrix_check(0, 10, 32, None, None, None) == -1
    # the entry point that never allocates checks its own limit first
    big = G.gosh_csr(G.GOSH_STATIC_MAX_N + 1, 8, 0x1000, 0x2000, 0)
    assert lib.gosh_train_epoch_static(C.byref(big), ok_ptr, 32, 3, 0.1, 1, 0, 0, 0, None) == -1
    assert "at most" in G.gosh_last_error()
    assert lib.gosh_train_epoch_static(C.byref(g), ok_ptr, 30, 3, 0.1, 1, 0, 0, 0, None) == -1
    assert lib.gosh_set_tuning(None) == 0
    assert lib.gosh_pair_level_parts(0, 100, 1, 5) == 0 and lib.gosh_pair_level_parts(10, 100, 1, 0) == 0


def test_header_is_plain_c():
    """include/gosh.h must compile as C99 on its own (the boundary is a C ABI)."""
    import subprocess
    import tempfile

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    with tempfile.TemporaryDirectory() as tmp:
        src = os.path.join(tmp, "use_header.c")
        with open(src, "w") as fh:
            fh.write('#include "gosh.h"\nint main(void) { gosh_level_stats s; gosh_parts_stats p; '
                     "gosh_csr g; (void)s; (void)p; (void)g; return gosh_hierarchy_levels(0); }\n")
        subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only",
                        "-I", os.path.join(root, "include"), src], check=True)


def test_cxx_example_links_against_the_header_and_runs_its_host_part():
    """paper_2008_12336_amd/examples/embed_example.cpp uses the library through include/gosh.h
    alone; its --host-only mode (validate, coarsen on the host, epoch split) needs no GPU."""
    import subprocess

    from paper_2008_12336_amd import build as B

    exe = B.EXAMPLE if os.path.exists(B.EXAMPLE) else B.build_example()
    out = subprocess.run([exe, "--host-only"], capture_output=True, text=True, check=True).stdout
    lines = out.strip().splitlines()
    assert lines[0].startswith("hierarchy: ") and " 4000/" in lines[0]
    levels = int(lines[0].split()[1])
    epochs = [int(x) for x in lines[1].split(":")[1].split()]
    assert len(epochs) == levels and sum(epochs) == 600
