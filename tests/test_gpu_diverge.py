"""Divergence is reported, not returned silently: gosh_matrix_check against torch, and
GOSH_EDIVERGED with complete statistics from the multilevel drivers and the rotation when a
learning rate far too large blows the rows up (nothing in Alg. 1 bounds a row)."""
import numpy as np
import pytest
import torch

import graphgen
import paper_2008_12336_amd as G

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("n,d", [(1, 4), (1000, 128), (777, 100), (65537, 8), (300, 512)])
def test_matrix_check_agrees_with_torch(n, d):
    gen = torch.Generator(device=DEV).manual_seed(n)
    M = torch.randn(n, d, device=DEV, generator=gen) * 3
    top, bad = G.gosh_matrix_check(M)
    assert bad == 0 and top == M.abs().max().item()
    if n * d >= 12:
        flat = M.view(-1)
        flat[3] = float("inf")
        flat[n * d - 1] = float("nan")
        flat[n * d // 2] = float("-inf")
        flat[5] = -1e30
        top, bad = G.gosh_matrix_check(M)
        assert bad == 3 and top == np.float32(1e30)
    Z = torch.zeros(n, d, device=DEV)
    assert G.gosh_matrix_check(Z) == (0.0, 0)


def hub_graph(n, m, seed):
    c = graphgen.to_csr(n, graphgen.chung_lu(n, m, seed))
    return c


def test_drivers_report_a_diverged_run():
    n, d, k = 4000, 32, 3
    c = hub_graph(n, 30000, 2)
    h = G.gosh_coarsen_device(n, c.xadj, c.adj, threshold=200, min_shrink=0.8)
    assert h.levels >= 2
    M0 = torch.zeros(n, d, device=DEV)
    # a sane learning rate: finite, max_abs reported per level
    stats = G.gosh_embed(h, M0, k, 40, 0.3, 0.05, 1)
    assert all(s["nonfinite"] == 0 and 0 < s["max_abs"] < 1e3 for s in stats)
    assert stats[0]["max_abs"] == M0.abs().max().item()
    # a learning rate of 1e12: rows overflow within a few epochs
    with pytest.raises(G.GoshError) as info:
        G.gosh_embed(h, M0, k, 40, 0.3, 1e12, 1)
    assert info.value.code == G.GOSH_EDIVERGED and "diverged" in str(info.value)
    stats = info.value.stats
    assert len(stats) == h.levels and stats[0]["nonfinite"] > 0
    assert stats[0]["nonfinite"] == int((~torch.isfinite(M0)).sum().item())  # M_0 is delivered as it is
    # the same through the host driver with a budget that sends level 0 through the rotation
    Mh = torch.zeros(n, d).pin_memory()
    with pytest.raises(G.GoshError) as info:
        G.gosh_embed_host(h, Mh, k, 40, 0.3, 1e12, 1, device_budget_bytes=300 << 10)
    assert info.value.code == G.GOSH_EDIVERGED
    assert info.value.stats[0]["parts_K"] > 1 and info.value.stats[0]["nonfinite"] > 0
    assert not torch.isfinite(Mh).all()
    h.free()


@pytest.mark.parametrize("where", ["host", "device"])
def test_rotation_reports_a_diverged_run(where):
    n, d, k = 3000, 16, 3
    c = hub_graph(n, 20000, 5)
    M = torch.randn(n, d) * 0.1
    M = M.to(DEV) if where == "device" else M.pin_memory()
    st = G.gosh_train_parts(n, c.xadj, c.adj, M, k, 20, 0.05, 1, force_K=4)
    assert st["nonfinite"] == 0 and 0 < st["max_abs"] < 1e3
    if where == "device":
        assert st["max_abs"] == M.abs().max().item()
    with pytest.raises(G.GoshError) as info:
        G.gosh_train_parts(n, c.xadj, c.adj, M, k, 40, 1e12, 1, force_K=4)
    assert info.value.code == G.GOSH_EDIVERGED and info.value.stats["nonfinite"] > 0
    assert not torch.isfinite(M).all()
