"""The multilevel driver (Alg. 2) on the GPU against the oracle's V-cycle."""
import sys

import numpy as np
import pytest
import torch

import graphgen
import paper_2008_12336_amd as G
from oracle import gosh_oracle as O
from tests.linkpred import aucroc, make_eval_sets
from tests.util import rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


COARSENERS = {"host": G.gosh_coarsen, "device": G.gosh_coarsen_device}


@pytest.mark.parametrize("where", sorted(COARSENERS))
def test_sequential_vcycle_matches_oracle(where):
    n = 1 << 11
    c = graphgen.to_csr(n, graphgen.rmat(11, 1 << 14, 3))
    xadj, adj = c.xadj.numpy(), c.adj.numpy()
    d, k, epochs, p, lr0, seed = 32, 3, 12, 0.3, 0.05, 5
    want, graphs, maps, e_i = O.embed(xadj, adj, d, k, epochs, p, lr0, seed, threshold=100,
                                      min_shrink=0.8)
    h = COARSENERS[where](n, c.xadj, c.adj, threshold=100, min_shrink=0.8)
    assert h.levels == len(graphs) >= 3
    M0 = torch.zeros(n, d, dtype=torch.float32, device=DEV)
    say(f"[vcycle {where}] D={h.levels} sizes={[g[0].size - 1 for g in graphs]} epochs={e_i.tolist()}")
    stats = G.gosh_embed(h, M0, k, epochs, p, lr0, seed, flags=G.GOSH_FLAG_SEQUENTIAL)
    torch.cuda.synchronize()
    assert [s["epochs"] for s in stats] == e_i.tolist()
    assert [s["n"] for s in stats] == [g[0].size - 1 for g in graphs]
    err = rel_err(M0.cpu().numpy(), want)
    say(f"[vcycle] relative error vs oracle {err:.2e}")
    assert err <= 1e-5


def test_edge_epochs_vcycle_matches_oracle():
    """GOSH_FLAG_EDGE_EPOCHS: an epoch samples |E_i| sources (the experiments' definition),
    i.e. ceil(|E_i| / |V_i|) passes of Alg. 3, with the learning rate decaying over all."""
    n = 1 << 10
    c = graphgen.to_csr(n, graphgen.rmat(10, 1 << 14, 8))
    xadj, adj = c.xadj.numpy(), c.adj.numpy()
    d, k, epochs, p, lr0, seed = 16, 2, 6, 0.3, 0.05, 3
    want, graphs, maps, passes = O.embed(xadj, adj, d, k, epochs, p, lr0, seed, threshold=100,
                                         min_shrink=0.8, edge_epochs=True)
    plain = O.epoch_split(epochs, p, len(graphs))
    assert any(int(a) > int(b) for a, b in zip(passes, plain))  # the flag changes something here
    h = G.gosh_coarsen_device(n, c.xadj, c.adj, threshold=100, min_shrink=0.8)
    M0 = torch.zeros(n, d, dtype=torch.float32, device=DEV)
    stats = G.gosh_embed(h, M0, k, epochs, p, lr0, seed,
                         flags=G.GOSH_FLAG_SEQUENTIAL | G.GOSH_FLAG_EDGE_EPOCHS)
    torch.cuda.synchronize()
    assert [s["epochs"] for s in stats] == [int(e) for e in passes]
    err = rel_err(M0.cpu().numpy(), want)
    say(f"[edge epochs] passes per level {[int(e) for e in passes]} (plain {plain.tolist()}) err {err:.2e}")
    assert err <= 1e-5


def test_single_level_hierarchy_and_budget():
    n = 300
    c = graphgen.to_csr(n, graphgen.er_gnm(n, 1500, 2))
    h = G.gosh_coarsen(n, c.xadj, c.adj, threshold=1000)
    assert h.levels == 1
    M0 = torch.zeros(n, 16, dtype=torch.float32, device=DEV)
    G.gosh_embed(h, M0, 3, 4, 0.5, 0.05, 9, flags=G.GOSH_FLAG_SEQUENTIAL)
    torch.cuda.synchronize()
    want = O.init_embedding(n, 16, 9, 0)
    O.train_level(c.xadj.numpy(), c.adj.numpy(), want, 3, 0.05, 4, 9, 0)
    assert rel_err(M0.cpu().numpy(), want) <= 1e-5
    with pytest.raises(G.GoshError, match="budget"):
        G.gosh_embed(h, M0, 3, 4, 0.5, 0.05, 9, device_budget_bytes=1000)
    with pytest.raises(G.GoshError):
        G.gosh_embed(h, M0, 3, 0, 0.5, 0.05, 9)  # no epochs for the level


def test_hogwild_vcycle_aucroc():
    """Multilevel training (coarsening on) reaches the oracle's link-prediction quality."""
    n = 1 << 13
    edges = graphgen.rmat(13, 1 << 17, 7)
    train, test = graphgen.holdout_split(edges, 0.1, 1007)
    c = graphgen.to_csr(n, train)
    xadj, adj = c.xadj.numpy(), c.adj.numpy()
    sets = make_eval_sets(n, train.numpy(), test.numpy(), seed=1)
    d, k, epochs, p, lr0, seed = 32, 3, 300, 0.3, 0.035, 1
    Mo, graphs, maps, e_i = O.embed(xadj, adj, d, k, epochs, p, lr0, seed, threshold=100,
                                    min_shrink=0.8)
    h = G.gosh_coarsen(n, c.xadj, c.adj, threshold=100, min_shrink=0.8)
    M0 = torch.zeros(n, d, dtype=torch.float32, device=DEV)
    stats = G.gosh_embed(h, M0, k, epochs, p, lr0, seed)
    torch.cuda.synchronize()
    ho, fo = aucroc(Mo, sets)
    hg, fg = aucroc(M0.cpu().numpy(), sets)
    say(f"[auc vcycle] D={h.levels} epochs={e_i.tolist()} oracle {ho:.4f}/{fo:.4f} gpu {hg:.4f}/{fg:.4f}")
    say("[auc vcycle] per level ms: " + ", ".join(f"L{s['level']}:{s['train_ms']:.1f}" for s in stats))
    assert hg > 0.65 and ho > 0.65
    assert abs(hg - ho) <= 0.01 and abs(fg - fo) <= 0.01


@pytest.mark.parametrize("where", sorted(COARSENERS))
@pytest.mark.parametrize("budget_kib,expect_parts", [(0, 0), (4096, 0), (300, 1), (200, 2), (64, 4)])
def test_budgeted_vcycle_on_host_matches_oracle(budget_kib, expect_parts, where):
    """Alg. 2 with levels above the device budget trained by the rotation: sequential mode
    against the oracle's composition of Alg. 3 / Alg. 5 levels."""
    n = 1 << 11
    c = graphgen.to_csr(n, graphgen.rmat(11, 1 << 14, 3))
    xadj, adj = c.xadj.numpy(), c.adj.numpy()
    d, k, epochs, p, lr0, seed = 32, 3, 40, 0.3, 0.05, 5
    budget = budget_kib * 1024
    want, modes = O.embed_budget(xadj, adj, d, k, epochs, p, lr0, seed,
                                 budget if budget else 1 << 40, threshold=100, min_shrink=0.8)
    h = COARSENERS[where](n, c.xadj, c.adj, threshold=100, min_shrink=0.8)
    M0 = torch.zeros(n, d, dtype=torch.float32).pin_memory()
    stats = G.gosh_embed_host(h, M0, k, epochs, p, lr0, seed, flags=G.GOSH_FLAG_SEQUENTIAL,
                              device_budget_bytes=budget)
    got_modes = [s["parts_K"] for s in stats]
    err = rel_err(M0.numpy(), want)
    say(f"[budget {budget_kib} KiB] oracle modes {modes} gpu modes {got_modes} err {err:.2e}")
    assert got_modes == modes
    assert sum(1 for m in modes if m) == expect_parts
    assert err <= 1e-5


def test_budgeted_vcycle_with_blocked_order_matches_oracle():
    """gosh_embed_host passes GOSH_FLAG_BLOCKED_ORDER on to the levels it trains by rotation."""
    n = 1 << 11
    c = graphgen.to_csr(n, graphgen.rmat(11, 1 << 14, 3))
    xadj, adj = c.xadj.numpy(), c.adj.numpy()
    d, k, epochs, p, lr0, seed, P = 32, 3, 40, 0.3, 0.05, 5, 5
    budget = 200 * 1024
    want, modes = O.embed_budget(xadj, adj, d, k, epochs, p, lr0, seed, budget, P_gpu=P, threshold=100,
                                 min_shrink=0.8, blocked=True)
    plain, _ = O.embed_budget(xadj, adj, d, k, epochs, p, lr0, seed, budget, P_gpu=P, threshold=100,
                              min_shrink=0.8)
    h = G.gosh_coarsen_device(n, c.xadj, c.adj, threshold=100, min_shrink=0.8)
    M0 = torch.zeros(n, d, dtype=torch.float32).pin_memory()
    stats = G.gosh_embed_host(h, M0, k, epochs, p, lr0, seed, device_budget_bytes=budget, P_gpu=P,
                              flags=G.GOSH_FLAG_SEQUENTIAL | G.GOSH_FLAG_BLOCKED_ORDER)
    assert [s["parts_K"] for s in stats] == modes and max(modes) >= 5
    err = rel_err(M0.numpy(), want)
    say(f"[budget blocked] modes {modes} err {err:.2e}")
    assert err <= 1e-5
    assert rel_err(plain, want) > 1e-4


def test_cxx_example_embeds_through_the_c_abi_alone():
    """The C++ example (no Python, no torch: hipMalloc + include/gosh.h) coarsens on the device,
    runs Alg. 2 and must find edges scoring higher than random pairs (its exit status)."""
    import os
    import subprocess

    from paper_2008_12336_amd import build as B

    if not os.path.exists(B.EXAMPLE):  # normally built with the library; a two-second link otherwise
        try:
            B.build_example()
        except Exception as ex:
            pytest.skip(f"the example is not built and cannot be built here: {ex}")
    run = subprocess.run([B.EXAMPLE], capture_output=True, text=True, timeout=100)
    print(run.stdout, run.stderr, flush=True)
    assert run.returncode == 0
    assert "mean dot over edges" in run.stdout


@pytest.fixture
def small_pair_levels():
    """Lowers the smallest part of GOSH_FLAG_PAIR_LEVELS to 300 vertices for one test."""
    G.gosh_set_tuning(pair_level_min_n=300)
    yield 300
    G.gosh_set_tuning()


@pytest.mark.parametrize("host_matrix", [False, True])
def test_pair_levels_vcycle_matches_the_oracle(host_matrix, small_pair_levels):
    """GOSH_FLAG_PAIR_LEVELS: resident levels above a size (lowered here through the tuning
    record) train in place with Alg. 5, on the part counts the library's rule gives (its own
    unit test: tests/test_parts_host.py); the oracle is handed those counts, and the
    sequential V-cycle must match its composition level by level."""
    n, d, k, epochs = 3000, 32, 3, 260
    c = graphgen.to_csr(n, graphgen.chung_lu(n, 24000, 4))
    xadj, adj = c.xadj.numpy(), c.adj.numpy()
    graphs, _, _ = O.coarsen(xadj, adj, threshold=100, min_shrink=0.8)
    e_i = O.epoch_split(epochs, 0.3, len(graphs))
    want_K = [G.gosh_pair_level_parts(int(e_i[i]), graphs[i][0].size - 1, small_pair_levels)
              for i in range(len(graphs))]
    assert any(want_K) and not all(want_K), want_K  # both kinds of level occur
    want, graphs, maps, e_i = O.embed(xadj, adj, d, k, epochs, 0.3, 0.05, 5, threshold=100, min_shrink=0.8,
                                      parts_K=want_K)
    h = G.gosh_coarsen_device(n, c.xadj, c.adj, threshold=100, min_shrink=0.8)
    flags = G.GOSH_FLAG_SEQUENTIAL | G.GOSH_FLAG_PAIR_LEVELS
    if host_matrix:
        M0 = torch.zeros(n, d, dtype=torch.float32).pin_memory()
        stats = G.gosh_embed_host(h, M0, k, epochs, 0.3, 0.05, 5, flags=flags)
        got = M0.numpy()
    else:
        M0 = torch.zeros(n, d, dtype=torch.float32, device=DEV)
        stats = G.gosh_embed(h, M0, k, epochs, 0.3, 0.05, 5, flags=flags)
        torch.cuda.synchronize()
        got = M0.cpu().numpy()
    assert [s["parts_K"] for s in sorted(stats, key=lambda s: s["level"])] == want_K
    assert rel_err(got, want) <= 1e-5
    h.free()
    # without the flag the same call trains every level with Alg. 3
    plain, *_ = O.embed(xadj, adj, d, k, epochs, 0.3, 0.05, 5, threshold=100, min_shrink=0.8)
    assert rel_err(got, plain) > 1e-3
