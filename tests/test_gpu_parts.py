"""The part-pair rotation (Alg. 5) on the GPU against the oracle."""
import sys

import numpy as np
import pytest
import torch

import graphgen
import paper_2008_12336_amd as G
from oracle import gosh_oracle as O
from tests.linkpred import aucroc, make_eval_sets
from tests.util import conditioned_bar, oracle_sensitivity, rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def graph(n, m, seed, kind="er"):
    edges = graphgen.er_gnm(n, m, seed) if kind == "er" else graphgen.chung_lu(n, m, seed)
    c = graphgen.to_csr(n, edges)
    G.gosh_csr_validate(G.csr_view(n, c.xadj, c.adj))
    return c


@pytest.mark.parametrize("n,K,pa,pb,B,k", [(50, 3, 1, 0, 4, 3), (50, 3, 2, 2, 4, 3), (1000, 4, 3, 1, 5, 3),
                                           (1000, 7, 6, 0, 2, 5), (1001, 5, 4, 4, 3, 0), (64, 1, 0, 0, 5, 15)])
def test_pair_sample_stream_bit_exact(n, K, pa, pb, B, k):
    say(f"[pair-stream] n={n} K={K} pair=({pa},{pb}) B={B} k={k}")
    c = graph(n, 6 * n, 5)
    xadj, adj = c.xadj.numpy(), c.adj.numpy()
    for seed, rot, level, q in [(1, 0, 0, 2), (2 ** 63 + 5, 9, 3, 11)]:
        got = G.gosh_parts_sample_pair(n, c.xadj, c.adj, K, pa, pb, B, k, seed, rot, level, q).numpy()
        M = O.init_embedding(n, 4, 1, 0)
        want = O.train_pair(xadj, adj, M, k, B, K, pa, pb, 0.0, seed, rot, level, q, want_stream=True)
        assert np.array_equal(got, want)


def budget_for(n, d, K, P, S, B):
    ps = -(-n // K)
    return min(P, K) * ps * d * 4 + S * 2 * ps * B * 4 + ((n + 63) // 64) * 8


@pytest.mark.parametrize("n,d,K,P,S,B,k,epochs", [
    (600, 32, 3, 3, 4, 5, 3, 30),
    (601, 128, 4, 2, 1, 2, 3, 16),
    (500, 8, 1, 3, 4, 5, 3, 10),
    (900, 64, 5, 3, 2, 3, 2, 45),
    (700, 100, 6, 4, 3, 1, 5, 12),
    (9, 8, 4, 3, 2, 2, 3, 16),  # ceil(9/4) = 3 rows per part: the fourth part is empty
    (1200, 32, 9, 4, 4, 2, 3, 40),  # four slots: eager write-back and two-visit lookahead
    (1200, 32, 9, 6, 2, 2, 3, 40),
])
def test_sequential_rotation_matches_oracle(n, d, K, P, S, B, k, epochs):
    say(f"[parts-seq] n={n} d={d} K={K} P={P} S={S} B={B} k={k} epochs={epochs}")
    c = graph(n, 5 * n, 8, "cl")
    xadj, adj = c.xadj.numpy(), c.adj.numpy()
    M0 = (O.init_embedding(n, d, 3, 0).astype(np.float64) * d * 0.8).astype(np.float32)
    want = M0.copy()
    O.train_parts(xadj, adj, want, k, epochs, 0.1, 7, 2, K, B)
    budget = budget_for(n, d, K, P, S, B)
    plan = G.gosh_parts_plan(n, d, epochs, budget, P, S, B)
    assert plan["K"] <= K
    M = torch.from_numpy(M0.copy()).pin_memory()
    st = G.gosh_train_parts(n, c.xadj, c.adj, M, k, epochs, 0.1, 7, level=2, device_budget_bytes=budget,
                            P_gpu=P, S_gpu=S, B=B, force_K=K, flags=G.GOSH_FLAG_SEQUENTIAL)
    err = rel_err(M.numpy(), want)
    say(f"            K={st['K']} rotations={st['rotations']} visits={st['pair_visits']} err={err:.2e} "
        f"h2d={st['bytes_h2d']} d2h={st['bytes_d2h']}")
    assert st["K"] == K and st["rotations"] == O.rotations(epochs, B, K)
    assert st["pair_visits"] == st["rotations"] * K * (K + 1) // 2
    assert st["device_bytes"] <= budget
    assert err <= 1e-5
    assert rel_err(M0, want) > 1e-3
    # every part went to the device at least once per rotation and came back as often
    part_bytes = n * d * 4
    assert st["bytes_d2h"] >= part_bytes and st["bytes_h2d"] >= part_bytes
    if K <= P:
        assert st["bytes_d2h"] == part_bytes  # everything stays resident until the end


@pytest.mark.parametrize("scale", [2.0, 1.0, 0.6])
def test_the_randomised_case_that_missed_the_bar(scale):
    """Chung-Lu, 1,000 vertices, d = 512, k = 5, K = 9, P = 3, S = 3, B = 4, 76 epochs, host
    graph, paper order: at scale 2 (rows uniform in [-1, 1)) a randomised sweep found the
    sequential rotation 4.8e-4 from the oracle.  The run is ill-conditioned there in the
    oracle itself (tests/test_fp32_model.py): the bar is eight times the oracle's own
    sensitivity to a one-ulp change of its input.  The same case from rows scaled to 1 or
    0.6 is well-conditioned and meets 1e-5 -- same graph, parts, swaps and pools, so slots,
    write-backs and ordering are not what differs."""
    n, d, k, K, P, S, B, epochs, seed, level = 1000, 512, 5, 9, 3, 3, 4, 76, 779413867887070026, 244
    c = graphgen.to_csr(n, graphgen.chung_lu(n, 5690, 26))
    xadj, adj = c.xadj.numpy().astype(np.int64), c.adj.numpy()
    R0 = (O.init_embedding(n, d, seed, 1).astype(np.float64) * d * scale).astype(np.float32)
    want, sens = oracle_sensitivity(lambda X: O.train_parts(xadj, adj, X, k, epochs, 0.1, seed, level, K, B), R0)
    bar = conditioned_bar(sens)
    M = torch.from_numpy(R0.copy()).pin_memory()
    st = G.gosh_train_parts(n, c.xadj, c.adj, M, k, epochs, 0.1, seed, level=level, P_gpu=P, S_gpu=S, B=B,
                            force_K=K, flags=G.GOSH_FLAG_SEQUENTIAL)
    err = rel_err(M.numpy(), want)
    say(f"[case 445] scale={scale}: oracle sensitivity {sens:.2e}, bar {bar:.2e}, gpu vs oracle {err:.2e}, "
        f"visits {st['pair_visits']}")
    assert st["pair_visits"] == 3 * 45
    assert (bar == 1e-5) == (scale < 2.0)
    assert err <= bar


def test_unpinned_host_matrix_and_forced_split():
    n, d, k = 400, 16, 3
    c = graph(n, 2000, 4)
    M0 = O.init_embedding(n, d, 1, 0) * 10
    want = M0.copy()
    O.train_parts(c.xadj.numpy(), c.adj.numpy(), want, k, 20, 0.05, 3, 0, 4, 5)
    M = torch.from_numpy(M0.copy())  # pageable memory
    st = G.gosh_train_parts(n, c.xadj, c.adj, M, k, 20, 0.05, 3, force_K=4, flags=G.GOSH_FLAG_SEQUENTIAL)
    assert st["K"] == 4
    assert rel_err(M.numpy(), want) <= 1e-5
    with pytest.raises(G.GoshError, match="budget"):
        G.gosh_train_parts(n, c.xadj, c.adj, M, k, 20, 0.05, 3, device_budget_bytes=100)
    with pytest.raises(G.GoshError):
        G.gosh_train_parts(n, c.xadj, c.adj, M, k, 20, 0.05, 3, force_K=4, P_gpu=1)


@pytest.mark.parametrize("n,d,K,P,S,B,k,epochs", [
    (600, 32, 3, 3, 4, 5, 3, 30),    # blocks of one part: column order
    (1200, 32, 9, 4, 4, 2, 3, 40),   # blocks of two
    (1300, 16, 13, 5, 3, 2, 2, 60),  # blocks of three, last block short
    (1100, 32, 7, 6, 2, 3, 3, 50),   # blocks of four
    (500, 8, 2, 4, 2, 2, 3, 10),     # fewer parts than slots: one block, the paper's order
    (9, 8, 4, 4, 2, 2, 3, 16),       # an empty last part
    (700, 16, 5, 2, 1, 1, 2, 10),    # two slots only: nothing can be fetched ahead
    (800, 16, 11, 8, 1, 1, 0, 22),   # more slots than a block can use up; no negatives
])
def test_sequential_blocked_rotation_matches_oracle(n, d, K, P, S, B, k, epochs):
    """GOSH_FLAG_BLOCKED_ORDER: the rotation visits the pairs in the blocked order (blocks of
    min(P, K) - 2 parts) with parts fetched several visits ahead; sequential mode against the
    oracle's rotation in the same order, and fewer bytes over the link than the paper's."""
    say(f"[parts-blocked] n={n} d={d} K={K} P={P} S={S} B={B} k={k} epochs={epochs}")
    c = graph(n, 5 * n, 8, "cl")
    xadj, adj = c.xadj.numpy(), c.adj.numpy()
    M0 = (O.init_embedding(n, d, 3, 0).astype(np.float64) * d * 0.8).astype(np.float32)
    want = M0.copy()
    block = O.blocked_block_size(P, K)
    O.train_parts(xadj, adj, want, k, epochs, 0.1, 7, 2, K, B, block=block)
    budget = budget_for(n, d, K, P, S, B)
    runs = {}
    for name, flags in (("blocked", G.GOSH_FLAG_BLOCKED_ORDER), ("paper", 0)):
        M = torch.from_numpy(M0.copy()).pin_memory()
        st = G.gosh_train_parts(n, c.xadj, c.adj, M, k, epochs, 0.1, 7, level=2, device_budget_bytes=budget,
                                P_gpu=P, S_gpu=S, B=B, force_K=K, flags=G.GOSH_FLAG_SEQUENTIAL | flags)
        runs[name] = (M.numpy().copy(), st)
    got, st = runs["blocked"]
    err = rel_err(got, want)
    say(f"            block={block} visits={st['pair_visits']} err={err:.2e} h2d blocked {st['bytes_h2d']} "
        f"paper {runs['paper'][1]['bytes_h2d']}")
    assert st["K"] == K and st["pair_visits"] == st["rotations"] * K * (K + 1) // 2
    assert err <= 1e-5
    if block >= K:
        assert np.array_equal(got, runs["paper"][0])  # one block: the paper's order itself
    elif K >= 3:
        assert rel_err(runs["paper"][0], want) > 1e-4  # the other order gives another result
    if block > 1 and K >= 2 * P:
        assert st["bytes_h2d"] < 0.85 * runs["paper"][1]["bytes_h2d"]


@pytest.mark.parametrize("offsets64", [False, True])
@pytest.mark.parametrize("order_flag", [0, G.GOSH_FLAG_BLOCKED_ORDER])
def test_device_resident_graph_gives_the_same_rotation(offsets64, order_flag):
    """A graph in device memory is sampled on the device (no host sampler, no pool uploads):
    the positives, hence the whole sequential rotation, must be bit for bit what the host
    sampler gives, and the oracle's within the usual bar."""
    n, d, K, P, S, B, k, epochs = 1300, 32, 7, 4, 2, 3, 3, 45
    c = graphgen.to_csr(n, graphgen.chung_lu(n, 5 * n, 8), offsets64=offsets64)
    M0 = (O.init_embedding(n, d, 3, 0).astype(np.float64) * d * 0.8).astype(np.float32)
    want = M0.copy()
    O.train_parts(c.xadj.numpy(), c.adj.numpy(), want, k, epochs, 0.1, 7, 1, K, B,
                  block=O.blocked_block_size(P, K) if order_flag else 0)
    got = {}
    for where in ("host", "device"):
        xadj = c.xadj if where == "host" else c.xadj.to(DEV)
        adj = c.adj if where == "host" else c.adj.to(DEV)
        M = torch.from_numpy(M0.copy()).pin_memory()
        st = G.gosh_train_parts(n, xadj, adj, M, k, epochs, 0.1, 7, level=1, P_gpu=P, S_gpu=S, B=B,
                                force_K=K, flags=G.GOSH_FLAG_SEQUENTIAL | order_flag)
        got[where] = (M.numpy().copy(), st)
    assert np.array_equal(got["host"][0], got["device"][0])
    assert got["device"][1]["sampler_ms"] == 0 and got["host"][1]["sampler_ms"] > 0
    assert got["device"][1]["bytes_h2d"] < got["host"][1]["bytes_h2d"]  # no pools go up
    assert rel_err(got["device"][0], want) <= 1e-5
    # concurrent mode with the hot-row bitmap built on the device: nothing moves at lr = 0
    M = torch.from_numpy(M0.copy()).pin_memory()
    G.gosh_train_parts(n, c.xadj.to(DEV), c.adj.to(DEV), M, k, epochs, 0.0, 7, force_K=K, flags=order_flag)
    assert np.array_equal(M.numpy(), M0)


@pytest.mark.parametrize("flags", [0, G.GOSH_FLAG_PLAIN_STORES])
def test_concurrent_rotation_with_zero_lr_moves_nothing(flags):
    n, d, k = 3000, 128, 3
    c = graph(n, 20000, 6, "cl")
    M0 = O.init_embedding(n, d, 2, 0)
    M = torch.from_numpy(M0.copy()).pin_memory()
    st = G.gosh_train_parts(n, c.xadj, c.adj, M, k, 30, 0.0, 1, force_K=5, flags=flags)
    assert np.array_equal(M.numpy(), M0)
    assert st["updates"] == st["rotations"] * 5 * (k + 1) * sum(
        (min(n, (a + 1) * 600) - a * 600) + ((min(n, (b + 1) * 600) - b * 600) if a != b else 0)
        for a, b in G.gosh_pair_order(5))


@pytest.mark.parametrize("blocked_on_device", [False, True])
def test_concurrent_rotation_aucroc(blocked_on_device):
    """Rotation training with a budget a quarter of the matrix reaches the quality of the
    oracle's rotation and of ordinary in-device training -- in the paper's pair order with
    the host sampler, and in the blocked order with four slots and positives drawn on the
    device."""
    n = 1 << 12
    edges = graphgen.rmat(12, 1 << 16, 2)
    train, test = graphgen.holdout_split(edges, 0.1, 1002)
    c = graphgen.to_csr(n, train)
    xadj, adj = c.xadj.numpy(), c.adj.numpy()
    sets = make_eval_sets(n, train.numpy(), test.numpy(), seed=1)
    d, k, epochs, lr0, B = 32, 3, 300, 0.045, 5
    budget = n * d * 4 // 4 * 2
    P = 4 if blocked_on_device else 3
    plan = G.gosh_parts_plan(n, d, epochs, budget, P, 4, B)
    K = plan["K"]
    Mo = O.init_embedding(n, d, 1, 0)
    O.train_parts(xadj, adj, Mo, k, epochs, lr0, 1, 0, K, B,
                  block=O.blocked_block_size(P, K) if blocked_on_device else 0)
    M = torch.from_numpy(O.init_embedding(n, d, 1, 0)).pin_memory()
    if blocked_on_device:
        st = G.gosh_train_parts(n, c.xadj.to(DEV), c.adj.to(DEV), M, k, epochs, lr0, 1, device_budget_bytes=budget,
                                P_gpu=P, B=B, flags=G.GOSH_FLAG_BLOCKED_ORDER)
    else:
        st = G.gosh_train_parts(n, c.xadj, c.adj, M, k, epochs, lr0, 1, device_budget_bytes=budget, B=B)
    ho, fo = aucroc(Mo, sets)
    hg, fg = aucroc(M.numpy(), sets)
    say(f"[auc parts] K={K} rotations={st['rotations']} oracle {ho:.4f}/{fo:.4f} gpu {hg:.4f}/{fg:.4f} "
        f"kernel_ms={st['kernel_ms']:.1f} wall_ms={st['wall_ms']:.1f}")
    assert K >= 4 and st["device_bytes"] <= budget
    assert hg > 0.7
    assert abs(hg - ho) <= 0.01 and abs(fg - fo) <= 0.01


@pytest.mark.parametrize("offsets64", [False, True])
def test_malformed_graph_keeps_the_rotation_inside_its_slots(offsets64):
    """Offsets that leave adj, entries that name no vertex and rows that are not ascending:
    the samplers (host and device) treat such rows as empty or draw what is there, the pair
    kernel drops every pool entry outside the partner part.  Both samplers make the same
    probes, so the sequential rotation is the same bit for bit, and finite."""
    from tests.util import corrupt

    n, d, K, P, S, B, k, epochs = 1300, 32, 5, 3, 2, 3, 3, 30
    c = graphgen.to_csr(n, graphgen.chung_lu(n, 5 * n, 8))
    xadj, adj, _ = corrupt(c, offsets64, 2, stray=300)
    M0 = (O.init_embedding(n, d, 3, 0).astype(np.float64) * d * 0.8).astype(np.float32)
    got = {}
    for where in ("host", "device"):
        x, a = torch.from_numpy(xadj), torch.from_numpy(adj)
        if where == "device":
            x, a = x.to(DEV), a.to(DEV)
        for flags in (G.GOSH_FLAG_SEQUENTIAL, 0):
            print(f"malformed graph on the {where}, offsets64={offsets64}, flags {flags}", flush=True)
            M = torch.from_numpy(M0.copy()).pin_memory()
            G.gosh_train_parts(n, x, a, M, k, epochs, 0.1, 7, level=1, P_gpu=P, S_gpu=S, B=B, force_K=K,
                               flags=flags)
            assert np.isfinite(M.numpy()).all()
            if flags:
                got[where] = M.numpy().copy()
    assert np.array_equal(got["host"], got["device"])
    assert not np.array_equal(got["host"], M0)


def test_a_slot_larger_than_the_device_is_an_allocation_failure():
    """One part of 2^28 rows of 512 floats is 550 GB: the first slot cannot be allocated, the
    call reports GOSH_ENOMEM (not a generic runtime failure), releases what it had and leaves
    the device usable.  No kernel runs and the matrix pointer is never followed."""
    import ctypes as C

    n, d = 1 << 28, 512
    xadj = torch.zeros(n + 1, dtype=torch.int32)  # an edgeless graph, untouched pages
    adj = torch.zeros(1, dtype=torch.int32)
    g = G.gosh_csr(n, 0, xadj.data_ptr(), adj.data_ptr(), 0)
    M = torch.zeros(16, d, dtype=torch.float32).pin_memory()
    rc = G.lib().gosh_train_parts(C.byref(g), M.data_ptr(), d, 3, 1, C.c_float(0.1), 1, 0, 0, 3, 4, 5, 1, 0, None)
    assert rc == -2, (rc, G.gosh_last_error())
    assert "part slot" in G.gosh_last_error()
    c = graph(500, 2000, 1, "er")
    M = torch.from_numpy(O.init_embedding(500, 32, 1, 0)).pin_memory()
    G.gosh_train_parts(500, c.xadj, c.adj, M, 3, 10, 0.05, 1, force_K=3)
    assert np.isfinite(M.numpy()).all()


@pytest.mark.parametrize("graph_on_device", [False, True])
@pytest.mark.parametrize("order_flag", [0, G.GOSH_FLAG_BLOCKED_ORDER])
def test_matrix_in_device_memory_is_trained_in_place(graph_on_device, order_flag):
    """With the matrix on the device every part is its own slot and nothing is copied: the
    sequential rotation is bit for bit the one of the host-matrix path (same kernels, same
    order, same pools) and within the bar of the oracle's; the part count defaults to 16."""
    n, d, K, P, S, B, k, epochs = 1500, 32, 6, 4, 2, 3, 3, 40
    c = graphgen.to_csr(n, graphgen.chung_lu(n, 5 * n, 9))
    xadj = c.xadj.to(DEV) if graph_on_device else c.xadj
    adj = c.adj.to(DEV) if graph_on_device else c.adj
    M0 = (O.init_embedding(n, d, 3, 0).astype(np.float64) * d * 0.8).astype(np.float32)
    want = M0.copy()
    O.train_parts(c.xadj.numpy(), c.adj.numpy(), want, k, epochs, 0.1, 7, 2, K, B,
                  block=O.blocked_block_size(P, K) if order_flag else 0)
    M_host = torch.from_numpy(M0.copy()).pin_memory()
    G.gosh_train_parts(n, xadj, adj, M_host, k, epochs, 0.1, 7, level=2, P_gpu=P, S_gpu=S, B=B, force_K=K,
                       flags=G.GOSH_FLAG_SEQUENTIAL | order_flag)
    M_dev = torch.from_numpy(M0.copy()).to(DEV)
    st = G.gosh_train_parts(n, xadj, adj, M_dev, k, epochs, 0.1, 7, level=2, P_gpu=P, S_gpu=S, B=B, force_K=K,
                            flags=G.GOSH_FLAG_SEQUENTIAL | order_flag)
    torch.cuda.synchronize()
    assert np.array_equal(M_dev.cpu().numpy(), M_host.numpy())
    assert rel_err(M_dev.cpu().numpy(), want) <= 1e-5
    assert st["bytes_d2h"] == 0 and st["K"] == K
    if graph_on_device:
        assert st["bytes_h2d"] == 0
    # concurrent kernels, default part count: nothing moves at lr = 0, and training stays finite
    M_dev = torch.from_numpy(M0.copy()).to(DEV)
    st = G.gosh_train_parts(n, xadj, adj, M_dev, k, epochs, 0.0, 7, flags=order_flag)
    assert st["K"] == 16 and np.array_equal(M_dev.cpu().numpy(), M0)
    G.gosh_train_parts(n, xadj, adj, M_dev, k, epochs, 0.05, 7, flags=order_flag)
    assert torch.isfinite(M_dev).all()
