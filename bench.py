#!/usr/bin/env python3
"""Benchmark of the GOSH training path on one MI355X.

A step is one epoch of the epoch kernel (Alg. 3 of the paper: every vertex is the
source of one positive and k negative updates) over a synthetic graph that is
already resident in HBM.  Prints ONE JSON line with the whole-job throughput in
training samples per second, the roofline figures of the epoch kernel (algorithmic
row bytes per launch over the measured launch duration, against 8 TB/s) and the
oracle's single-threaded CPU rate on a bounded slice of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E

WORKLOADS = {
    # Workload 4, level 0: the shape the bandwidth target is stated on.
    "cfg4_level0": dict(gen="chung_lu", log2n=24, log2m=28, d=128, k=3, lr0=0.045, offsets64=True,
                        desc="Chung-Lu power law (exponent 2.1), 2^24 vertices, 2^28 undirected "
                             "edge draws, int64 offsets, d=128 fp32, k=3, level 0"),
    # Workload 3: multilevel run (use --mode levels).
    "cfg3": dict(gen="rmat", log2n=22, log2m=26, d=128, k=3, lr0=0.035, offsets64=False,
                 threshold=10000, min_shrink=0.8,
                 desc="R-MAT, 2^22 vertices, 2^26 undirected edge draws, d=128 fp32, k=3, "
                      "hierarchy to |V| < 10,000 or shrink below 20 %"),
    # Workload 5: the shape of the paper's largest graph, trained with the part-pair
    # rotation under an 8 GB device budget (use --mode parts).
    "cfg5": dict(gen="chung_lu", n=65_000_000, m=1_800_000_000, d=128, k=3, lr0=0.035,
                 offsets64=True, budget=8 << 30,
                 desc="Chung-Lu power law (exponent 2.1), 6.5e7 vertices, 1.8e9 undirected edge "
                      "draws, int64 offsets, d=128 fp32 (33 GB matrix on the host), k=3, "
                      "8 GB device budget"),
    # Workload 2 (matrix 512 MB: partly cache resident).
    "cfg2": dict(gen="rmat", log2n=20, log2m=24, d=128, k=3, lr0=0.045, offsets64=False,
                 desc="R-MAT (0.57,0.19,0.19,0.05), 2^20 vertices, 2^24 undirected edge draws, "
                      "int32 offsets, d=128 fp32, k=3"),
}


def read_traffic(workload: str):
    """HBM bytes per launch measured with rocprofv3 counters, if a summary is committed."""
    path = os.path.join(ROOT, "profiles", f"train_epoch_{workload}_traffic.txt")
    if not os.path.exists(path):
        return None
    vals = {}
    for line in open(path):
        if "=" in line and not line.lstrip().startswith("#"):
            k, v = line.split("=", 1)
            try:
                vals[k.strip()] = float(v.split()[0])
            except ValueError:
                pass
    if "hbm_bytes_per_launch" in vals:
        return vals["hbm_bytes_per_launch"]
    return None


def release_generator_memory(torch) -> None:
    """Give the generator's device memory back and wait until it is usable again.

    The driver clears freed device memory in the background (about 33 GB/s measured on
    this machine).  Until it is done, an allocation that needs memory not yet cleared waits
    for it and host<->device copies run at about half their rate; without the pause the
    timed region would pay for the generator."""
    held = torch.cuda.memory_reserved()
    torch.cuda.empty_cache()
    freed = held - torch.cuda.memory_reserved()
    time.sleep(0.5 + freed / 25e9)


def settle_after_placement(placement) -> None:
    """The arena pieces the placement gave back are being cleared by the driver: wait for that
    before the large allocations that follow (see release_generator_memory)."""
    if placement.get("mode") == "search":
        time.sleep(0.5 + (placement["arena_bytes"] - placement["kept_bytes"]) / 25e9)


def run_levels(args, w, csr, n, n_edges, t_graph) -> int:
    """Coarsening (timed separately) + Alg. 2 over all levels, per-level rates."""
    import torch

    import paper_2008_12336_amd as G

    d, k = w["d"], w["k"]
    if args.graph == "device" and args.coarsen == "device":
        xadj_h, adj_h = csr.xadj, csr.adj  # stays where the generator left it
    else:
        xadj_h, adj_h = csr.xadj.cpu(), csr.adj.cpu()
    del csr
    release_generator_memory(torch)
    budget = int(w.get("budget", 0)) if args.log2n is None else 0
    if args.budget_gb is not None:
        budget = int(args.budget_gb * (1 << 30))
    # the output matrix is allocated before the coarsening takes its scratch
    placement = {"mode": "plain"}
    if budget:
        M0 = torch.empty(n, d, dtype=torch.float32, pin_memory=True)
    elif args.placement == "search":
        from paper_2008_12336_amd.placement import place_matrix

        M0, placement = place_matrix(n, d)
        settle_after_placement(placement)
    else:
        M0 = torch.empty(n, d, dtype=torch.float32, device="cuda:0")
    t0 = time.perf_counter()
    coarsen = G.gosh_coarsen_device if args.coarsen == "device" else G.gosh_coarsen
    h = coarsen(n, xadj_h, adj_h, threshold=w.get("threshold", 100),
                min_shrink=w.get("min_shrink", 0.8))
    t_coarsen = time.perf_counter() - t0
    coarsen_stages = [dict(level=i, **h.times(i)) for i in range(h.levels - 1)]
    print(f"[bench] hierarchy of {h.levels} levels in {t_coarsen:.1f}s; budget {budget}",
          file=sys.stderr, flush=True)
    if budget:
        # Alg. 2 with its fits-into-GPU test: levels above the budget use the rotation
        t0 = time.perf_counter()
        stats = G.gosh_embed_host(h, M0, k, args.epochs, 0.3, w["lr0"], args.seed, flags=args.flags,
                                  device_budget_bytes=budget, P_gpu=args.p_gpu, S_gpu=args.s_gpu)
    else:
        t0 = time.perf_counter()
        stats = G.gosh_embed(h, M0, k, args.epochs, 0.3, w["lr0"], args.seed, flags=args.flags)
    torch.cuda.synchronize()
    t_embed = time.perf_counter() - t0
    levels = []
    samples = 0
    train_ms = 0.0
    for s_ in stats:
        per_epoch = s_["train_ms"] / max(1, s_["epochs"])
        row_bytes = s_["n"] * (2 + 2 * (k + 1)) * 4 * d
        levels.append({"level": s_["level"], "n": s_["n"], "nnz": s_["nnz"], "epochs": s_["epochs"],
                       "parts_K": s_["parts_K"], "train_ms": s_["train_ms"],
                       "ms_per_epoch": per_epoch, "row_GBps": row_bytes / per_epoch / 1e6,
                       "upload_ms": s_["upload_ms"], "project_ms": s_["project_ms"]})
        samples += s_["n"] * (k + 1) * s_["epochs"]
        train_ms += s_["train_ms"]
    out = {"metric": "training samples/sec and achieved HBM GB/s (% of peak) at d=128, 1 GPU",
           "value": samples / (train_ms / 1e3), "unit": "samples/s", "n_gpus": 1,
           "steps": args.epochs, "warmup": 0, "ms_per_step": train_ms / args.epochs,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
           "data": "synthetic",
           "config": {"workload": args.workload + "_levels", "desc": w["desc"], "n": n,
                      "device_budget_bytes": budget, "finite": bool(torch.isfinite(M0[::4097]).all()),
                      "undirected_edges": n_edges, "d": d, "k_neg": k, "total_epochs": args.epochs,
                      "coarsen": args.coarsen, "graph": args.graph, "placement": placement, "coarsen_s": t_coarsen, "coarsen_stages": coarsen_stages, "embed_wall_s": t_embed, "graph_build_s": t_graph,
                      "levels": levels}}
    print(json.dumps(out))
    return 0


def run_parts(args, w, csr, n, n_edges, t_graph) -> int:
    """One rotation of the part-pair scheme with the matrix on the (pinned) host."""
    import torch

    import paper_2008_12336_amd as G

    d, k, B = w["d"], w["k"], 5
    placement = {"mode": "plain"}
    if args.graph == "device":
        xadj_h, adj_h = csr.xadj, csr.adj  # sampled where the generator left it
    else:
        xadj_h, adj_h = csr.xadj.cpu(), csr.adj.cpu()
    del csr
    release_generator_memory(torch)
    M_dev = torch.empty(n, d, dtype=torch.float32, device="cuda:0")
    G.gosh_init_embedding(M_dev, args.seed, 0)
    if args.matrix == "device":
        # every part trained where it is: the pair order and sampling rule of Alg. 5 without
        # its copies (the budget then only covers the pools)
        M_host, budget = M_dev, 0
        if args.placement == "search":
            from paper_2008_12336_amd.placement import place_matrix

            del M_dev, M_host
            M_host, placement = place_matrix(n, d)
            settle_after_placement(placement)
            G.gosh_init_embedding(M_host, args.seed, 0)
        K = args.parts if args.parts > 0 else 16
        st = G.gosh_train_parts(n, xadj_h, adj_h, M_host, k, B * K, w["lr0"], args.seed, S_gpu=args.s_gpu,
                                B=B, force_K=K, flags=args.flags)
        torch.cuda.synchronize()
    else:
        M_host = torch.empty(n, d, dtype=torch.float32, pin_memory=True)
        M_host.copy_(M_dev)
        del M_dev
        release_generator_memory(torch)
        print("[bench] matrix on the pinned host", file=sys.stderr, flush=True)
        if "budget" in w and args.log2n is None:
            budget = int(w["budget"])
        else:
            budget = int(n * d * 4 / args.budget_ratio)
        print(f"[bench] parts: n={n} budget={budget}", file=sys.stderr, flush=True)
        plan = G.gosh_parts_plan(n, d, 1, budget, args.p_gpu, args.s_gpu, B)
        epochs = B * plan["K"]  # exactly one rotation
        st = G.gosh_train_parts(n, xadj_h, adj_h, M_host, k, epochs, w["lr0"], args.seed,
                                device_budget_bytes=budget, P_gpu=args.p_gpu, S_gpu=args.s_gpu, B=B,
                                flags=args.flags)
    out = {"metric": "training samples/sec and achieved HBM GB/s (% of peak) at d=128, 1 GPU",
           "value": st["updates"] / (st["wall_ms"] / 1e3), "unit": "samples/s", "n_gpus": 1,
           "steps": 1, "warmup": 0, "ms_per_step": st["wall_ms"], "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": args.workload + "_parts", "desc": w["desc"], "n": n,
                      "undirected_edges": n_edges, "d": d, "k_neg": k, "B": B, "graph": args.graph, "matrix": args.matrix, "placement": placement,
                      "ms_per_epoch_worth_of_samples": st["wall_ms"] / (B * st["K"] * st["rotations"]),
                      "flags": args.flags, "P_gpu": args.p_gpu,
                      "S_gpu": args.s_gpu, "device_budget_bytes": budget, "matrix_bytes": n * d * 4,
                      "graph_build_s": t_graph, "finite": bool(torch.isfinite(M_host[::4097]).all()),
                      **st,
                      "kernel_only_samples_per_s": st["updates"] / (st["kernel_ms"] / 1e3),
                      "h2d_GBps_wall": st["bytes_h2d"] / st["wall_ms"] / 1e6,
                      "d2h_GBps_wall": st["bytes_d2h"] / st["wall_ms"] / 1e6,
                      "sampler_ms": st["sampler_ms"], "sampler_wait_ms": st["sampler_wait_ms"]}}
    print(json.dumps(out))
    return 0


def run_probe(args, w, n) -> int:
    """What the memory system allows a kernel that moves rows of 4*d bytes at random: the
    library's row probe (gosh_row_probe: the kernels' traffic without their arithmetic) in its
    four modes, on a matrix in an allocation of its own and on a placed one, beside a plain
    streaming copy of the same matrix.  No graph is involved."""
    import numpy as np
    import torch

    import paper_2008_12336_amd as G

    d = w["d"]
    row = 4 * d
    modes = [("read_write", G.GOSH_PROBE_READ_WRITE, 2, 4 * n), ("read", G.GOSH_PROBE_READ, 1, 8 * n),
             ("epoch_mix", G.GOSH_PROBE_EPOCH_MIX, 10, n), ("write", G.GOSH_PROBE_WRITE, 1, 8 * n)]
    results = {}
    windows = [("plain", None)]
    if args.placement == "search":
        windows.append(("placed", None))
    for where, _ in windows:
        placement = {"mode": "plain"}
        if where == "placed":
            from paper_2008_12336_amd.placement import place_matrix

            M, placement = place_matrix(n, d)
            settle_after_placement(placement)
        else:
            M = torch.empty(n, d, dtype=torch.float32, device="cuda:0")
        G.gosh_init_embedding(M, args.seed, 0)
        torch.cuda.synchronize()
        res = {"placement": placement}
        for name, mode, transfers, accesses in modes:
            ms = []
            for rep in range(args.warmup + args.steps):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                G.gosh_row_probe(M, accesses, seed=args.seed + rep, mode=mode)
                b.record()
                torch.cuda.synchronize()
                if rep >= args.warmup:
                    ms.append(a.elapsed_time(b))
            med = float(np.median(ms))
            res[name] = {"ms": med, "accesses": accesses, "row_transfers_per_access": transfers,
                         "GBps": accesses * transfers * row / med / 1e6,
                         "G_rows_per_s": accesses * transfers / med / 1e6}
        if where == "plain":
            other = torch.empty_like(M)
            ms = []
            for rep in range(args.warmup + args.steps):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                other.copy_(M)
                b.record()
                torch.cuda.synchronize()
                if rep >= args.warmup:
                    ms.append(a.elapsed_time(b))
            med = float(np.median(ms))
            res["streaming_copy"] = {"ms": med, "GBps": 2 * n * row / med / 1e6}
            del other
        results[where] = res
        if where == "placed" and placement.get("mode") == "search":
            G.gosh_matrix_release(M)
        del M
    out = {"metric": "row probe: random row traffic without arithmetic", "unit": "GB/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"row_probe_n{n}_d{d}", "n": n, "d": d, "row_bytes": row,
                      "matrix_bytes": n * row},
           "peak_GBps": HBM_PEAK_GBPS, "probe": results}
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg4_level0", choices=sorted(WORKLOADS))
    ap.add_argument("--log2n", type=int, default=None, help="override vertex count (scaled runs)")
    ap.add_argument("--log2m", type=int, default=None, help="override edge draws (scaled runs)")
    ap.add_argument("--d", type=int, default=None)
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--mode", default="epoch", choices=["epoch", "levels", "parts", "probe"],
                    help="epoch: the epoch kernel on one graph (the headline number); levels: "
                         "coarsening + multilevel training with per-level rates; parts: one "
                         "rotation of the part-pair scheme under a device budget; probe: the "
                         "library's row probe on a matrix of the workload's shape (no graph): "
                         "what the memory system allows random row traffic of 4*d bytes")
    ap.add_argument("--coarsen", default="device", choices=["device", "host"],
                    help="--mode levels: where the coarse graphs are rebuilt")
    ap.add_argument("--graph", default="host", choices=["host", "device"],
                    help="--mode levels with --coarsen device, --mode parts: where G_0 is handed over")
    ap.add_argument("--placement", default="search", choices=["search", "plain"],
                    help="--mode epoch: where the matrix lies (search: the fastest window of a large "
                         "arena, which straddles two HBM ranks; plain: an allocation of its own)")
    ap.add_argument("--matrix", default="host", choices=["host", "device"],
                    help="--mode parts: where the matrix lives (device: parts trained in place, no copies)")
    ap.add_argument("--parts", type=int, default=0, help="--mode parts --matrix device: part count (default 16)")
    ap.add_argument("--epochs", type=int, default=40, help="total epochs of --mode levels")
    ap.add_argument("--p-gpu", type=int, default=3, help="--mode parts: device slots for parts")
    ap.add_argument("--s-gpu", type=int, default=4, help="--mode parts: device sample pools")
    ap.add_argument("--budget-ratio", type=float, default=4.2,
                    help="--mode parts: matrix bytes / device budget")
    ap.add_argument("--budget-gb", type=float, default=None,
                    help="--mode levels: device budget in GiB instead of the workload's "
                         "(0 = none: every level resident)")
    ap.add_argument("--flags", type=int, default=0,
                    help="gosh_train_epoch flags (0 = default mix of plain stores and atomic adds)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain device copy of the matrix (known size) so that "
                         "profiler byte counters can be scaled against it")
    ap.add_argument("--cpu-seconds", type=float, default=15.0,
                    help="CPU time budget for the oracle baseline slice (0 = skip)")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import graphgen
    import paper_2008_12336_amd as G

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the training path has no CPU fallback", file=sys.stderr)
        return 2
    G.lib()  # fail loudly if libgosh.so is missing

    w = dict(WORKLOADS[args.workload])
    scaled = False
    for key in ("log2n", "log2m", "d"):
        if getattr(args, key) is not None:
            w[key] = getattr(args, key)
            scaled = True
    n = w["n"] if "n" in w and args.log2n is None else 1 << w["log2n"]
    m = w["m"] if "m" in w and args.log2m is None else 1 << w["log2m"]
    d, k = w["d"], w["k"]
    dev = "cuda:0"
    if args.mode == "probe":
        return run_probe(args, w, n)

    t0 = time.time()
    if w["gen"] == "chung_lu":
        edges = graphgen.chung_lu(n, m, args.seed, gamma=2.1, device=dev)
    else:
        edges = graphgen.rmat(w["log2n"], m, args.seed, device=dev)
    print(f"[bench] graph generated: {int(edges.shape[0])} edges", file=sys.stderr, flush=True)
    csr = graphgen.to_csr(n, edges, offsets64=w["offsets64"])
    n_edges = int(edges.shape[0])
    del edges
    torch.cuda.synchronize()
    t_graph = time.time() - t0
    g = G.csr_view(n, csr.xadj, csr.adj)

    if args.mode == "levels":
        return run_levels(args, w, csr, n, n_edges, t_graph)
    if args.mode == "parts":
        return run_parts(args, w, csr, n, n_edges, t_graph)

    placement = {"mode": "plain"}
    if args.placement == "search":
        release_generator_memory(torch)
        from paper_2008_12336_amd.placement import place_matrix

        M, placement = place_matrix(n, d)
    else:
        M = torch.empty(n, d, dtype=torch.float32, device=dev)
    G.gosh_init_embedding(M, args.seed, 0)
    torch.cuda.synchronize()

    total_epochs = args.warmup + args.steps
    for j in range(args.warmup):
        G.gosh_train_epoch(g, M, k, G.gosh_lr(w["lr0"], j, total_epochs), args.seed, j, 0, args.flags)
    torch.cuda.synchronize()

    starts = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    ends = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        j = args.warmup + i
        starts[i].record()  # same (current) stream the kernel is launched on
        G.gosh_train_epoch(g, M, k, G.gosh_lr(w["lr0"], j, total_epochs), args.seed, j, 0, args.flags)
        ends[i].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    kernel_ms = [s.elapsed_time(e) for s, e in zip(starts, ends)]
    avg_kernel_s = float(np.mean(kernel_ms)) / 1e3
    finite = bool(torch.isfinite(M[:: max(1, n // 4096)]).all())

    if args.copy_calibration:
        scratch = torch.empty_like(M)
        scratch.copy_(M)  # reads and writes n*d*4 bytes each
        torch.cuda.synchronize()
        del scratch

    samples_per_step = n * (k + 1)
    value = samples_per_step * args.steps / elapsed
    # Algorithmic row traffic: the source row is read and written once, each of the k+1
    # sample rows is read and written once: (2 + 2(k+1)) * 4d bytes per source.
    row_bytes_per_launch = n * (2 + 2 * (k + 1)) * 4 * d
    achieved = row_bytes_per_launch / avg_kernel_s / 1e9
    traffic = None if scaled else read_traffic(args.workload)

    cpu = cpu_hogwild = None
    if args.cpu_seconds > 0:
        from oracle import gosh_oracle as O  # cpu_baseline leg only

        xadj_h = csr.xadj.cpu().numpy().astype(np.int64)
        adj_h = csr.adj.cpu().numpy()
        M_h = M.cpu().numpy()
        probe = min(n, 1 << 15)
        t1 = time.perf_counter()
        O.train_sources(xadj_h, adj_h, M_h, k, 0.01, args.seed, total_epochs, 0, 0, probe)
        dt = time.perf_counter() - t1
        count = int(min(n - probe, max(probe, args.cpu_seconds / max(dt, 1e-6) * probe)))
        t1 = time.perf_counter()
        O.train_sources(xadj_h, adj_h, M_h, k, 0.01, args.seed, total_epochs, 0, probe, count)
        dt = time.perf_counter() - t1
        cpu = {"value": count * (k + 1) / dt, "unit": "samples/s", "cores": 1, "kind": "oracle",
               "sample": f"sources {probe}..{probe + count - 1} of one sequential epoch on the same "
                         f"graph and matrix ({count * (k + 1)} updates, {dt:.1f} s)"}
        # the paper's own CPU baseline is the same loop, lock-free on all cores (Sec. 4.8)
        threads = min(os.cpu_count() or 1, 16)
        hog_count = int(min(n - probe, count * threads // 2))
        t1 = time.perf_counter()
        O.train_sources_hogwild(xadj_h, adj_h, M_h, k, 0.01, args.seed, total_epochs, 0, probe, hog_count,
                                threads)
        dt = time.perf_counter() - t1
        cpu_hogwild = {"value": hog_count * (k + 1) / dt, "unit": "samples/s", "cores": threads,
                       "kind": "oracle loop under an OpenMP parallel-for (Hogwild)",
                       "sample": f"sources {probe}..{probe + hog_count - 1} of one epoch "
                                 f"({hog_count * (k + 1)} updates, {dt:.1f} s)"}
        del M_h, xadj_h, adj_h

    out = {
        "metric": "training samples/sec and achieved HBM GB/s (% of peak) at d=128, 1 GPU",
        "value": value,
        "unit": "samples/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": args.workload + ("_scaled" if scaled else ""), "desc": w["desc"],
                   "n": n, "undirected_edges": n_edges, "nnz": int(csr.adj.numel()), "d": d,
                   "k_neg": k, "seed": args.seed, "flags": args.flags, "placement": placement, "graph_build_s": round(t_graph, 2),
                   "finite": finite},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                     "traffic_source": None if traffic is None else
                     f"profiles/train_epoch_{args.workload}_traffic.txt (rocprofv3 counters of an earlier run of "
                     "this command, calibrated on a copy of known size; quoted, not measured by this run)",
                     "kernel": "sgd_kernel<EpochWork>", "kernel_ms_avg": avg_kernel_s * 1e3,
                     "kernel_ms_min": float(np.min(kernel_ms)),
                     "algorithmic_bytes_per_launch": row_bytes_per_launch},
        "cpu_baseline": cpu,
        "cpu_baseline_hogwild": cpu_hogwild,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
