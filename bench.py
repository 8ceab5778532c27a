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
    # BASELINE config 4, level 0: the shape the bandwidth target is stated on.
    "cfg4_level0": dict(gen="chung_lu", log2n=24, log2m=28, d=128, k=3, lr0=0.045, offsets64=True,
                        desc="Chung-Lu power law (exponent 2.1), 2^24 vertices, 2^28 undirected "
                             "edge draws, int64 offsets, d=128 fp32, k=3, level 0"),
    # BASELINE config 2 (matrix 512 MB: partly cache resident).
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
    n, m, d, k = 1 << w["log2n"], 1 << w["log2m"], w["d"], w["k"]
    dev = "cuda:0"

    t0 = time.time()
    if w["gen"] == "chung_lu":
        edges = graphgen.chung_lu(n, m, args.seed, gamma=2.1, device=dev)
    else:
        edges = graphgen.rmat(w["log2n"], m, args.seed, device=dev)
    csr = graphgen.to_csr(n, edges, offsets64=w["offsets64"])
    n_edges = int(edges.shape[0])
    del edges
    torch.cuda.synchronize()
    t_graph = time.time() - t0
    g = G.csr_view(n, csr.xadj, csr.adj)

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

    cpu = None
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
                   "k_neg": k, "seed": args.seed, "flags": args.flags, "graph_build_s": round(t_graph, 2),
                   "finite": finite},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                     "kernel": "train_epoch_kernel", "kernel_ms_avg": avg_kernel_s * 1e3,
                     "kernel_ms_min": float(np.min(kernel_ms)),
                     "algorithmic_bytes_per_launch": row_bytes_per_launch},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
