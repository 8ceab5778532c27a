"""Choosing where in device memory an embedding matrix lies.

The HBM of an MI355X answers in three classes of addresses -- its stacks are twelve dies
high, three ranks of four, 96 GB per rank over the eight stacks -- and random 512-byte row
traffic confined to one class runs at about 5.2 TB/s, spread over two at about 6.2 TB/s (a
probe of plain random row read-modify-writes: 4.7 against 5.35 TB/s).  An allocation of a few
GB lies inside one class.  `place_matrix` takes a large arena, times the library's row probe
(random rows read and written back unchanged: the training kernels' traffic without their
arithmetic) on windows of it and hands back the fastest window, in practice one that
straddles the border between two classes.  Nothing here computes anything of the method.
"""
from __future__ import annotations

import time

import torch

from . import binding as G


def place_matrix(n: int, d: int, seed: int = 1, arena_bytes: int = 120 << 30,
                 keep_free_bytes: int = 24 << 30):
    """Returns (M, arena, info): M is an n x d float32 window of `arena` (keep `arena` alive
    as long as M is used), or a plain allocation with arena None if no arena of at least three
    times the matrix can be had.  The windows are timed with gosh_row_probe, 4n accesses each
    (half a window apart but at most 4 GiB, then four times finer around the best); M comes
    back uninitialised.  The whole arena stays allocated while M is in use -- the price of the
    placement; a smaller arena_bytes holds less but may contain no border (borders were seen
    16 to 64 GiB apart), in which case the first window comes back and nothing is gained."""
    row_bytes = d * 4
    need = n * row_bytes
    free_bytes, _ = torch.cuda.mem_get_info()
    arena_bytes = min(arena_bytes, free_bytes - keep_free_bytes)
    if arena_bytes < 3 * need:
        return torch.empty(n, d, dtype=torch.float32, device="cuda"), None, {"mode": "plain (no room for an arena)"}
    t0 = time.perf_counter()
    try:
        arena = torch.empty(arena_bytes // row_bytes, d, dtype=torch.float32, device="cuda")
    except RuntimeError:
        return torch.empty(n, d, dtype=torch.float32, device="cuda"), None, {"mode": "plain (arena refused)"}
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def epoch_ms(first_row: int) -> float:
        window = arena[first_row:first_row + n]
        start.record()
        G.gosh_row_probe(window, 4 * n, seed)
        stop.record()
        torch.cuda.synchronize()
        return start.elapsed_time(stop)

    rows_per_gib = max(1, (1 << 30) // row_bytes)
    last = arena.shape[0] - n
    # a window gains only while it straddles a border, i.e. within its own length of one: scan
    # at half the window's length (at most 4 GiB, at most about a thousand windows), then at
    # an eighth around the best
    coarse = max(1, min(4 * rows_per_gib, max(n // 2, last // 1000)))
    fine = max(1, coarse // 4)
    timed = {r: epoch_ms(r) for r in range(0, last + 1, coarse)}
    best = min(timed, key=timed.get)
    for r in range(max(0, best - 3 * fine), min(last, best + 3 * fine) + 1, fine):
        if r not in timed:
            timed[r] = epoch_ms(r)
    best = min(timed, key=timed.get)
    # The gain falls off linearly on both sides of the best position (a window sliding off a
    # border between two classes): the centre of gravity of the gains around the fastest
    # window is a steadier estimate of that position than the fastest single timing.
    median = sorted(timed.values())[len(timed) // 2]
    near = {r: median - t for r, t in timed.items() if abs(r - best) <= coarse and t < median}
    if near and sum(near.values()) > 0:
        centre = int(sum(r * w for r, w in near.items()) / sum(near.values()))
        centre = max(0, min(last, centre))
        timed[centre] = epoch_ms(centre)
        if timed[centre] <= timed[best] * 1.01:
            best = centre
    info = {"mode": "search", "arena_GiB": arena_bytes / (1 << 30), "window_at_GiB": best / rows_per_gib,
            "probe_ms_best": timed[best], "probe_ms_median": sorted(timed.values())[len(timed) // 2],
            "windows_timed": len(timed), "search_s": time.perf_counter() - t0}
    return arena[best:best + n], arena, info
