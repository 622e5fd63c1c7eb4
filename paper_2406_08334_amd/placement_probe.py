"""Diagnostic: how the speed of the update depends on where its arrays lie in physical memory.

    python -m paper_2406_08334_amd.placement_probe [--anchors 0,105,220] [--chunks 8]

Fills the free device memory with 1 GiB allocations (in a fresh process on an idle GPU they
come out of physical memory in order), then
  1. for a few anchor allocations holding the gradient, parameter, master and momentum arrays
     of one chunk, times pt_chunk_adamw_step with the variance array in every other allocation
     and prints the runs of allocations that are fast / slow partners of the anchor: the
     boundaries are the boundaries of the memory's regions;
  2. times the update of a few chunks with each of the five arrays assigned to one of the
     regions found (named A, B, C ...), for a list of assignments.
Uses nothing but the library's public calls; needs the GPU to itself.
"""
from __future__ import annotations

import argparse

import torch

from . import binding as B

S = 1 << 26
MIB = 1 << 20
GIB = 1 << 30


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--anchors", default="0,105,220", help="indices of the anchor allocations")
    ap.add_argument("--chunks", type=int, default=8, help="chunks per timed launch in part 2")
    ap.add_argument("--leave-gib", type=int, default=22, help="device memory left unallocated")
    args = ap.parse_args()
    dev = "cuda"
    free, _ = torch.cuda.mem_get_info()
    n_pool = max(8, free // GIB - args.leave_gib)
    pool = [torch.zeros(GIB, dtype=torch.uint8, device=dev) for _ in range(n_pool)]
    print(f"{n_pool} allocations of 1 GiB", flush=True)
    ctx = B.pt_ctx_create(B.PT_BF16, S, args.chunks, None)
    hp = B.hparams(1e-4, 0.9, 0.95, 1e-8, 0.1, 1.0)
    st = torch.cuda.current_stream()

    def rate(g, p, w, m, v, reps=3):
        n = len(g)
        ts = []
        for _ in range(reps):
            B.pt_step_override(ctx, 0.0121, False, st)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(st)
            B.pt_chunk_adamw_step(ctx, hp, 0, n, g, w, m, v, p, st)
            e1.record(st)
            B.pt_step_end(ctx, st)
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        return 28 * S * n / min(ts) / 1e6

    # ---- part 1: partners of an anchor
    edges = set()
    for a in [int(x) for x in args.anchors.split(",") if int(x) < n_pool]:
        base = pool[a].data_ptr()
        g, p, w, m = base + 768 * MIB, base + 896 * MIB, base, base + 256 * MIB
        marks = []
        for i in range(n_pool):
            if i == a:
                marks.append(".")
                continue
            r = rate([g], [p], [w], [m], [pool[i].data_ptr()])
            marks.append("FAST" if r > 6150 else ("slow" if r < 5950 else "mid"))
        runs, start = [], 0
        for i in range(1, n_pool + 1):
            if i == n_pool or marks[i] != marks[start]:
                runs.append(f"{start}-{i - 1}:{marks[start]}")
                if i < n_pool and {marks[start], marks[i]} == {"FAST", "slow"}:
                    edges.add(i)
                start = i
        print(f"anchor {a:3d} (g, p, w, m inside it; v elsewhere): " + " ".join(runs), flush=True)
    bounds = [0] + sorted(edges) + [n_pool]
    regions = [(bounds[i], bounds[i + 1]) for i in range(len(bounds) - 1) if bounds[i + 1] - bounds[i] >= 40]
    print("regions (allocation indices):", regions, flush=True)
    if len(regions) < 2:
        print("fewer than two regions found: nothing to assign")
        return 0

    # ---- part 2: assignments of the five arrays to regions
    names = "ABCDEFGH"[:len(regions)]
    start_of = {names[i]: regions[i][0] + 8 for i in range(len(regions))}
    n = args.chunks

    def rows(letter, kind):
        off = {"g": 0, "p": 4, "w": 8, "m": 16, "v": 24}[kind]
        per, step = (8, 128 * MIB) if kind in "gp" else (4, 256 * MIB)
        return [pool[start_of[letter] + off + c // per].data_ptr() + (c % per) * step for c in range(n)]

    last = names[-1]
    mid = names[1]
    cases = ["AAAAA", "AAAA" + mid, "AAA" + mid + "A", "AA" + mid + "AA", "AAA" + mid + mid, "AAA" + mid + last,
             mid + last + "A" + mid + last, mid + mid + "AAA", last + last + "AAA", "AA" + mid * 3]
    for case in dict.fromkeys(cases):
        r = rate(rows(case[0], "g"), rows(case[1], "p"), rows(case[2], "w"), rows(case[3], "m"), rows(case[4], "v"), reps=4)
        print(f"g p w m v = {' '.join(case)} : {r:6.0f} GB/s", flush=True)
    B.pt_ctx_destroy(ctx)
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
