#!/usr/bin/env python3
"""Benchmark of the chunked model-state hot path on one MI355X.

One "step" = pt_chunk_pack_grads -> pt_chunk_grad_sqnorm(finalize) -> pt_chunk_adamw_step
-> pt_step_end over a whole synthetic model state that is resident in HBM.  The headline
workload is the LLaMA-7B-shaped state (101 chunks of 2^26 elements, bf16 params/grads + fp32
master/m/v).  Prints ONE JSON line: whole-step algorithmic GB/s and ms/step, the roofline of
the dominant kernel (the fused AdamW update, 28 B/element) measured with events on the launch
stream, two calibrations of the box (a plain copy kernel, and the update's own access pattern
with the arithmetic taken out), the CPU oracle timed on a bounded sample of the same state,
and - unless --headline-only - one entry per other benchmark configuration under
"other_configs": the GPT-2 block, the GPT-2-XL shape with outlier gradients, the LLaMA-7B shape
in fp16 with dynamic loss scaling, and the LLaMA-13B shape with half of the chunks in pinned
host memory (streamed through chunk buffers, and updated by host threads).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llama_7b] [--headline-only]
    python bench.py --stream [--host-update] [--model]                 # the split configuration alone
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "chunked AdamW step: achieved HBM GB/s (% of peak) + ms/step, 7B-shaped state"
HBM_PEAK_GBPS = 8000.0
HP = dict(lr=1e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, max_norm=1.0)
ADAMW_BYTES_PER_ELEM = 28          # read g16 2 + w,m,v 12 ; write w,m,v 12 + p16 2
PACK_BYTES_PER_ELEM = 4            # read 2 + write 2

# HBM traffic of one AdamW launch from rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE, scaled by the
# same counters on pt_calib_copy); filled from the summaries under profiles/.  bytes per launch.
MEASURED_TRAFFIC = {
    # profiles/k_adamw_llama7b_hbm_traffic.md: (46 334 527.47 x 1.999776 + 92 669 076.19 x 0.999986) KiB
    "llama_7b": 189_774_262_972,
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def mean(x):
    return float(sum(x) / len(x))


def median(x):
    s = sorted(x)
    n = len(s)
    return float(s[n // 2] if n % 2 else 0.5 * (s[n // 2 - 1] + s[n // 2]))


def release():
    import torch
    gc.collect()
    torch.cuda.synchronize()
    torch.cuda.empty_cache()


def host_memory_gb():
    try:
        for line in open("/proc/meminfo"):
            if line.startswith("MemTotal:"):
                return round(int(line.split()[1]) * 1024 / 1e9, 1)
    except OSError:
        pass
    return None


# ------------------------------------------------------------------------------- all chunks resident

def run_resident(workload, steps, warmup, fp16=False, grad_sets=3, layout="dense", no_decay_1d=False, grad_accum=0,
                 zero_grads=False, graph=False, unpack=False, calib=False, cpu_sample_chunks=0, cpu_one_thread_chunks=0):
    """One configuration with every chunk resident in HBM.  Returns the measurement as a dict."""
    import numpy as np
    import torch

    from paper_2406_08334_amd import binding as B
    from paper_2406_08334_amd import shapes, synth
    from paper_2406_08334_amd.arena import spread_arenas

    dev = "cuda:0"
    table, S = shapes.workload(workload)
    sizes = [n for _, n in table]
    N = sum(sizes)
    layout_note = "dense layout (tensors cut at chunk boundaries, last chunk padded)"
    if layout == "grouped":
        # the paper's layout: no tensor split, one transformer block per chunk, chunk size by least waste
        gids = shapes.block_ids(table)
        per_block = {}
        for n, g in zip(sizes, gids):
            if g is not None:
                per_block[g] = per_block.get(g, 0) + n
        t_s = time.perf_counter()
        S, C, waste = B.pt_chunk_size_search(sizes, gids, max(per_block.values()), 1 << 25, 1 << 20)
        segs, C, waste = B.pt_layout_grouped(sizes, gids, S)
        layout_note = (f"grouped layout (no tensor split, blocks kept whole; searched chunk size {S}, waste {waste} "
                       f"elements = {100.0 * waste / N:.2f} %, search + layout {1e3 * (time.perf_counter() - t_s):.1f} ms on the host)")
    else:
        segs, C = B.pt_layout_dense(sizes, S)
    N_pad = C * S
    n_sets = max(1, min(grad_sets, steps + warmup))
    log(f"[bench] workload {workload}{' fp16' if fp16 else ''}: {N:,} elements, {C} chunks of {S:,}; {layout_note}; "
        f"state {16 * N_pad / 1e9:.2f} GB + {n_sets} gradient sets of {2 * N / 1e9:.2f} GB")

    t0 = time.time()
    dt16 = torch.float16 if fp16 else torch.bfloat16
    sigma = 65536.0 if fp16 else 1.0
    ctx = B.pt_ctx_create(B.PT_FP16 if fp16 else B.PT_BF16, S, C, B.pt_scaler_cfg(sigma, 2.0, 0.5, 2000, 0) if fp16 else None)
    outlier_every = 1000 if workload == "gpt2_xl" else 0      # 0.1 % of the gradients x100: clipping triggers
    if no_decay_1d:
        one_d = {i for i, (name, _) in enumerate(table) if name.endswith(".bias") or "norm" in name or ".ln_" in name}
        nd = [B.pt_segment(0, 0, s.len, s.chunk_off, s.chunk, s.tensor) for s in segs if s.tensor in one_d]
        B.pt_ctx_set_no_decay(ctx, nd)
        layout_note += f"; {len(one_d)} one-dimensional tensors ({sum(s.len for s in nd)} elements) without weight decay"
    A = grad_accum
    if A:
        B.pt_ctx_set_option(ctx, "grad_fp32", 1)
        layout_note += f"; {A} micro-batches per step accumulated into fp32 gradient chunks"
    if zero_grads:
        B.pt_ctx_set_option(ctx, "adamw_zero_grads", 1)
        layout_note += "; gradients zeroed by the update"
    # The five state arenas are spread over the physical memory (see arena.py).  fp32 gradient chunks are read,
    # added to and written back by one kernel: their arena is cut in two halves, the second allocated last,
    # behind the source gradient sets, so that the accumulate kernel's two tile streams fall on distant memory.
    g_dtype = torch.float32 if A else dt16
    C_lo = C // 2 if A else C
    specs = [((C_lo, S), g_dtype), ((C, S), dt16), ((C, S), torch.float32), ((C, S), torch.float32), ((C, S), torch.float32)]
    if C_lo < C:
        specs += [((N,), dt16)] * n_sets + [((C - C_lo, S), g_dtype)]
    arenas = spread_arenas(specs, device=dev, keep_free_bytes=(2 * N if layout == "grouped" else 0) +
                           (0 if C_lo < C else 2 * N * n_sets))
    g16, p16, w, m, v = arenas[:5]
    grad_set_mem = arenas[5:5 + n_sets] if C_lo < C else [torch.empty(N, dtype=dt16, device=dev) for _ in range(n_sets)]
    g_hi = arenas[-1] if C_lo < C else None
    del arenas
    offs = np.cumsum([0] + sizes[:-1]).tolist()
    if layout == "grouped":
        # parameters are generated as the model's tensors and brought into chunk space by the same copy
        flat = torch.empty(N, dtype=dt16, device=dev)
        synth.normal_16(synth.SEED_PARAMS, 0, 0, 0, N, 0.02, dt16, dev, out=flat)
        for s in segs:
            s.src = flat.data_ptr() + 2 * offs[s.tensor]
        plan0 = B.pt_pack_plan_create(ctx, segs)
        B.pt_chunk_pack_grads(ctx, plan0, [p16[c] for c in range(C)], torch.cuda.current_stream())
        torch.cuda.synchronize()
        B.pt_pack_plan_destroy(plan0)
        del flat
    else:
        synth.normal_16(synth.SEED_PARAMS, 0, 0, 0, N, 0.02, dt16, dev, out=p16.view(-1)[:N])
    for c in range(C):
        w[c].copy_(p16[c])
    grad_sets_, plans = [], []
    for k in range(n_sets):
        gs = grad_set_mem[k]
        synth.normal_16(synth.SEED_GRADS, k + 1, 0, 0, N, 1e-3, dt16, dev, scale=sigma, outlier_every=outlier_every, out=gs)
        for s in segs:
            s.src = gs.data_ptr() + 2 * offs[s.tensor]
        grad_sets_.append(gs)
        plans.append(B.pt_pack_plan_create(ctx, segs))
    torch.cuda.synchronize()
    log(f"[bench] state generated in {time.time() - t0:.1f} s")

    hp = B.hparams(**HP)
    rows = lambda a: [a[c] for c in range(C)]
    r_g, r_w, r_m, r_v, r_p = [g16[c] for c in range(C_lo)], rows(w), rows(m), rows(v), rows(p16)
    if g_hi is not None:
        r_g += [g_hi[c] for c in range(C - C_lo)]
    stream = torch.cuda.current_stream()

    # ---- CPU baseline input: the sample chunks' state BEFORE any step (the oracle runs afterwards)
    n_cpu = max(0, min(max(cpu_sample_chunks, cpu_one_thread_chunks), C))
    cpu_in = None
    if n_cpu and not (A or fp16 or layout != "dense" or no_decay_1d):
        u16 = lambda t: t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16).reshape(-1).copy()
        cpu_in = dict(p=u16(p16[:n_cpu]), w=w[:n_cpu].cpu().numpy().reshape(-1).copy(), src=u16(grad_sets_[0][:n_cpu * S]))

    def one_step(k, ev=None):
        if A:
            for j in range(A):
                B.pt_chunk_accum_grads(ctx, plans[(k * A + j) % n_sets], r_g, j == 0, j == A - 1, stream)
        else:
            B.pt_chunk_pack_grads(ctx, plans[k % n_sets], r_g, stream)
        if ev: ev[0].record(stream)
        B.pt_chunk_grad_sqnorm(ctx, None, 0, C, True, stream)
        if ev: ev[1].record(stream)
        B.pt_chunk_adamw_step(ctx, hp, 0, C, r_g, r_w, r_m, r_v, r_p, stream)
        if ev: ev[2].record(stream)
        B.pt_step_end(ctx, stream)

    for k in range(warmup):
        one_step(k)
    torch.cuda.synchronize()

    K = steps
    # the K timed steps: nothing but the step's own calls between the two synchronisations
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for k in range(K):
        one_step(warmup + k)
    torch.cuda.synchronize()
    t_total = time.perf_counter() - t_start
    # K more steps with events between the calls, for the per-kernel figures (four event records a step would
    # weigh on a small state's step time: 73 against 59 us for the GPT-2 block)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(K)]
    torch.cuda.synchronize()
    for k in range(K):
        evs[k][3].record(stream)
        one_step(warmup + K + k, evs[k])
    torch.cuda.synchronize()

    rep = B.pt_step_report_read(ctx, stream)
    ms_step = 1e3 * t_total / K
    pack_ms = [evs[k][3].elapsed_time(evs[k][0]) for k in range(K)]
    norm_ms = [evs[k][0].elapsed_time(evs[k][1]) for k in range(K)]
    adamw_ms = [evs[k][1].elapsed_time(evs[k][2]) for k in range(K)]
    step_ev_ms = [evs[k][3].elapsed_time(evs[k + 1][3]) for k in range(K - 1)]       # begin of a step to begin of the next
    g_bytes = 4 if A else 2
    adamw_per_elem = ADAMW_BYTES_PER_ELEM + (g_bytes - 2) + (g_bytes if zero_grads else 0)
    # accumulation: 2 B read + 4 B written for the first micro-batch, 2 + 4 read + 4 written for each further one
    fill_bytes = (6 + 10 * (A - 1)) * N if A else PACK_BYTES_PER_ELEM * N
    step_bytes = fill_bytes + adamw_per_elem * N_pad
    adamw_bytes = adamw_per_elem * N_pad
    achieved = adamw_bytes / (mean(adamw_ms) * 1e-3) / 1e9
    value = step_bytes / (ms_step * 1e-3) / 1e9
    kname = "k_adamw<%s, unroll 4, non-temporal%s%s%s>" % ("fp16" if fp16 else "bf16", ", no-decay runs" if no_decay_1d else "",
                                                          ", fp32 gradients" if A else "", ", zeroing gradients" if zero_grads else "")
    out = {
        "workload": f"{workload}: {N} elements in {C} chunks of {S}, {layout_note}; arenas spread over physical memory, all "
                    f"GPU-resident, {'fp16, loss scale 2^16' if fp16 else 'bf16'} params/grads N(0,0.02)/N(0,1e-3)"
                    f"{' with 0.1 % of the gradients x100' if outlier_every else ''}, fp32 master/m/v, AdamW lr 1e-4 betas "
                    "(0.9,0.95) eps 1e-8 wd 0.1 clip 1.0",
        "chunk_elems": S, "n_chunks": C, "elements": N, "padded_elements": N_pad, "step_bytes": step_bytes, "grad_sets": n_sets,
        "steps": K, "warmup": warmup, "value": round(value, 1), "ms_per_step": round(ms_step, 4),
        "ms_per_step_median_of_event_pairs": round(median(step_ev_ms), 4) if step_ev_ms else None,
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "kernels_ms": {("accum_grads x%d+chunk_reduce" % A if A else "pack_grads+chunk_reduce"): round(mean(pack_ms), 4),
                       "finalize": round(mean(norm_ms), 4), "adamw(+prepare)": round(mean(adamw_ms), 4)},
        "fill_GBps": round(fill_bytes / (mean(pack_ms) * 1e-3) / 1e9, 1),
        "step_report": {"norm": rep.norm, "clip_coef": rep.clip_coef, "found_inf": rep.found_inf, "step": rep.step,
                        "loss_scale": rep.loss_scale},
        "roofline": {"kernel": kname, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": MEASURED_TRAFFIC.get(workload) if layout == "dense" and not A and not zero_grads and not fp16 else None,
                     "bytes_per_launch": adamw_bytes, "avg_launch_ms": round(mean(adamw_ms), 4),
                     "median_launch_ms": round(median(adamw_ms), 4)},
    }

    if graph:
        # the same step captured once and replayed: what is left when launch overhead goes (small states)
        side = torch.cuda.Stream()

        def step_on(st_):
            if A:
                for j in range(A):
                    B.pt_chunk_accum_grads(ctx, plans[j % n_sets], r_g, j == 0, j == A - 1, st_)
            else:
                B.pt_chunk_pack_grads(ctx, plans[0], r_g, st_)
            B.pt_chunk_grad_sqnorm(ctx, None, 0, C, True, st_)
            B.pt_chunk_adamw_step(ctx, hp, 0, C, r_g, r_w, r_m, r_v, r_p, st_)
            B.pt_step_end(ctx, st_)

        with torch.cuda.stream(side):
            step_on(side)                      # pointer tables are bound outside the capture
        torch.cuda.synchronize()
        g_ = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_, stream=side):
            step_on(torch.cuda.current_stream())
        torch.cuda.synchronize()
        for _ in range(warmup):
            g_.replay()
        torch.cuda.synchronize()
        t_g = time.perf_counter()
        for _ in range(K):
            g_.replay()
        torch.cuda.synchronize()
        t_g = (time.perf_counter() - t_g) / K
        out["hip_graph"] = {"ms_per_step": round(1e3 * t_g, 4), "GBps": round(step_bytes / t_g / 1e9, 1),
                            "speedup_over_eager": round(ms_step * 1e-3 / t_g, 3)}
        del g_

    if unpack:
        # the inverse copy: updated 16-bit parameter chunks back to the model's tensors (same kernel, other direction)
        flat_p = torch.empty(N, dtype=dt16, device=dev)
        for s_ in segs:
            s_.src = flat_p.data_ptr() + 2 * offs[s_.tensor]
        plan_u = B.pt_pack_plan_create(ctx, segs)
        ts = []
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            B.pt_chunk_unpack(ctx, plan_u, r_p, stream)
            e1.record(stream)
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        B.pt_pack_plan_destroy(plan_u)
        out["unpack"] = {"ms": round(min(ts), 4), "GBps": round(4 * N / min(ts) / 1e6, 1)}
        del flat_p

    if calib:
        # (1) a plain copy kernel between two of the state's arrays: what a 1:1 read/write stream attains here
        a_, b_ = m, v
        nbytes = a_[0].numel() * 4
        n_cp = min(C, 16)
        times = []
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for c in range(n_cp):
                B.pt_calib_copy(a_[c], b_[(c + 1) % C], nbytes, stream)       # moments are rewritten by the next step anyway
            e1.record(stream)
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1))
        out["hbm_copy_GBps"] = round(2 * nbytes * n_cp / (min(times) * 1e-3) / 1e9, 1)
        # (2) the update's own access pattern (4 read + 4 write streams, same tiles and hints) without the arithmetic
        if not (A or no_decay_1d):
            times = []
            for _ in range(5):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                B.pt_calib_adamw_pattern(ctx, 0, C, stream)
                e1.record(stream)
                torch.cuda.synchronize()
                times.append(e0.elapsed_time(e1))
            pat = ADAMW_BYTES_PER_ELEM * N_pad / (median(times) * 1e-3) / 1e9
            out["roofline"]["pattern_ceiling_GBps"] = round(pat, 1)
            out["roofline"]["pattern_ceiling_ms"] = round(median(times), 4)
            out["roofline"]["kernel_over_pattern_ceiling"] = round(achieved / pat, 4)
        out["roofline"]["hbm_copy_GBps"] = out["hbm_copy_GBps"]

    for p_ in plans:
        B.pt_pack_plan_destroy(p_)
    B.pt_ctx_destroy(ctx)
    del g16, p16, w, m, v, grad_set_mem, grad_sets_, g_hi, r_g, r_w, r_m, r_v, r_p
    release()

    if cpu_in is not None:
        out.update(cpu_oracle_legs(cpu_in, S, cpu_sample_chunks, cpu_one_thread_chunks))
    return out


def cpu_oracle_legs(cpu_in, S, n_threads_chunks, n_one_thread_chunks):
    """The oracle as it stands, timed on the host cores over the first chunks of the same state: its step
    (non-finite scan + fp64 norm + clip + the fp32-sequence AdamW) with all hardware threads, pack timed on
    its own, and optionally the same step with ONE thread."""
    import numpy as np

    import oracle as O
    hp_o = O.Hparams(**HP)
    out = {}

    def leg(n_chunks, threads, reps):
        n_el = n_chunks * S
        t_pack = time.perf_counter()
        chunks = O.pack_dense([cpu_in["src"][:n_el]], S, n_chunks=n_chunks).reshape(-1)
        t_pack = time.perf_counter() - t_pack
        ow, op = cpu_in["w"][:n_el].copy(), cpu_in["p"][:n_el].copy()
        om, ov = np.zeros(n_el, np.float32), np.zeros(n_el, np.float32)
        ost = O.new_state(None)
        t = time.perf_counter()
        for _ in range(reps):
            O.step(hp_o, None, ost, chunks, ow, om, ov, op, S, O.BF16, use_f32seq=True, threads=threads)
        t = (time.perf_counter() - t) / reps
        return n_el, t, t_pack

    if n_threads_chunks:
        threads = O.hardware_threads()
        n_el, t, t_pack = leg(n_threads_chunks, threads, 2)
        out["cpu_baseline"] = {
            "value": round(ADAMW_BYTES_PER_ELEM * n_el / t / 1e9, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"first {n_threads_chunks} chunks ({n_el} elements) of the same state, 2 steps: the oracle's step = "
                      f"non-finite scan (one thread) + fp64 norm + clip + AdamW in its fp32 operation sequence, "
                      f"{t * 1e3:.1f} ms/step on {threads} threads, counted as 28 B/element like the GPU's update; pack is "
                      f"timed on its own (one thread): {t_pack * 1e3:.1f} ms = {PACK_BYTES_PER_ELEM * n_el / t_pack / 1e9:.2f} GB/s",
            "ms_per_step_sample": round(t * 1e3, 2), "pack_ms_sample": round(t_pack * 1e3, 2),
            "pack_GBps": round(PACK_BYTES_PER_ELEM * n_el / t_pack / 1e9, 3)}
    if n_one_thread_chunks:
        n_el, t, _ = leg(n_one_thread_chunks, 1, 1)
        out["cpu_one_thread"] = {"value": round(ADAMW_BYTES_PER_ELEM * n_el / t / 1e9, 3), "unit": "GB/s", "cores": 1,
                                 "kind": "oracle", "ms_per_step_sample": round(t * 1e3, 2),
                                 "sample": f"first {n_one_thread_chunks} chunks ({n_el} elements), 1 step, one thread"}
    return out


# ---------------------------------------------------------------- half of the chunks in pinned host memory

def run_split(steps, warmup, slots=3, host_chunks=0, host_update=False, host_threads=0, model=False):
    """LLaMA-13B-shaped state: chunks [0, C/2) resident in HBM, chunks [C/2, C/2 + n_host) in pinned host memory
    (as many of the configuration's 97 as the box lets the process pin).  Timed step = pack (resident) -> finalize ->
    pt_chunk_stream_step (host chunks, side streams) -> pt_chunk_adamw_step (resident, overlapped) -> pt_step_end
    (join).  The host chunks' gradients were packed and reduced on the GPU and offloaded in the untimed set-up."""
    import numpy as np
    import torch

    from paper_2406_08334_amd import binding as B
    from paper_2406_08334_amd import shapes, synth
    from paper_2406_08334_amd.arena import spread_arenas

    dev = "cuda:0"
    table, S = shapes.workload("llama_13b")
    sizes = [n for _, n in table]
    N = sum(sizes)
    segs, C = B.pt_layout_dense(sizes, S)
    n_persist = C // 2
    n_want = C - n_persist if host_chunks <= 0 else min(host_chunks, C - n_persist)
    n_host = n_want
    log(f"[bench] llama_13b: {C} chunks of {S:,}; {n_persist} resident ({16 * n_persist * S / 1e9:.1f} GB HBM), "
        f"{n_host} wanted in pinned host memory ({16 * n_host * S / 1e9:.1f} GB; host RAM {host_memory_gb()} GB), "
        f"{slots} chunk buffers")
    t0 = time.time()
    ctx = B.pt_ctx_create(B.PT_BF16, S, C, None)
    B.pt_stream_reserve(ctx, slots)
    stream_status = B.pt_stream_status(ctx)
    log(f"[bench] copy streams: {stream_status}")
    n_res = n_persist * S
    g16, p16, w, m, v = spread_arenas(
        [((n_persist, S), torch.bfloat16), ((n_persist, S), torch.bfloat16), ((n_persist, S), torch.float32),
         ((n_persist, S), torch.float32), ((n_persist, S), torch.float32)], device=dev, keep_free_bytes=2 * n_res + 16 * S)
    synth.normal_16(synth.SEED_PARAMS, 0, 0, 0, n_res, 0.02, torch.bfloat16, dev, out=p16.view(-1))
    for c in range(n_persist):
        w[c].copy_(p16[c])
    grad_src = torch.empty(n_res, dtype=torch.bfloat16, device=dev)
    synth.normal_16(synth.SEED_GRADS, 1, 0, 0, n_res, 1e-3, torch.bfloat16, dev, out=grad_src)
    offs = np.cumsum([0] + sizes[:-1]).tolist()
    res_segs = [s for s in segs if s.chunk < n_persist]
    for s in res_segs:
        s.src = grad_src.data_ptr() + 2 * offs[s.tensor]
    plan = B.pt_pack_plan_create(ctx, res_segs)
    # host chunks: generated on the GPU, reduced there, then offloaded (untimed)
    pin = lambda dt: torch.empty(S, dtype=dt).pin_memory()
    h_g, h_p, h_w, h_m, h_v = [], [], [], [], []
    tmp16 = torch.empty(S, dtype=torch.bfloat16, device=dev)
    tmp32 = torch.empty(S, dtype=torch.float32, device=dev)
    pin_limit_gb = None
    for i in range(n_want):
        c = n_persist + i
        real = max(0, min(S, N - c * S))
        try:
            bufs = [pin(torch.bfloat16), pin(torch.bfloat16), pin(torch.float32), pin(torch.float32), pin(torch.float32)]
        except RuntimeError as e:       # the box pins only so much host memory: run with what fits
            if "out of memory" not in str(e):
                raise
            n_host = max(0, i - 2)      # two chunks of headroom for the runtime's own pinned allocations
            bufs = None
            for lst in (h_g, h_p, h_w, h_m, h_v):
                del lst[n_host:]
            gc.collect()
            torch._C._host_emptyCache()  # hands them back to the driver (a freed pinned tensor stays in torch's cache)
            pin_limit_gb = round(16 * i * S / 1e9, 1)
            log(f"[bench] pinned host memory exhausted after {i} chunks ({pin_limit_gb} GB of {host_memory_gb()} GB RAM): "
                f"streaming {n_host} host chunks instead of {n_want}")
            break
        tmp16.zero_()
        if real:
            synth.normal_16(synth.SEED_GRADS, 1, 0, c * S, real, 1e-3, torch.bfloat16, dev, out=tmp16[:real])
        ptrs = [None] * C
        ptrs[c] = tmp16
        B.pt_chunk_grad_sqnorm(ctx, ptrs, c, 1, False)
        h_g.append(bufs[0]); h_g[-1].copy_(tmp16)
        tmp16.zero_()
        if real:
            synth.normal_16(synth.SEED_PARAMS, 0, 0, c * S, real, 0.02, torch.bfloat16, dev, out=tmp16[:real])
        h_p.append(bufs[1]); h_p[-1].copy_(tmp16)
        tmp32.copy_(tmp16)
        h_w.append(bufs[2]); h_w[-1].copy_(tmp32)
        h_m.append(bufs[3]); h_m[-1].zero_()
        h_v.append(bufs[4]); h_v[-1].zero_()
        if i % 16 == 0:
            log(f"[bench] host chunk {i}/{n_want} ready ({time.time() - t0:.0f} s)")
    assert n_host >= 2, "could not pin even two host chunks"
    torch.cuda.synchronize()
    log(f"[bench] state generated in {time.time() - t0:.1f} s")

    # ---- bare link rate with the same pinned buffers: one direction at a time, then both at once
    stream = torch.cuda.current_stream()
    s_a, s_b = torch.cuda.Stream(), torch.cuda.Stream()
    dst_up, src_dn = torch.empty(S, dtype=torch.float32, device=dev), torch.empty(S, dtype=torch.float32, device=dev)
    n_cal = min(8, n_host)

    def link(up, down):
        torch.cuda.synchronize()
        t = time.perf_counter()
        for i in range(n_cal):
            if up:
                with torch.cuda.stream(s_a):
                    dst_up.copy_(h_w[i], non_blocking=True)
            if down:
                with torch.cuda.stream(s_b):
                    h_v[i].copy_(src_dn, non_blocking=True)
        torch.cuda.synchronize()
        return 4 * S * n_cal / (time.perf_counter() - t) / 1e9
    src_dn.zero_()
    link(True, True)
    bare = {"h2d_alone": round(link(True, False), 2), "d2h_alone": round(link(False, True), 2),
            "each_direction_when_both": round(link(True, True), 2)}
    log(f"[bench] bare pinned copies, GB/s: {bare}")

    hp = B.hparams(**HP)
    rows = lambda a: [a[c] for c in range(n_persist)]
    r_g, r_w, r_m, r_v, r_p = rows(g16), rows(w), rows(m), rows(v), rows(p16)
    pack_rows = r_g + [None] * (C - n_persist)
    host_threads = host_threads if host_threads > 0 else (os.cpu_count() or 1)
    CARRY = B.PT_FINALIZE_CARRY       # the host chunks' sums of squares were taken once, before they were offloaded

    def one_step(streamed=True, resident=True, on_host=False):
        B.pt_chunk_pack_grads(ctx, plan, pack_rows, stream)
        B.pt_chunk_grad_sqnorm(ctx, None, 0, C, CARRY, stream)
        if streamed and not on_host:
            B.pt_chunk_stream_step(ctx, hp, n_persist, n_host, h_g, h_w, h_m, h_v, h_p, stream)
        if resident:
            B.pt_chunk_adamw_step(ctx, hp, 0, n_persist, r_g, r_w, r_m, r_v, r_p, stream)
        if streamed and on_host:        # the paper's placement: host threads, while the GPU kernel runs
            B.pt_chunk_host_adamw_step(ctx, hp, n_persist, n_host, h_g, h_w, h_m, h_v, h_p, host_threads, stream)
        B.pt_step_end(ctx, stream)

    def timed(k, **kw):
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(k):
            one_step(**kw)
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / k

    for _ in range(warmup):
        one_step()
    K = steps
    t_step = timed(K)
    t_res = timed(max(K, 3), streamed=False)
    t_str = timed(max(1, K - 1), resident=False)
    host_upd = None
    if host_update:
        one_step(on_host=True)          # starts the worker threads
        t_h = timed(K, on_host=True)
        t_h_only = timed(max(1, K - 1), on_host=True, resident=False)
        # what still has to cross the link in that variant: 16-bit parameters up (gradients came down during backward)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for i in range(n_host):
            tmp16.copy_(h_p[i], non_blocking=True)
        torch.cuda.synchronize()
        t_up = time.perf_counter() - t
        host_upd = {"threads": host_threads, "ms_per_step": round(1e3 * t_h, 2),
                    "ms_host_chunks_only": round(1e3 * t_h_only, 2),
                    "host_elements_per_s": round(n_host * S / t_h_only / 1e9, 3),
                    "host_GBps_at_28B_per_element": round(28 * n_host * S / t_h_only / 1e9, 1),
                    "overlap_ratio_step_over_max": round(t_h / max(t_h_only, t_res), 4),
                    "ms_param16_upload_afterwards": round(1e3 * t_up, 2),
                    "speedup_over_streaming_through_the_gpu": round(t_step / t_h, 3)}
    model_out = None
    if model:
        model_out = fit_optim_model(B, np, torch, ctx, hp, stream, S, C, n_persist, n_host, plan, res_segs, pack_rows,
                                    (r_g, r_w, r_m, r_v, r_p), (h_g, h_w, h_m, h_v, h_p), host_threads, slots)
    rep = B.pt_step_report_read(ctx, stream)
    link_bytes = 14 * S * n_host
    per_dir = link_bytes / t_step / 1e9
    one_dir = min(bare["h2d_alone"], bare["d2h_alone"])
    out = {
        "workload": f"llama_13b: {C} chunks of {S}; chunks [0,{n_persist}) resident, [{n_persist},{n_persist + n_host}) in pinned "
                    f"host memory ({n_host} of the configuration's {C - n_persist}: the box pins at most "
                    f"{pin_limit_gb if pin_limit_gb else '>= ' + str(round(16 * n_host * S / 1e9, 1))} GB of its {host_memory_gb()} GB RAM), "
                    f"{slots} chunk buffers",
        "n_persist": n_persist, "n_host": n_host, "n_host_wanted": n_want, "slots": slots,
        "link_bytes_per_direction": link_bytes, "steps": K, "warmup": warmup,
        "link_GBps_per_direction": round(per_dir, 2), "ms_per_step": round(1e3 * t_step, 2),
        "bare_link_GBps": bare,
        "link_utilisation_vs_one_direction_rate": round(per_dir / one_dir, 4),
        "link_utilisation_vs_bare_both_directions": round(per_dir / bare["each_direction_when_both"], 4),
        "ms_resident_only": round(1e3 * t_res, 2), "ms_streamed_only": round(1e3 * t_str, 2),
        "copy_streams_self_test": stream_status,
        "overlap_ratio_step_over_max": round(t_step / max(t_res, t_str), 4),
        "resident_GBps": round((PACK_BYTES_PER_ELEM + ADAMW_BYTES_PER_ELEM) * n_res / t_res / 1e9, 1),
        "step_report": {"norm": rep.norm, "found_inf": rep.found_inf, "step": rep.step},
    }
    if host_upd:
        out["host_side_update"] = host_upd
    if model_out:
        out["optim_model"] = model_out
    B.pt_pack_plan_destroy(plan)
    B.pt_ctx_destroy(ctx)
    del g16, p16, w, m, v, grad_src, h_g, h_p, h_w, h_m, h_v, tmp16, tmp32, dst_up, src_dn, r_g, r_w, r_m, r_v, r_p, pack_rows
    release()
    return out


def fit_optim_model(B, np, torch, ctx, hp, stream, S, C, n_persist, n_host, plan, res_segs, pack_rows, res, hst, host_threads, slots):
    """OPTIM-phase cost model: fit linear times on a few sizes, validate on held-out splits, ask the chooser."""
    r_g, r_w, r_m, r_v, r_p = res
    h_g, h_w, h_m, h_v, h_p = hst
    plans_by_n = {n_persist: plan}

    def plan_for(n):
        if n not in plans_by_n:
            plans_by_n[n] = B.pt_pack_plan_create(ctx, [s_ for s_ in res_segs if s_.chunk < n])
        return plans_by_n[n]

    def run(n_res, n_h, mode, k=3, update=True):
        pl = plan_for(n_res) if n_res else None

        def once():
            if pl is not None:
                B.pt_chunk_pack_grads(ctx, pl, pack_rows, stream)
            B.pt_chunk_grad_sqnorm(ctx, None, 0, C, B.PT_FINALIZE_CARRY, stream)
            if n_h and mode == B.PT_OPTIM_STREAM:
                B.pt_chunk_stream_step(ctx, hp, n_persist, n_h, h_g[:n_h], h_w[:n_h], h_m[:n_h], h_v[:n_h], h_p[:n_h], stream)
            if n_res and update:
                B.pt_chunk_adamw_step(ctx, hp, 0, n_res, r_g[:n_res], r_w[:n_res], r_m[:n_res], r_v[:n_res], r_p[:n_res], stream)
            if not update:
                B.pt_step_report_read(ctx, stream)      # a step that ends at the norm: the scalar kernel runs here
            if n_h and mode == B.PT_OPTIM_HOST:
                B.pt_chunk_host_adamw_step(ctx, hp, n_persist, n_h, h_g[:n_h], h_w[:n_h], h_m[:n_h], h_v[:n_h], h_p[:n_h],
                                           host_threads, stream)
            B.pt_step_end(ctx, stream)
        once()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(k):
            once()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / k

    def fit(points):                 # least squares t = a + b * elems
        xs = np.array([p_[0] for p_ in points], dtype=np.float64)
        ys = np.array([p_[1] for p_ in points], dtype=np.float64)
        b_, a_ = np.polyfit(xs, ys, 1)
        return float(a_), float(b_)

    hs = sorted({max(2, n_host // 8), max(3, n_host // 3), n_host})
    gs = sorted({n_persist // 4, n_persist // 2, n_persist})
    g_fix, g_per = fit([(n * S, run(n, 0, B.PT_OPTIM_HOST)) for n in gs])
    l_fix, l_per = fit([(n * S, run(0, n, B.PT_OPTIM_STREAM, k=2)) for n in hs])
    h_fix, h_per = fit([(n * S, run(0, n, B.PT_OPTIM_HOST)) for n in hs])
    tg_, tl_ = g_fix + g_per * n_persist * S, l_fix + l_per * hs[1] * S
    # the resident work that comes before the norm is final (pack + reduction): the same step without its update
    share = min(1.0, run(n_persist, 0, B.PT_OPTIM_HOST, update=False) / tg_)
    t_mix = run(n_persist, hs[1], B.PT_OPTIM_STREAM, k=2)
    beside_ = (1.0 - share) * tg_
    cont = max(0.0, (t_mix - share * tg_ - max(beside_, tl_)) / min(beside_, tl_))
    rates = B.pt_optim_rates(g_fix, g_per, l_fix, l_per, h_fix, h_per, cont, share)
    held_out = [(n_persist // 2, n_host // 2, B.PT_OPTIM_STREAM), (n_persist, n_host, B.PT_OPTIM_STREAM),
                (3 * n_persist // 4, n_host // 4, B.PT_OPTIM_STREAM),
                (n_persist, n_host, B.PT_OPTIM_HOST), (n_persist // 2, n_host // 2, B.PT_OPTIM_HOST),
                (n_persist // 4, n_host, B.PT_OPTIM_HOST), (n_persist, max(2, n_host // 10), B.PT_OPTIM_HOST)]
    rows_ = []
    for n_res, n_h, mode in held_out:
        meas = run(n_res, n_h, mode, k=2)
        pred = B.pt_optim_predict(rates, S, n_res + n_h, n_res, mode)[2]
        rows_.append({"n_persist": n_res, "n_other": n_h, "mode": "stream" if mode == B.PT_OPTIM_STREAM else "host",
                      "measured_ms": round(1e3 * meas, 2), "predicted_ms": round(1e3 * pred, 2),
                      "error_pct": round(100.0 * (pred - meas) / meas, 2)})
        log(f"[model] {rows_[-1]}")
    total = n_persist + n_host
    choices = {}
    for gb in (40, 80, 120, 200):
        for mode, name in ((B.PT_OPTIM_STREAM, "stream"), (B.PT_OPTIM_HOST, "host")):
            try:
                ch = B.pt_optim_choose(rates, S, total, gb * 10**9, mode, slots)
                choices[f"{gb}GB_{name}"] = {"n_persist": ch.n_persist, "n_slots": ch.n_slots,
                                              "predicted_ms": round(1e3 * ch.t_step, 2), "hbm_GB": round(ch.hbm_bytes / 1e9, 1)}
            except B.PtError:
                choices[f"{gb}GB_{name}"] = None
    for n, pl in plans_by_n.items():
        if n != n_persist:
            B.pt_pack_plan_destroy(pl)
    return {"rates": {"gpu_s_fixed": g_fix, "gpu_s_per_elem": g_per, "link_s_fixed": l_fix, "link_s_per_elem": l_per,
                      "host_s_fixed": h_fix, "host_s_per_elem": h_per, "stream_contention": round(cont, 3),
                      "gpu_serial_share": round(share, 4)},
            "fit_sizes_chunks": {"gpu": gs, "other": hs}, "held_out": rows_,
            "max_abs_error_pct": max(abs(r_["error_pct"]) for r_ in rows_),
            "chooser_for_%d_chunks" % total: choices}


# ------------------------------------------------------------------------------------------------- main

def brief(d):
    """the figures of a configuration that go under other_configs"""
    keep = ("workload", "steps", "warmup", "ms_per_step", "ms_per_step_median_of_event_pairs", "value", "pct_of_hbm_peak",
            "kernels_ms", "fill_GBps", "step_report", "hip_graph", "hbm_copy_GBps", "cpu_one_thread")
    out = {k: d[k] for k in keep if k in d}
    out["GBps"] = out.pop("value")
    r = d["roofline"]
    out["adamw"] = {k: r[k] for k in ("achieved", "frac", "avg_launch_ms", "bytes_per_launch", "pattern_ceiling_GBps",
                                      "kernel_over_pattern_ceiling") if k in r}
    return out


OTHER_CONFIGS = ("gpt2_block_768", "gpt2_xl_outliers", "llama_7b_fp16_loss_scaling", "llama_13b_half_in_pinned_host_memory")


def run_other_config(name, with_cpu):
    """One of the benchmark's other configurations, in this (fresh) process; returns its figures."""
    if name == "gpt2_block_768":
        d = brief(run_resident("gpt2_block_768", 300, 30, graph=True, calib=False))
        d["note"] = ("0.13 GB of state: lives in the 256 MB Infinity Cache and is launch-bound; effective GB/s, "
                     "not an HBM figure")
        return d
    if name == "gpt2_xl_outliers":
        return brief(run_resident("gpt2_xl", 20, 5, calib=True, cpu_one_thread_chunks=3 if with_cpu else 0))
    if name == "llama_7b_fp16_loss_scaling":
        return brief(run_resident("llama_7b", 10, 3, fp16=True, calib=True))
    if name == "llama_13b_half_in_pinned_host_memory":
        return run_split(2, 1, slots=3, host_update=True, model=True)
    raise ValueError(name)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama_7b", help="llama_7b | gpt2_xl | gpt2_block_768")
    ap.add_argument("--headline-only", action="store_true", help="skip the other benchmark configurations")
    ap.add_argument("--grad-sets", type=int, default=3, help="distinct pre-generated gradient sets, rotated")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-chunks", type=int, default=24)
    ap.add_argument("--no-calib", action="store_true", help="skip the plain-copy and access-pattern calibrations")
    ap.add_argument("--layout", default="dense", choices=["dense", "grouped"],
                    help="dense: the benchmark configurations' layout; grouped: the paper's no-split, block-per-chunk layout")
    ap.add_argument("--no-decay-1d", action="store_true",
                    help="keep biases and normalisation gains out of the weight decay (masked update kernel)")
    ap.add_argument("--grad-accum", type=int, default=0, metavar="K",
                    help="variant: K micro-batches accumulated into fp32 gradient chunks per step (0 = the 16-bit pack path)")
    ap.add_argument("--graph", action="store_true",
                    help="also time the whole step replayed from a HIP graph (one gradient set); reported beside the eager figure")
    ap.add_argument("--unpack", action="store_true", help="also time pt_chunk_unpack of the parameter chunks into tensors")
    ap.add_argument("--fp16", action="store_true",
                    help="fp16 parameters and gradients with dynamic loss scaling (scale 2^16; gradients drawn scaled)")
    ap.add_argument("--zero-grads", action="store_true", help="variant: the update zeroes the gradient chunks it has read")
    ap.add_argument("--stream", action="store_true",
                    help="the split configuration alone: LLaMA-13B shape, first half of the chunks resident, the rest in "
                         "pinned host memory through pt_chunk_stream_step")
    ap.add_argument("--host-chunks", type=int, default=0, help="--stream: host-resident chunks (default: all of the second half)")
    ap.add_argument("--slots", type=int, default=3, help="--stream: device chunk buffers")
    ap.add_argument("--host-update", action="store_true",
                    help="--stream: also time the paper's placement, host chunks updated by host threads")
    ap.add_argument("--model", action="store_true",
                    help="--stream: fit the OPTIM-phase cost model on this box and validate it on held-out splits")
    ap.add_argument("--host-threads", type=int, default=0, help="--host-update: threads (default: all cores)")
    ap.add_argument("--one-config", default="", choices=[""] + list(OTHER_CONFIGS), help=argparse.SUPPRESS)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "run it with --gpus 1.", file=sys.stderr)
        return 2

    import torch

    from paper_2406_08334_amd import binding as B
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    B.lib()

    if args.one_config:
        print(json.dumps(run_other_config(args.one_config, not args.no_cpu_baseline)), flush=True)
        return 0

    if args.stream:
        d = run_split(args.steps if args.steps != 20 else 3, min(args.warmup, 1), slots=args.slots,
                      host_chunks=args.host_chunks, host_update=args.host_update, host_threads=args.host_threads, model=args.model)
        out = {"metric": "streamed chunked AdamW step: host-link GB/s per direction (both directions busy) + ms/step",
               "value": d["link_GBps_per_direction"], "unit": "GB/s per direction", "n_gpus": 1, "steps": d["steps"],
               "warmup": d["warmup"], "ms_per_step": d["ms_per_step"], "higher_is_better": True, "scaling": "weak",
               "vs_baseline": None, "dtype": "f32", "data": "synthetic", "config": {"workload": d.pop("workload")}}
        out.update({k: v for k, v in d.items() if k not in ("steps", "warmup", "ms_per_step")})
        print(json.dumps(out), flush=True)
        return 0

    variant = args.layout != "dense" or args.no_decay_1d or args.grad_accum or args.zero_grads or args.fp16
    headline = args.workload == "llama_7b" and not variant
    n_cpu = 0 if (args.no_cpu_baseline or variant) else args.cpu_sample_chunks
    d = run_resident(args.workload, args.steps, args.warmup, fp16=args.fp16, grad_sets=args.grad_sets, layout=args.layout,
                     no_decay_1d=args.no_decay_1d, grad_accum=args.grad_accum, zero_grads=args.zero_grads, graph=args.graph,
                     unpack=args.unpack, calib=not args.no_calib, cpu_sample_chunks=n_cpu)
    out = {
        "metric": METRIC, "value": d["value"], "unit": "GB/s", "n_gpus": 1, "steps": d["steps"], "warmup": d["warmup"],
        "ms_per_step": d["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": d["workload"], "chunk_elems": d["chunk_elems"], "n_chunks": d["n_chunks"], "elements": d["elements"],
                   "padded_elements": d["padded_elements"], "step_bytes": d["step_bytes"], "grad_sets": d["grad_sets"]},
    }
    for k in ("ms_per_step_median_of_event_pairs", "pct_of_hbm_peak", "kernels_ms", "fill_GBps", "step_report", "roofline",
              "hbm_copy_GBps", "hip_graph", "unpack", "cpu_baseline"):
        if k in d:
            out[k] = d[k]

    if headline and not args.headline_only:
        # The other benchmark configurations, each bounded to a few seconds of timed work and each in a fresh
        # process of its own, one after the other: what a configuration measures must not depend on what ran
        # before it in this process (the physical placement of its arenas, and which hardware queues its side
        # streams get - the streamed step moved 28 instead of 48 GB/s per direction when it ran fourth in one
        # process).  This process has released its device memory and only waits meanwhile.
        release()
        others = {}
        t_o = time.time()
        for name in OTHER_CONFIGS:
            extra = ["--no-cpu-baseline"] if args.no_cpu_baseline else []
            try:
                res = subprocess.run([sys.executable, os.path.abspath(__file__), "--one-config", name] + extra,
                                     stdout=subprocess.PIPE, text=True, timeout=420)
            except subprocess.TimeoutExpired:
                others[name] = {"error": "child process did not finish within 420 s and was stopped"}
                log(f"[bench] configuration {name} did not finish within 420 s")
                continue
            lines = [l for l in res.stdout.splitlines() if l.startswith("{")]
            if res.returncode != 0 or not lines:
                others[name] = {"error": f"child process exited with code {res.returncode}"}
                log(f"[bench] configuration {name} failed (exit code {res.returncode})")
                continue
            others[name] = json.loads(lines[-1])
        out["other_configs"] = others
        log(f"[bench] other configurations measured in {time.time() - t_o:.1f} s")
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
