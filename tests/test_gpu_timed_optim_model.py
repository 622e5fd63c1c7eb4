"""The OPTIM-phase cost model on the GPU machine: fitted from three small sizes per part, it must predict
held-out splits - one streamed through the chunk buffers, one updated by host threads - within 10 %
(the paper's estimator stays under 10 % over its models; Appendix A.1, Eq. 2 restricted to the
optimizer phase), and the chooser must respect the memory budget and return the best feasible split
under the model."""
import time

import numpy as np
import pytest
import torch

from paper_2406_08334_amd import binding as B
from paper_2406_08334_amd import synth
from gpu_harness import hp_pair

pytestmark = pytest.mark.gpu

S = 1 << 22
N_RES, N_HOST = 48, 12
THREADS = 8


@pytest.fixture(scope="module")
def rig():
    dev = "cuda"
    C = N_RES + N_HOST
    ctx = B.pt_ctx_create(B.PT_BF16, S, C, None)
    B.pt_stream_reserve(ctx, 3)
    g16 = torch.zeros(N_RES, S, dtype=torch.bfloat16, device=dev)
    p16 = torch.zeros(N_RES, S, dtype=torch.bfloat16, device=dev)
    synth.normal_16(synth.SEED_PARAMS, 0, 0, 0, N_RES * S, 0.02, torch.bfloat16, dev, out=p16.view(-1))
    w = p16.float()
    m, v = torch.zeros_like(w), torch.zeros_like(w)
    src = torch.empty(N_RES * S, dtype=torch.bfloat16, device=dev)
    synth.normal_16(synth.SEED_GRADS, 1, 0, 0, N_RES * S, 1e-3, torch.bfloat16, dev, out=src)
    host = {k: [torch.zeros(S, dtype=dt, pin_memory=True) for _ in range(N_HOST)]
            for k, dt in (("g", torch.bfloat16), ("p", torch.bfloat16), ("w", torch.float32), ("m", torch.float32),
                          ("v", torch.float32))}
    tmp = torch.empty(S, dtype=torch.bfloat16, device=dev)
    for i in range(N_HOST):
        synth.normal_16(synth.SEED_GRADS, 1, 0, (N_RES + i) * S, S, 1e-3, torch.bfloat16, dev, out=tmp)
        ptrs = [None] * C
        ptrs[N_RES + i] = tmp
        B.pt_chunk_grad_sqnorm(ctx, ptrs, N_RES + i, 1, False)          # reduced on the GPU before the offload
        host["g"][i].copy_(tmp)
        synth.normal_16(synth.SEED_PARAMS, 0, 0, (N_RES + i) * S, S, 0.02, torch.bfloat16, dev, out=tmp)
        host["p"][i].copy_(tmp)
        host["w"][i].copy_(tmp.float())
    torch.cuda.synchronize()
    plans = {}

    def plan_for(n):
        if n not in plans:
            plans[n] = B.pt_pack_plan_create(ctx, [B.pt_segment(src.data_ptr(), c * S, S, 0, c, c) for c in range(n)])
        return plans[n]

    hp_b, _, _ = hp_pair()
    rows = lambda a, n: [a[c] for c in range(n)]
    stream = torch.cuda.current_stream()

    def step(n_res, n_h, mode, update=True):
        if n_res:
            B.pt_chunk_pack_grads(ctx, plan_for(n_res), rows(g16, n_res) + [None] * (C - n_res), stream)
        B.pt_chunk_grad_sqnorm(ctx, None, 0, C, B.PT_FINALIZE_CARRY, stream)
        if n_h and mode == B.PT_OPTIM_STREAM:
            B.pt_chunk_stream_step(ctx, hp_b, N_RES, n_h, host["g"][:n_h], host["w"][:n_h], host["m"][:n_h],
                                   host["v"][:n_h], host["p"][:n_h], stream)
        if n_res and update:
            B.pt_chunk_adamw_step(ctx, hp_b, 0, n_res, rows(g16, n_res), rows(w, n_res), rows(m, n_res), rows(v, n_res),
                                  rows(p16, n_res), stream)
        if n_h and mode == B.PT_OPTIM_HOST:
            B.pt_chunk_host_adamw_step(ctx, hp_b, N_RES, n_h, host["g"][:n_h], host["w"][:n_h], host["m"][:n_h],
                                       host["v"][:n_h], host["p"][:n_h], THREADS, stream)
        B.pt_step_end(ctx, stream)

    def measure(n_res, n_h, mode, reps=7, update=True):
        """least of `reps` timed steps: the box is a virtual machine whose host threads are now and then late,
        and the least time is what the model is about"""
        step(n_res, n_h, mode, update)
        best = float("inf")
        for _ in range(reps):
            torch.cuda.synchronize()
            t = time.perf_counter()
            step(n_res, n_h, mode, update)
            B.pt_step_report_read(ctx, stream)       # the scalars are read back in either case (pack-only steps end here)
            torch.cuda.synchronize()
            best = min(best, time.perf_counter() - t)
        return best

    yield measure
    torch.cuda.synchronize()
    for pl in plans.values():
        B.pt_pack_plan_destroy(pl)
    B.pt_ctx_destroy(ctx)


def fit(points):
    xs = np.array([p[0] for p in points], dtype=np.float64)
    ys = np.array([p[1] for p in points], dtype=np.float64)
    slope, icept = np.polyfit(xs, ys, 1)
    return float(icept), float(slope)


def fit_and_validate(measure):
    """one fit and its held-out errors: (rates, [(name, measured, predicted, relative error)])"""
    g_fix, g_per = fit([(n * S, measure(n, 0, B.PT_OPTIM_HOST, reps=15)) for n in (12, 24, 48)])
    l_fix, l_per = fit([(n * S, measure(0, n, B.PT_OPTIM_STREAM, reps=4)) for n in (3, 6, 12)])
    h_fix, h_per = fit([(n * S, measure(0, n, B.PT_OPTIM_HOST, reps=15)) for n in (3, 6, 12)])
    # the share of the resident part that comes before the norm (pack + reduction): the same step without its update
    share = min(1.0, measure(48, 0, B.PT_OPTIM_HOST, reps=15, update=False) / (g_fix + g_per * 48 * S))
    # the share of the shorter part a streamed step pays on top of the longer one, from one mixed run
    tg, tl = g_fix + g_per * 48 * S, l_fix + l_per * 6 * S
    t_mix = measure(48, 6, B.PT_OPTIM_STREAM, reps=4)
    beside = (1.0 - share) * tg
    cont = min(1.0, max(0.0, (t_mix - share * tg - max(beside, tl)) / min(beside, tl)))
    rates = B.pt_optim_rates(g_fix, g_per, l_fix, l_per, h_fix, h_per, cont, share)
    print(f"[optim-model] resident {g_per * 1e12:.2f} ps/element + {g_fix * 1e3:.3f} ms, {100 * share:.1f} % of it before the norm; "
          f"streamed {l_per * 1e12:.1f} ps/element + "
          f"{l_fix * 1e3:.3f} ms; host ({THREADS} threads) {h_per * 1e12:.1f} ps/element + {h_fix * 1e3:.3f} ms; "
          f"contention {cont:.2f}", flush=True)
    assert 0.0 < share < 0.6
    assert g_per > 0 and l_per > 0 and h_per > 0
    rows = []
    for n_res, n_h, mode, name in ((36, 9, B.PT_OPTIM_STREAM, "streamed"), (36, 9, B.PT_OPTIM_HOST, "host")):
        meas = measure(n_res, n_h, mode, reps=5 if mode == B.PT_OPTIM_STREAM else 15)
        pred = B.pt_optim_predict(rates, S, n_res + n_h, n_res, mode)[2]
        err = (pred - meas) / meas
        print(f"[optim-model] held out {name}: {n_res} resident + {n_h} other: measured {meas * 1e3:.3f} ms, "
              f"predicted {pred * 1e3:.3f} ms ({100 * err:+.1f} %)", flush=True)
        rows.append((name, meas, pred, err))
    return rates, rows


def test_fitted_model_predicts_held_out_splits_and_the_chooser_obeys_the_budget(rig):
    measure = rig
    # Wall-clock figures of a few milliseconds on a shared virtual machine: if a fit misses the bar, ONE more fit is
    # taken before the test fails (a model that is wrong misses twice; a late host thread does not).
    rates, rows = fit_and_validate(measure)
    if any(abs(err) > 0.10 for _, _, _, err in rows):
        print("[optim-model] a held-out split missed 10 %: fitting once more", flush=True)
        rates, rows = fit_and_validate(measure)
    for name, meas, pred, err in rows:
        assert abs(err) <= 0.10, (name, meas, pred)
    # chooser: inside the budget, and the best feasible split under the model (brute force over n_persist)
    C = 60
    for budget_chunks, mode, slots in ((20, B.PT_OPTIM_STREAM, 3), (60, B.PT_OPTIM_STREAM, 2), (33, B.PT_OPTIM_HOST, 0),
                                       (100, B.PT_OPTIM_HOST, 0)):
        budget = 16 * S * budget_chunks
        ch = B.pt_optim_choose(rates, S, C, budget, mode, slots if slots else 3)
        assert ch.hbm_bytes <= budget and ch.hbm_bytes == 16 * S * (ch.n_persist + ch.n_slots)
        best = None
        for n in range(C + 1):
            buf = slots if (mode == B.PT_OPTIM_STREAM and n < C) else 0
            if 16 * S * (n + buf) > budget:
                continue
            t = B.pt_optim_predict(rates, S, C, n, mode)[2]
            if best is None or t < best[0]:
                best = (t, n)
        assert ch.n_persist == best[1] and abs(ch.t_step - best[0]) <= 1e-15
    with pytest.raises(B.PtError):
        B.pt_optim_choose(rates, S, C, 16 * S * 2, B.PT_OPTIM_STREAM, 3)      # not even the chunk buffers fit
