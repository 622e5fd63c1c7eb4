"""GPU parity on inputs the layouts never produce, long runs and concurrent contexts:
random segment tables (gaps, partial tensors, shuffled order, odd alignments) through pack,
unpack and accumulate; forty steps with loss-scale back-offs and growths, bit for bit;
two contexts stepping on two streams at once."""
import numpy as np
import pytest
import torch

from paper_2406_08334_amd import binding as B
from paper_2406_08334_amd import synth

from gpu_harness import ChunkedState, hp_pair, to_u16, same_bits, assert_same_bits

pytestmark = pytest.mark.gpu


def random_table(rng, C, S, n_tensors, max_len):
    """Segments at random, non-overlapping places: every chunk is cut into random pieces, a random
    subset of the pieces receives a random sub-range of a random tensor."""
    sizes = [int(rng.integers(1, max_len)) for _ in range(n_tensors)]
    table = []
    for c in range(C):
        cuts = np.unique(np.concatenate(([0, S], rng.integers(0, S, 24))))
        for lo, hi in zip(cuts[:-1], cuts[1:]):
            if rng.random() < 0.35:
                continue                                            # a gap
            t = int(rng.integers(0, n_tensors))
            n = int(min(hi - lo, sizes[t]))
            n = int(rng.integers(1, n + 1))
            so = int(rng.integers(0, sizes[t] - n + 1))
            table.append((t, so, n, c, int(lo)))
    order = rng.permutation(len(table))
    return sizes, [table[i] for i in order]


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("seed,C,S", [(1, 3, 40_000), (2, 2, 8192 * 3 + 8), (3, 5, 1000)])
def test_random_segment_tables_through_pack_unpack_and_norm(orc, dtype, seed, C, S):
    rng = np.random.default_rng(seed)
    sizes, table = random_table(rng, C, S, n_tensors=9, max_len=30_000)
    orc_dtype = orc.BF16 if dtype == torch.bfloat16 else orc.FP16
    # tensors: random finite 16-bit patterns
    host_t = []
    for n in sizes:
        w = rng.integers(0, 1 << 16, n, dtype=np.uint16)
        exp = 0x7F80 if dtype == torch.bfloat16 else 0x7C00
        w[(w & exp) == exp] &= np.uint16(0x3FFF)                   # no inf / NaN
        host_t.append(w)
    dev_t = [torch.from_numpy(w.view(np.int16)).cuda().view(dtype) for w in host_t]
    ctx = B.pt_ctx_create(B.PT_BF16 if dtype == torch.bfloat16 else B.PT_FP16, S, C, None)
    plan = None
    try:
        segs = [B.pt_segment(dev_t[t].data_ptr(), so, n, co, c, t) for t, so, n, c, co in table]
        plan = B.pt_pack_plan_create(ctx, segs)
        chunks = torch.full((C, S), 0.5, dtype=dtype, device="cuda")       # sentinel in the gaps
        sent = int(to_u16(chunks[0, :1])[0])
        B.pt_chunk_pack_grads(ctx, plan, [chunks[c] for c in range(C)])
        B.pt_chunk_grad_sqnorm(ctx, None, 0, C, B.PT_FINALIZE_CARRY)     # a random table may leave a chunk untouched
        rep = B.pt_step_report_read(ctx)
        want = np.full((C, S), sent, np.uint16)
        orc.pack_segments([(host_t[t], so, n, c, co) for t, so, n, c, co in table], want)
        assert_same_bits(to_u16(chunks), want, "pack")
        covered = np.zeros((C, S), np.uint16)
        orc.pack_segments([(host_t[t], so, n, c, co) for t, so, n, c, co in table], covered)
        want_sq = orc.sqnorm(covered.reshape(-1), orc_dtype, block=S, threads=4)      # gaps hold zero here
        assert rep.found_inf == 0 and abs(rep.sqnorm - want_sq) <= 1e-12 * want_sq
        # inverse copy into fresh tensors: exactly the covered source ranges come back
        back = [torch.full((n,), 0.25, dtype=dtype, device="cuda") for n in sizes]
        q = int(to_u16(back[0][:1])[0])
        segs_b = [B.pt_segment(back[t].data_ptr(), so, n, co, c, t) for t, so, n, c, co in table]
        plan_b = B.pt_pack_plan_create(ctx, segs_b)
        B.pt_chunk_unpack(ctx, plan_b, [chunks[c] for c in range(C)])
        torch.cuda.synchronize()
        B.pt_pack_plan_destroy(plan_b)
        exp_back = [np.full(n, q, np.uint16) for n in sizes]
        for t, so, n, c, co in table:          # a source range used twice receives equal words both times
            exp_back[t][so:so + n] = host_t[t][so:so + n]
        for t in range(len(sizes)):
            assert_same_bits(to_u16(back[t]), exp_back[t], ("unpack", t))
    finally:
        torch.cuda.synchronize()
        if plan is not None:
            B.pt_pack_plan_destroy(plan)
        B.pt_ctx_destroy(ctx)


@pytest.mark.parametrize("seed,C,S", [(4, 3, 40_000), (5, 2, 4096 * 5 + 24)])
def test_random_segment_tables_through_accumulate(orc, seed, C, S):
    rng = np.random.default_rng(seed)
    sizes, table = random_table(rng, C, S, n_tensors=7, max_len=25_000)
    ctx = B.pt_ctx_create(B.PT_BF16, S, C, None)
    B.pt_ctx_set_option(ctx, "grad_fp32", 1)
    plan = None
    try:
        dev_t = [torch.empty(n, dtype=torch.bfloat16, device="cuda") for n in sizes]
        segs = [B.pt_segment(dev_t[t].data_ptr(), so, n, co, c, t) for t, so, n, c, co in table]
        plan = B.pt_pack_plan_create(ctx, segs)
        acc = torch.full((C, S), -3.0, dtype=torch.float32, device="cuda")
        want = np.full(C * S, -3.0, np.float32)
        for k in range(3):
            host_t = []
            for i, n in enumerate(sizes):
                dev_t[i].normal_(0, 1.0, generator=None)
                host_t.append(to_u16(dev_t[i]).copy())
            B.pt_chunk_accum_grads(ctx, plan, [acc[c] for c in range(C)], k == 0, k == 2)
            for t, so, n, c, co in table:
                view = want[c * S + co: c * S + co + n]
                part = view.copy()
                orc.accum_f32(host_t[t][so:so + n], part, orc.BF16, overwrite=(k == 0))
                view[:] = part
            assert_same_bits(acc.cpu().numpy().reshape(-1), want, ("accumulate", k))
        B.pt_chunk_grad_sqnorm(ctx, None, 0, C, B.PT_FINALIZE_CARRY)
        rep = B.pt_step_report_read(ctx)
        cov = np.zeros(C * S, np.float32)
        for t, so, n, c, co in table:
            cov[c * S + co: c * S + co + n] = want[c * S + co: c * S + co + n]
        want_sq = orc.sqnorm_f32(cov, block=S, threads=4)
        assert abs(rep.sqnorm - want_sq) <= 1e-12 * want_sq
    finally:
        torch.cuda.synchronize()
        if plan is not None:
            B.pt_pack_plan_destroy(plan)
        B.pt_ctx_destroy(ctx)


def test_forty_steps_with_loss_scale_events_stay_bit_exact(orc):
    """growth every 3 good steps, an inf every 7th step: back-offs and growths interleave; the GPU
    state follows the oracle's fp32 sequence bit for bit through all of it"""
    sb = B.pt_scaler_cfg(1024.0, 2.0, 0.5, 3, 0)
    so = orc.ScalerCfg(1024.0, 2.0, 0.5, 3, 1)
    S = 4096 * 2 + 40
    st = ChunkedState([2 * S + 1000, 77], S, dtype=torch.float16, scaler=sb)
    try:
        hp_b, hp_o, _ = hp_pair(lr=3e-4)
        host = st.host_state()
        ost = orc.new_state(so)
        scales = []
        for s in range(1, 41):
            sigma = ost.loss_scale
            scales.append(sigma)
            st.set_grads(s, scale=sigma)
            if s % 7 == 0:
                st.grad_src.view(torch.int16)[(s * 131) % st.N] = 0x7C00
            st.pack(); st.norm(); st.adamw(hp_b)
            rep = B.pt_step_report_read(st.ctx)
            k = B.pt_update_consts_read(st.ctx)
            st.end()
            g16 = st.oracle_packed(orc)                              # the oracle packs the seeded sources itself
            assert_same_bits(to_u16(st.g16).reshape(-1), g16, ("g16", s))
            # the whole step in the oracle, fp32 sequence, its own norm, constants and loss-scale machine
            orep = orc.step(hp_o, so, ost, g16, host["w"], host["m"], host["v"], host["p16"], st.S, orc.FP16,
                            use_f32seq=True, threads=4)
            assert rep.found_inf == orep.found_inf == int(s % 7 == 0) and rep.loss_scale == orep.loss_scale_used == sigma
            if not orep.found_inf:
                assert same_bits(np.array(list(k.c), np.float32), orc.consts_f32(hp_o, ost.t, orep.grad_mult))
            after = B.pt_step_report_read(st.ctx)
            assert (after.step, after.loss_scale, after.good_steps) == (ost.t, ost.loss_scale, ost.good_steps), s
            got = st.host_state()
            for name in ("w", "m", "v", "p16"):
                assert_same_bits(got[name], host[name], (name, s))
        assert ost.t == 35 and len(set(scales)) >= 3            # the scale really moved both ways
    finally:
        st.close()


def test_two_contexts_on_two_streams_do_not_disturb_each_other(orc):
    sizes, S = [300_000, 4099, 65_536], 1 << 16
    solo = [ChunkedState(sizes, S, seed=i) for i in (0, 1)]
    duo = [ChunkedState(sizes, S, seed=i) for i in (0, 1)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    try:
        hp_b, _, _ = hp_pair()

        def step_on(st, stream):
            B.pt_chunk_pack_grads(st.ctx, st.plan, st.rows(st.g16), stream)
            B.pt_chunk_grad_sqnorm(st.ctx, None, 0, st.C, True, stream)
            B.pt_chunk_adamw_step(st.ctx, hp_b, 0, st.C, st.rows(st.g16), st.rows(st.w), st.rows(st.m), st.rows(st.v),
                                  st.rows(st.p16), stream)
            B.pt_step_end(st.ctx, stream)

        for s in (1, 2, 3, 4):
            for st in solo + duo:
                st.set_grads(s)
            torch.cuda.synchronize()
            for st in solo:                                     # one after the other, default stream
                step_on(st, torch.cuda.current_stream())
                torch.cuda.synchronize()
            for st, stream in zip(duo, streams):                # both enqueued before either is waited for
                step_on(st, stream)
            torch.cuda.synchronize()
        for a, b in zip(solo, duo):
            ha, hb = a.host_state(), b.host_state()
            for name in ("g16", "w", "m", "v", "p16"):
                assert_same_bits(hb[name], ha[name], name)
            assert a.report().norm == b.report().norm
    finally:
        for st in solo + duo:
            st.close()


def test_stream_reserve_tries_its_copy_streams_out_and_ends_with_a_pair_that_overlaps():
    """A stream keeps the copy engine of its first copy, and two copy streams that took the same one carry one
    direction of the link at a time.  pt_stream_reserve makes the first copies itself, side by side, then measures
    (one copy up, one down, both at once) and replaces a pair that does not overlap.  Here: a process that has created
    and destroyed other streams right before, several contexts in a row - every reservation must end with an
    overlapping pair; the replacement forced from the host; and small chunk buffers, which skip the test."""
    S = 1 << 22                                   # 64 MiB chunk buffers: large enough to measure
    ctxs = []
    try:
        for k in range(3):
            junk = [torch.cuda.Stream() for _ in range(k + 1)]
            for s in junk:
                with torch.cuda.stream(s):
                    torch.zeros(8, device="cuda")
            torch.cuda.synchronize()
            del junk
            ctx = B.pt_ctx_create(B.PT_BF16, S, 4, None)
            ctxs.append(ctx)
            B.pt_stream_reserve(ctx, 2)
            st = B.pt_stream_status(ctx)
            print(f"[stream self-test] context {k}: {st}", flush=True)
            assert st["duplex_tested"] and st["duplex_ok"] and 1 <= st["attempts"] <= 6, st
        # the replacement itself, forced from the host: two stream pairs rejected whatever they measure, the third
        # kept; the streamed update through the replaced stream still gives the resident bits
        forced = B.pt_ctx_create(B.PT_BF16, S, 4, None)
        ctxs.append(forced)
        B.pt_ctx_set_option(forced, "stream_test_reject", 2)
        B.pt_stream_reserve(forced, 2)
        st = B.pt_stream_status(forced)
        assert st["duplex_tested"] and st["duplex_ok"] and st["attempts"] == 3, st
        hp_b, _, _ = hp_pair()
        dev = {k: torch.zeros(2, S, dtype=dt, device="cuda") for k, dt in
               (("g", torch.bfloat16), ("p", torch.bfloat16), ("w", torch.float32), ("m", torch.float32), ("v", torch.float32))}
        synth.normal_16(synth.SEED_GRADS, 1, 0, 0, 2 * S, 1e-3, torch.bfloat16, "cuda", out=dev["g"].view(-1))
        synth.normal_16(synth.SEED_PARAMS, 0, 0, 0, 2 * S, 0.02, torch.bfloat16, "cuda", out=dev["p"].view(-1))
        dev["w"].copy_(dev["p"])
        host = {k: [t[c].cpu().pin_memory() for c in range(2)] for k, t in dev.items()}
        rows = lambda k: [dev[k][0], dev[k][1]]

        def step_and_compare(tag):
            B.pt_chunk_grad_sqnorm(forced, [dev["g"][0], dev["g"][1], None, None], 0, 2, False)
            B.pt_chunk_grad_sqnorm(forced, None, 0, 4, B.PT_FINALIZE_CARRY)
            B.pt_chunk_stream_step(forced, hp_b, 2, 2, host["g"], host["w"], host["m"], host["v"], host["p"])
            B.pt_chunk_adamw_step(forced, hp_b, 0, 2, rows("g"), rows("w"), rows("m"), rows("v"), rows("p"))
            B.pt_step_end(forced)
            torch.cuda.synchronize()
            for k in ("w", "m", "v", "p"):
                for c in range(2):
                    view = torch.int16 if k == "p" else torch.int32
                    assert torch.equal(host[k][c].view(view), dev[k][c].cpu().view(view)), (tag, k, c)
        step_and_compare("first step")
        assert B.pt_stream_status(forced)["rebuilds"] == 0
        # A step that ran with its two directions behind each other makes the next call replace the side streams;
        # here the verdict on the finished step is forced from the host.  Same bits through the new streams.
        B.pt_ctx_set_option(forced, "stream_test_unhealthy", 1)
        step_and_compare("step after the verdict")
        st = B.pt_stream_status(forced)
        assert st["rebuilds"] == 1 and st["duplex_tested"], st
        step_and_compare("a further step")
        assert B.pt_stream_status(forced)["rebuilds"] == 1
        small = B.pt_ctx_create(B.PT_BF16, 4096, 2, None)
        ctxs.append(small)
        B.pt_stream_reserve(small, 2)
        assert B.pt_stream_status(small) == {"duplex_tested": False, "duplex_ok": False, "attempts": 0, "rebuilds": 0}
    finally:
        torch.cuda.synchronize()
        for ctx in ctxs:
            B.pt_ctx_destroy(ctx)
