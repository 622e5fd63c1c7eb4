"""GPU parity of the gradient-accumulation variant: micro-batches of 16-bit gradients summed
into fp32 gradient chunks, norm / clipping / update reading those chunks (resident, streamed
and host-side), and the update that zeroes the gradients it has read."""
import math

import numpy as np
import pytest
import torch

from paper_2406_08334_amd import binding as B
from paper_2406_08334_amd import shapes

from gpu_harness import ChunkedState, hp_pair, to_u16, same_bits, assert_same_bits
from test_gpu_parity import RAGGED, ALIGNED
from tolerance import ScaleTracker, check_p16, far_cap

pytestmark = pytest.mark.gpu

SCALER_B = B.pt_scaler_cfg(65536.0, 2.0, 0.5, 2000, 0)


def flat_words(orc, st):
    """the micro-batch's source words laid out as the chunks' flat concatenation (oracle pack)"""
    return st.oracle_packed(orc)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("sizes,S", [(RAGGED, 16384 * 2 + 64), (RAGGED, 1024), (ALIGNED, 32768), ([5], 8),
                                     ([7_087_872], 1 << 22)])
def test_accumulation_is_bit_exact_and_leaves_padding_alone(orc, dtype, sizes, S):
    st = ChunkedState(sizes, S, dtype=dtype, grad_fp32=True, init_params=False)
    try:
        N, pad = st.N, st.C * S - st.N
        st.g32.fill_(-7.5)                                        # sentinel: overwrite must not depend on old content
        want = np.full(st.C * S, -7.5, np.float32)
        sigma = 1.0
        for k in range(3):
            st.set_grads(1, std=1e-3, micro=k)
            if k == 1 and N > 4:                                   # an inf now, the opposite one next: NaN
                st.grad_src.view(torch.int16)[N // 2] = 0x7C00 if dtype == torch.float16 else 0x7F80
            if k == 2 and N > 4:
                st.grad_src.view(torch.int16)[N // 2] = -1024 if dtype == torch.float16 else -128   # 0xFC00 / 0xFF80
            st.accum(overwrite=(k == 0), take_norm=(k == 2))
            words = flat_words(orc, st)
            part = want[:N].copy()
            orc.accum_f32(words[:N], part, st.orc_dtype, overwrite=(k == 0))
            want[:N] = part
            got = st.host_state()["g32"]
            same = (got.view(np.uint32) == want.view(np.uint32)) | (np.isnan(got) & np.isnan(want))
            assert same.all(), (k, int((~same).sum()), np.flatnonzero(~same)[:5])
        if pad:
            assert (got[N:] == -7.5).all()                         # never written
        st.g32.view(-1)[N:].zero_()
        st.norm()
        rep = st.report()
        assert rep.found_inf == (1 if N > 4 else 0)
        if N > 4:
            assert math.isnan(got[N // 2])
        # finite case for the norm: put a finite value back, recompute from the chunks
        if N > 4:
            st.g32.view(-1)[N // 2] = 0.25
            got[N // 2] = 0.25
        got[N:] = 0
        st.norm(recompute=True)
        rep = st.report()
        want_sq = orc.sqnorm_f32(got, loss_scale=sigma, block=S, threads=8)
        assert rep.found_inf == 0 and abs(rep.sqnorm - want_sq) <= 1e-12 * want_sq
    finally:
        st.close()


@pytest.mark.parametrize("dtype,scaler", [(torch.bfloat16, None), (torch.float16, SCALER_B)])
def test_fused_norm_of_the_last_micro_batch_equals_the_recomputed_one(orc, dtype, scaler):
    st = ChunkedState(RAGGED + [300_000], 65536 + 8, dtype=dtype, scaler=scaler, grad_fp32=True)
    try:
        sigma = 65536.0 if scaler is not None else 1.0
        for k in range(4):
            st.set_grads(1, std=1e-3, scale=sigma, micro=k)
            st.accum(overwrite=(k == 0), take_norm=(k == 3))
        st.norm()
        fused = st.report()
        st.norm(recompute=True)
        again = st.report()
        g = st.host_state()["g32"]
        want = orc.sqnorm_f32(g, loss_scale=sigma, block=st.S, threads=8)
        assert abs(fused.sqnorm - want) <= 1e-12 * want and abs(again.sqnorm - want) <= 1e-12 * want
        assert abs(math.sqrt(want) - 2e-3 * math.sqrt(st.N)) < 0.02 * 2e-3 * math.sqrt(st.N)     # four draws: std doubles
        assert fused.found_inf == 0 and again.found_inf == 0
    finally:
        st.close()


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("unroll,zero,masked", [(4, False, False), (1, True, False), (8, False, True), (4, True, True)])
def test_update_from_fp32_gradients_is_bit_exact_against_the_f32_sequence(orc, dtype, unroll, zero, masked):
    S, C = 4096 * 3 + 40, 3
    st = ChunkedState([S * C - 5], S, dtype=dtype, grad_fp32=True)
    try:
        B.pt_ctx_set_option(st.ctx, "adamw_unroll", unroll)
        B.pt_ctx_set_option(st.ctx, "adamw_zero_grads", int(zero))
        B.pt_ctx_set_option(st.ctx, "adamw_nt", 1 if unroll != 8 else 2)     # hinted accesses too (a small state gets none by default)
        mask = st.set_no_decay(runs=[(0, 100, 5000), (1, 0, S), (2, S - 41, 41)]) if masked else None
        hp_b, hp_o, hpd = hp_pair()
        host = st.host_state()
        h64 = {k: a.copy() for k, a in host.items()}
        trk = ScaleTracker(host["w"], host["m"], hpd)
        gm = 0.0121
        for t in (1, 2, 3):
            g32 = np.zeros(st.C * S, np.float32)
            for k in range(2):
                st.set_grads(t, micro=k)
                st.accum(overwrite=(k == 0), take_norm=False)
                part = g32[:st.N].copy()                          # the oracle accumulates the same sources itself
                orc.accum_f32(flat_words(orc, st)[:st.N], part, st.orc_dtype, overwrite=(k == 0))
                g32[:st.N] = part
            assert_same_bits(st.host_state()["g32"], g32, ("g32", t))
            assert not np.array_equal(orc.decode16(orc.encode16_rne(g32, st.orc_dtype), st.orc_dtype), g32)
            B.pt_step_override(st.ctx, gm, False)
            st.adamw(hp_b)
            k_ = B.pt_update_consts_read(st.ctx)
            st.end()
            consts = orc.consts_f32(hp_o, t, float(np.float32(gm)))
            assert same_bits(np.array(list(k_.c), dtype=np.float32), consts)    # the oracle runs on its own constants
            orc.adamw_f32seq_g32(consts, g32, host["w"], host["m"], host["v"], host["p16"], st.orc_dtype, threads=8,
                                 no_decay=mask)
            got = st.host_state()
            for name in ("w", "m", "v", "p16"):
                assert_same_bits(got[name], host[name], (name, t))
            if zero:
                assert not got["g32"].view(np.uint32).any()        # +0.0 everywhere
            else:
                assert same_bits(got["g32"], g32)                  # read-only otherwise
            gmf = float(np.float32(gm))
            orc.adamw_f64_g32(hp_o, t, gmf, g32, h64["w"], h64["m"], h64["v"], h64["p16"], st.orc_dtype, threads=8,
                              no_decay=mask)
            trk.advance(t, g32.astype(np.float64) * gmf, h64["v"])
            trk.check((got["w"], got["m"], got["v"]), (h64["w"], h64["m"], h64["v"]), tol=1e-6)
            far = check_p16(orc.decode16(got["p16"], st.orc_dtype), orc.decode16(h64["p16"], st.orc_dtype), h64["w"],
                            trk.W, dtype == torch.float16)
            assert far <= far_cap(got["p16"].size)
    finally:
        st.close()


def test_zeroing_also_serves_16_bit_gradient_chunks_and_clears_a_skipped_step(orc):
    S = 4096 * 2 + 8
    st = ChunkedState([3 * S - 3], S, dtype=torch.float16, scaler=SCALER_B)
    try:
        B.pt_ctx_set_option(st.ctx, "adamw_zero_grads", 1)
        hp_b, _, _ = hp_pair()
        ref = ChunkedState([3 * S - 3], S, dtype=torch.float16, scaler=SCALER_B)
        for step, bad in ((1, False), (2, True), (3, False)):
            for s_ in (st, ref):
                s_.set_grads(step, scale=65536.0 if step < 3 else 32768.0)
                if bad:
                    s_.grad_src.view(torch.int16)[77] = 0x7C00
                s_.pack(); s_.norm()
            st.adamw(hp_b); ref.adamw(hp_b)
            st.end(); ref.end()
            a, b = st.host_state(), ref.host_state()
            for name in ("w", "m", "v", "p16"):
                assert same_bits(a[name], b[name]), (name, step)     # zeroing changes no result
            assert not a["g16"].any()                                  # zeroed after an applied AND after a skipped step
        assert st.report().step == 2
        ref.close()
    finally:
        st.close()


def test_add_into_accumulation_recovers_after_an_overflow(orc):
    """A caller whose backward pass ADDS into the fp32 gradient chunks (no overwrite for the first
    micro-batch) relies on the update to zero them.  With an inf in step 2 the step is skipped, the
    loss scale halves, and step 3 must be applied again: the inf may not stay in the sums."""
    S = 4096 + 8
    sizes = [2 * S - 5]
    st = ChunkedState(sizes, S, dtype=torch.float16, scaler=SCALER_B, grad_fp32=True)
    try:
        B.pt_ctx_set_option(st.ctx, "adamw_zero_grads", 1)
        hp_b, hp_o, _ = hp_pair()
        host = st.host_state()
        SCALER_O = orc.ScalerCfg(65536.0, 2.0, 0.5, 2000, 1)
        ost = orc.new_state(SCALER_O)
        n = st.C * S
        found = []
        for step, bad in ((1, False), (2, True), (3, False), (4, False)):
            sigma = ost.loss_scale
            g32 = np.zeros(n, np.float32)
            for micro in range(2):
                st.set_grads(step, scale=sigma, micro=micro)
                if bad and micro == 0:
                    st.grad_src.view(torch.int16)[31] = 0x7C00
                st.accum(overwrite=False, take_norm=(micro == 1))      # always adds: the chunks start at zero
                src = to_u16(st.grad_src[:st.N])
                part = np.zeros(n, np.uint16); part[:st.N] = src
                orc.accum_f32(part, g32, st.orc_dtype, overwrite=False)
            st.norm()
            st.adamw(hp_b)
            rep = st.report()
            st.end()
            found.append(rep.found_inf)
            orep = orc.step_g32(hp_o, SCALER_O, ost, g32, host["w"], host["m"], host["v"], host["p16"], S, st.orc_dtype,
                                use_f32seq=True, threads=4)
            assert rep.found_inf == orep.found_inf == int(bad)
            got = st.host_state()
            for name in ("w", "m", "v", "p16"):
                assert_same_bits(got[name], host[name], (name, step))
            assert not got["g32"].view(np.uint32).any(), step
        assert found == [0, 1, 0, 0] and st.report().step == 3 and st.report().loss_scale == 32768.0
    finally:
        st.close()


def end_to_end_accum(orc, sizes, S, dtype, steps, micro, scaler_b=None, scaler_o=None, inf_at=None, no_decay_tensors=None):
    st = ChunkedState(sizes, S, dtype=dtype, scaler=scaler_b, grad_fp32=True)
    try:
        hp_b, hp_o, hpd = hp_pair()
        mask = st.set_no_decay(tensors=no_decay_tensors) if no_decay_tensors is not None else None
        host = st.host_state()
        fa = {k: a.copy() for k, a in host.items()}
        ost = orc.new_state(scaler_o)
        trk = ScaleTracker(host["w"], host["m"], hpd)
        reps = []
        for s in range(1, steps + 1):
            sigma = ost.loss_scale
            g32 = np.zeros(st.C * S, np.float32)
            for k in range(micro):
                st.set_grads(s, std=1e-3, scale=sigma, micro=k)
                if inf_at == (s, k):
                    st.grad_src.view(torch.int16)[st.N // 3] = 0x7C00 if dtype == torch.float16 else 0x7F80
                st.accum(overwrite=(k == 0), take_norm=(k == micro - 1))
                part = g32[:st.N].copy()                          # the oracle accumulates the same sources itself
                orc.accum_f32(st.oracle_packed(orc)[:st.N], part, st.orc_dtype, overwrite=(k == 0))
                g32[:st.N] = part
            st.norm()
            st.adamw(hp_b)
            rep = B.pt_step_report_read(st.ctx)
            k_ = B.pt_update_consts_read(st.ctx)
            st.end()
            got = st.host_state()
            same = (got["g32"].view(np.uint32) == g32.view(np.uint32)) | (np.isnan(got["g32"]) & np.isnan(g32))
            assert same.all()
            orep = orc.step_g32(hp_o, scaler_o, ost, g32, host["w"], host["m"], host["v"], host["p16"], S, st.orc_dtype,
                                threads=8, no_decay=mask)
            reps.append((rep, orep))
            assert rep.found_inf == orep.found_inf and rep.loss_scale == orep.loss_scale_used
            after = B.pt_step_report_read(st.ctx)
            assert after.step == ost.t and after.loss_scale == ost.loss_scale
            if orep.found_inf:
                assert k_.skip == 1
                for name in ("w", "m", "v", "p16"):
                    assert_same_bits(got[name], fa[name], name)
                continue
            assert abs(rep.norm - orep.norm) <= 1e-12 * orep.norm
            assert abs(rep.grad_mult - orep.grad_mult) <= 6e-8 * orep.grad_mult
            trk.advance(ost.t, g32.astype(np.float64) * orep.grad_mult, host["v"])
            trk.check((got["w"], got["m"], got["v"]), (host["w"], host["m"], host["v"]), tol=1e-6)
            far = check_p16(orc.decode16(got["p16"], st.orc_dtype), orc.decode16(host["p16"], st.orc_dtype),
                            host["w"], trk.W, dtype == torch.float16)
            assert far <= far_cap(got["p16"].size)
            consts = orc.consts_f32(hp_o, ost.t, orep.grad_mult)            # the oracle's own constants
            assert same_bits(np.array(list(k_.c), dtype=np.float32), consts)
            orc.adamw_f32seq_g32(consts, g32, fa["w"], fa["m"], fa["v"], fa["p16"], st.orc_dtype, threads=8, no_decay=mask)
            for name in ("w", "m", "v", "p16"):
                assert_same_bits(got[name], fa[name], (name, s))
        return reps
    finally:
        st.close()


def test_end_to_end_gpt2_block_four_micro_batches(orc):
    table, _ = shapes.workload("gpt2_block_768")
    nd = [i for i, (name, _) in enumerate(table) if name.endswith(".bias") or ".ln_" in name]
    reps = end_to_end_accum(orc, [n for _, n in table], 1 << 20, torch.bfloat16, steps=3, micro=4, no_decay_tensors=nd)
    for rep, orep in reps:
        assert abs(orep.norm - 2 * 2.662) < 0.03 and rep.clip_coef < 0.2       # sum of four draws: twice the norm of one


def test_end_to_end_fp16_loss_scaling_with_an_inf_in_the_middle_micro_batch(orc):
    so = orc.ScalerCfg(65536.0, 2.0, 0.5, 2000, 1)
    reps = end_to_end_accum(orc, [1_000_000, 333, 4096 * 9], 1 << 18, torch.float16, steps=4, micro=3,
                            scaler_b=SCALER_B, scaler_o=so, inf_at=(2, 1))
    assert [r.found_inf for r, _ in reps] == [0, 1, 0, 0]
    assert [r.loss_scale for r, _ in reps] == [65536.0, 65536.0, 32768.0, 32768.0]


def run_split(n_persist, mode, dtype, scaler, steps=2, micro=2, masked=True, orc=None):
    """6 chunks with fp32 gradient chunks; chunks >= n_persist live in pinned host memory and are
    streamed through chunk buffers (mode 'stream') or updated by host threads (mode 'host').  With
    `orc` the oracle accumulates the same seeded micro-batches and takes every step itself; all
    chunks must end up with its bits."""
    S = 40_000
    st = ChunkedState([6 * S - 24], S, dtype=dtype, scaler=scaler, grad_fp32=True)
    try:
        hp_b, hp_o, _ = hp_pair()
        mask = None
        if masked:
            mask = st.set_no_decay(runs=[(0, 0, 100), (2, 0, S), (3, 4095, 3), (5, 39_900, 76)])
        C = st.C
        host = {}
        if orc is not None:
            shadow = st.host_state()
            sc_o = None if scaler is None else orc.ScalerCfg(scaler.init_scale, scaler.growth, scaler.backoff,
                                                             scaler.growth_interval, 1)
            ost = orc.new_state(sc_o)
            og32 = np.zeros(C * S, np.float32)
        if n_persist < C:
            if mode == "stream":
                B.pt_stream_reserve(st.ctx, 3)
            for name, arena in (("g32", st.g32), ("p16", st.p16), ("w", st.w), ("m", st.m), ("v", st.v)):
                host[name] = [torch.empty(S, dtype=arena.dtype, pin_memory=True) for _ in range(n_persist, C)]
            for name, arena in (("p16", st.p16), ("w", st.w), ("m", st.m), ("v", st.v)):
                for i, c in enumerate(range(n_persist, C)):
                    host[name][i].copy_(arena[c])
                arena[n_persist:].fill_(7)
        sigma = 65536.0 if scaler is not None else 1.0
        for s in range(1, steps + 1):
            for k in range(micro):
                st.set_grads(s, scale=sigma, micro=k)
                st.accum(overwrite=(k == 0), take_norm=(k == micro - 1))
                if orc is not None:
                    orc.accum_f32(st.oracle_packed(orc), og32, st.orc_dtype, overwrite=(k == 0))
            if orc is not None:
                orc.step_g32(hp_o, sc_o, ost, og32, shadow["w"], shadow["m"], shadow["v"], shadow["p16"], S, st.orc_dtype,
                             use_f32seq=True, threads=4, no_decay=mask)
            for i, c in enumerate(range(n_persist, C)):
                host["g32"][i].copy_(st.g32[c])
            torch.cuda.synchronize()
            st.norm()
            if n_persist < C and mode == "stream":
                B.pt_chunk_stream_step(st.ctx, hp_b, n_persist, C - n_persist, host["g32"], host["w"], host["m"],
                                       host["v"], host["p16"])
            if n_persist > 0:
                st.adamw(hp_b, 0, n_persist)
            if n_persist < C and mode == "host":
                B.pt_chunk_host_adamw_step(st.ctx, hp_b, n_persist, C - n_persist, host["g32"], host["w"], host["m"],
                                           host["v"], host["p16"], 5)
            st.end()
        torch.cuda.synchronize()
        out = {}
        for name, arena in (("p16", st.p16), ("w", st.w), ("m", st.m), ("v", st.v)):
            full = arena.clone()
            for i, c in enumerate(range(n_persist, C)):
                full[c].copy_(host[name][i])
            out[name] = full.cpu()
        if orc is not None:
            for name in ("p16", "w", "m", "v"):
                got = to_u16(out[name]).reshape(-1) if out[name].element_size() == 2 else out[name].numpy().reshape(-1)
                assert_same_bits(got, shadow[name], (name, "against the oracle", n_persist, mode))
        return out
    finally:
        st.close()


@pytest.mark.parametrize("dtype,scaler", [(torch.bfloat16, None), (torch.float16, SCALER_B)])
def test_streamed_and_host_updated_chunks_with_fp32_gradients_equal_the_oracle_and_the_resident_bits(orc, dtype, scaler):
    ref = run_split(6, "stream", dtype, scaler, orc=orc)
    for n_persist, mode in ((3, "stream"), (0, "stream"), (5, "stream"), (3, "host"), (0, "host")):
        got = run_split(n_persist, mode, dtype, scaler, orc=orc)
        for name in ("p16", "w", "m", "v"):
            view = torch.int16 if got[name].element_size() == 2 else torch.int32
            assert torch.equal(got[name].view(view), ref[name].view(view)), (name, n_persist, mode)


def test_the_two_gradient_storages_refuse_each_other_s_calls():
    st = ChunkedState([10_000], 4096, grad_fp32=True)
    try:
        with pytest.raises(B.PtError) as e:
            st.pack()
        assert e.value.status == B.PT_ERR_STATE
        B.pt_stream_reserve(st.ctx, 2)
        with pytest.raises(B.PtError) as e:
            B.pt_ctx_set_option(st.ctx, "grad_fp32", 0)           # the chunk buffers are sized already
        assert e.value.status == B.PT_ERR_STATE
        B.pt_ctx_set_option(st.ctx, "grad_fp32", 1)                # unchanged value: fine
        st.set_grads(1)
        st.accum(True, True)                                       # the context still works
    finally:
        st.close()
    st = ChunkedState([10_000], 4096)
    try:
        g32 = torch.zeros(st.C, st.S, dtype=torch.float32, device="cuda")
        with pytest.raises(B.PtError) as e:
            B.pt_chunk_accum_grads(st.ctx, st.plan, [g32[c] for c in range(st.C)], True, True)
        assert e.value.status == B.PT_ERR_STATE
    finally:
        st.close()
