"""Pins for the oracle's AdamW update and loss-scale machine.

The paper names the optimizer only ("FusedAdam" on the GPU, "CPU Adam" on the
host, Appendix A.1; fp32 update under mixed precision, Background).  The update is
the textbook one and is pinned here against: closed forms, a 60-digit evaluation
(mpmath), and torch.optim.AdamW + clip_grad_norm_ in fp64 as a library routine.
"""
import math

import mpmath
import numpy as np
import pytest
import torch

import oracle as O
from tolerance import ScaleTracker, ulp16_distance
from paper_2406_08334_amd import synth

HP = dict(lr=1e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, max_norm=1.0)


def hp(**kw):
    d = dict(HP); d.update(kw)
    return O.Hparams(**d)


def bf16w(x):
    return torch.as_tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def fresh(n, seed=0, std_w=0.02, std_g=1e-3):
    p = synth.normal_16(synth.SEED_PARAMS + seed, 0, 0, 0, n, std_w, torch.bfloat16, "cpu")
    g = synth.normal_16(synth.SEED_GRADS + seed, 1, 0, 0, n, std_g, torch.bfloat16, "cpu")
    w = p.float().numpy().copy()
    return synth.as_u16(g).copy(), w, np.zeros(n, np.float32), np.zeros(n, np.float32), synth.as_u16(p).copy()


def ulp32(x):
    return np.spacing(np.abs(x).astype(np.float32)).astype(np.float64)


def test_first_step_from_zero_state_closed_form(orc):
    n = 5000
    g16, w, m, v, p16 = fresh(n)
    w0 = w.astype(np.float64)
    gm = 0.0123
    g = orc.decode16(g16, orc.BF16).astype(np.float64) * gm
    h = hp()
    orc.adamw_f64(h, 1, gm, g16, w, m, v, p16, orc.BF16)
    # m = (1-b1) g, v = (1-b2) g^2, and exactly dw = -lr g/(|g|+eps) - lr wd w
    assert np.all(np.abs(m - (1 - 0.9) * g) <= 0.5 * ulp32(m) * 1.0001)
    assert np.all(np.abs(v - (1 - 0.95) * g * g) <= 0.5 * ulp32(v) * 1.0001)
    want = w0 - 1e-4 * g / (np.abs(g) + 1e-8) - 1e-4 * 0.1 * w0
    assert np.all(np.abs(w - want) <= 0.5 * ulp32(w) * 1.0001 + 1e-17)
    assert np.array_equal(p16, orc.encode16_rne(w, orc.BF16))


def test_first_step_is_about_lr_sign_g(orc):
    n = 2000
    g16, w, m, v, p16 = fresh(n, std_g=1.0)
    g = orc.decode16(g16, orc.BF16)
    big = np.abs(g) >= 1e-3
    w0 = w.copy()
    orc.adamw_f64(hp(weight_decay=0.0), 1, 1.0, g16, w, m, v, p16, orc.BF16)
    dw = w.astype(np.float64) - w0
    assert np.all(np.abs(dw[big] + 1e-4 * np.sign(g[big])) < 1e-4 * 2e-5 + ulp32(w0[big]))


def test_zero_gradient_only_decays(orc):
    n = 1000
    _, w, m, v, p16 = fresh(n)
    g16 = np.zeros(n, np.uint16)
    w0 = w.astype(np.float64)
    orc.adamw_f64(hp(), 1, 1.0, g16, w, m, v, p16, orc.BF16)
    assert not m.any() and not v.any()
    assert np.all(np.abs(w - w0 * (1 - 1e-5)) <= 0.5 * ulp32(w) * 1.0001)
    # padding (w = 0, g = 0) stays exactly zero forever
    wz, mz, vz = (np.zeros(16, np.float32) for _ in range(3))
    pz = np.zeros(16, np.uint16)
    for t in range(1, 6):
        orc.adamw_f64(hp(), t, 0.37, np.zeros(16, np.uint16), wz, mz, vz, pz, orc.BF16)
    assert not wz.any() and not mz.any() and not vz.any() and not pz.any()


def test_constant_gradient_moves_lr_per_step(orc):
    # with wd = 0 and the same g every step, bias correction gives m^ = g, v^ = g^2
    n, T = 512, 7
    g16, w, m, v, p16 = fresh(n, std_g=1.0)
    g = orc.decode16(g16, orc.BF16).astype(np.float64)
    w0 = w.astype(np.float64)
    h = hp(weight_decay=0.0)
    for t in range(1, T + 1):
        orc.adamw_f64(h, t, 1.0, g16, w, m, v, p16, orc.BF16)
    want = w0 - T * 1e-4 * g / (np.abs(g) + 1e-8)
    # fp32 storage of m, v, w perturbs each step by a few ulp
    assert np.all(np.abs(w - want) <= 1e-6 * (np.abs(w0) + T * 1e-4))


def test_zero_betas_is_sign_descent_and_zero_lr_freezes_w(orc):
    n = 512
    g16, w, m, v, p16 = fresh(n, std_g=1.0)
    g = orc.decode16(g16, orc.BF16).astype(np.float64)
    w0 = w.astype(np.float64)
    h = hp(beta1=0.0, beta2=0.0, weight_decay=0.0)
    orc.adamw_f64(h, 1, 1.0, g16, w, m, v, p16, orc.BF16)
    orc.adamw_f64(h, 2, 1.0, g16, w, m, v, p16, orc.BF16)
    assert np.allclose(m, g, rtol=1e-7) and np.allclose(v, g * g, rtol=1e-7)
    assert np.all(np.abs(w - (w0 - 2e-4 * g / (np.abs(g) + 1e-8))) <= 2e-7 * (np.abs(w0) + 2e-4))
    g16, w, m, v, p16 = fresh(n)
    w0 = w.copy()
    orc.adamw_f64(hp(lr=0.0), 1, 1.0, g16, w, m, v, p16, orc.BF16)
    assert np.array_equal(w, w0) and m.any() and v.any()


def test_against_60_digit_evaluation(orc):
    mpmath.mp.dps = 60
    rng = np.random.default_rng(11)
    n = 64
    g16 = bf16w(rng.normal(0, 1e-3, n))
    w = rng.normal(0, 0.02, n).astype(np.float32)
    m = rng.normal(0, 1e-5, n).astype(np.float32)
    v = (rng.normal(0, 1e-5, n) ** 2).astype(np.float32)
    p16 = np.zeros(n, np.uint16)
    t, gm = 3, 0.0121212
    h = hp()
    w0, m0, v0 = w.copy(), m.copy(), v.copy()
    gd = orc.decode16(g16, orc.BF16)
    orc.adamw_f64(h, t, gm, g16, w, m, v, p16, orc.BF16)
    M = mpmath.mpf
    for i in range(n):
        g = M(float(gd[i])) * M(gm)
        mn = M(0.9) * M(float(m0[i])) + (1 - M(0.9)) * g
        vn = M(0.95) * M(float(v0[i])) + (1 - M(0.95)) * g * g
        den = mpmath.sqrt(vn) / mpmath.sqrt(1 - M(0.95) ** t) + M(1e-8)
        wn = M(float(w0[i])) * (1 - M(1e-4) * M(0.1)) - M(1e-4) / (1 - M(0.9) ** t) * mn / den
        for got, want in ((m[i], mn), (v[i], vn), (w[i], wn)):
            # fp64 evaluation rounded once to fp32: within half an fp32 ulp (+ fp64 noise)
            err = abs(M(float(got)) - want)
            assert err <= M(float(np.spacing(np.float32(abs(got))))) * M("0.5000001"), (i, got, want)


def _torch_reference(g_steps, w0, hpd, steps):
    p = torch.nn.Parameter(torch.tensor(w0, dtype=torch.float64))
    opt = torch.optim.AdamW([p], lr=hpd["lr"], betas=(hpd["beta1"], hpd["beta2"]), eps=hpd["eps"],
                            weight_decay=hpd["weight_decay"], amsgrad=False)
    norms = []
    for s in range(steps):
        p.grad = torch.tensor(g_steps[s], dtype=torch.float64)
        norms.append(float(torch.nn.utils.clip_grad_norm_([p], hpd["max_norm"])))
        opt.step()
    st = opt.state[p]
    return p.detach().numpy(), st["exp_avg"].numpy(), st["exp_avg_sq"].numpy(), norms


@pytest.mark.parametrize("f32seq", [False, True])
def test_whole_step_against_torch_adamw_fp64(orc, f32seq):
    # library routine as the pin: clip_grad_norm_ (global L2, coef = c/(norm+1e-6) clamped to 1)
    # followed by torch.optim.AdamW, all in fp64, three steps with fresh gradients (norm ~ 14 > 1)
    n, S, steps = 20_000, 4096, 3
    _, w, m, v, p16 = fresh(n)
    w0 = w.copy()
    gs16 = [synth.as_u16(synth.normal_16(synth.SEED_GRADS, s + 1, 0, 0, n, 0.1, torch.bfloat16, "cpu")).copy()
            for s in range(steps)]
    h = hp()
    st = orc.new_state(None)
    trk = ScaleTracker(w0, m, HP)
    gsf = [orc.decode16(g, orc.BF16).astype(np.float64) for g in gs16]
    reps = []
    for s in range(steps):
        reps.append(orc.step(h, None, st, gs16[s], w, m, v, p16, S, orc.BF16, use_f32seq=f32seq, threads=2))
        trk.advance(s + 1, gsf[s] * reps[-1].grad_mult, v)
    assert st.t == steps
    wt, mt, vt, norms = _torch_reference(gsf, w0, HP, steps)
    for r, nt in zip(reps, norms):
        assert abs(r.norm - nt) <= 1e-12 * nt and r.found_inf == 0
        assert r.clip_coef < 0.1
    trk.check((w, m, v), (wt, mt, vt), tol=1e-6)
    assert np.array_equal(p16, orc.encode16_rne(w, orc.BF16))


def test_clip_is_active_and_inactive_as_the_norm_says(orc):
    n, S = 20_000, 4096
    g16, w, m, v, p16 = fresh(n)                       # norm ~ 1e-3*sqrt(20000) = 0.141 < 1
    st = orc.new_state(None)
    r = orc.step(hp(), None, st, g16, w, m, v, p16, S, orc.BF16)
    assert r.clip_coef == 1.0 and r.grad_mult == 1.0
    g16, w, m, v, p16 = fresh(n, std_g=0.1)            # norm ~ 14.1 > 1
    r = orc.step(hp(), None, orc.new_state(None), g16, w, m, v, p16, S, orc.BF16)
    assert r.clip_coef == 1.0 / (r.norm + 1e-6)
    gm = orc.decode16(g16, orc.BF16).astype(np.float64) * r.grad_mult
    assert abs(math.sqrt(float(np.sum(gm * gm))) - 1.0) < 1e-6     # clipped to the unit ball
    assert np.all(np.abs(m - 0.1 * gm) <= 0.5 * ulp32(m) * 1.0001)


def test_f32_sequence_stays_within_tolerance_of_fp64(orc):
    n = 200_000
    g16, w, m, v, p16 = fresh(n)
    wa, ma, va, pa = w.copy(), m.copy(), v.copy(), p16.copy()
    h = hp()
    gm = 1.0 / 82.0
    trk = ScaleTracker(w, m, HP)
    for t in range(1, 6):
        g16 = synth.as_u16(synth.normal_16(synth.SEED_GRADS, t, 0, 0, n, 1e-3, torch.bfloat16, "cpu")).copy()
        orc.adamw_f64(h, t, gm, g16, w, m, v, p16, orc.BF16)
        orc.adamw_f32seq(orc.consts_f32(h, t, gm), g16, wa, ma, va, pa, orc.BF16)
        trk.advance(t, orc.decode16(g16, orc.BF16).astype(np.float64) * gm, v)
        trk.check((wa, ma, va), (w, m, v), tol=1e-6)
        # 16-bit params: at most one unit in the last place apart
        assert ulp16_distance(pa, p16).max() <= 1


def test_consts_f32_values(orc):
    c = orc.consts_f32(hp(), 3, 0.25)
    want = [0.9, 0.95, 1 - 0.9, 1 - 0.95, 1 - 1e-4 * 0.1, 1e-4 / (1 - 0.9 ** 3),
            1 / math.sqrt(1 - 0.95 ** 3), 1e-8, 0.25]
    assert np.array_equal(c, np.array(want, dtype=np.float64).astype(np.float32))


# ------------------------------------------------------------ loss-scale machine

def _fp16_grads(n, step, sigma):
    g = synth.normal_16(synth.SEED_GRADS, step, 0, 0, n, 1e-3, torch.float16, "cpu", scale=sigma)
    return synth.as_u16(g).copy()


def test_skipped_step_leaves_state_and_halves_scale(orc):
    n, S = 10_000, 2048
    sc = orc.ScalerCfg(65536.0, 2.0, 0.5, 2000, 1)
    st = orc.new_state(sc)
    p = synth.normal_16(synth.SEED_PARAMS, 0, 0, 0, n, 0.02, torch.float16, "cpu")
    w = p.float().numpy().copy(); m = np.zeros(n, np.float32); v = np.zeros(n, np.float32)
    p16 = synth.as_u16(p).copy()
    h = hp()
    for s in (1, 2):
        r = orc.step(h, sc, st, _fp16_grads(n, s, st.loss_scale), w, m, v, p16, S, orc.FP16)
        assert r.found_inf == 0 and r.loss_scale_used == 65536.0
    snap = [a.copy() for a in (w, m, v, p16)]
    g = _fp16_grads(n, 3, st.loss_scale)
    g[synth.pick_element(synth.SEED_INF, 3, n)] = 0x7C00
    r = orc.step(h, sc, st, g, w, m, v, p16, S, orc.FP16)
    assert r.found_inf == 1 and st.t == 2 and st.loss_scale == 32768.0 and st.good_steps == 0
    for a, b in zip(snap, (w, m, v, p16)):
        assert np.array_equal(a, b)


def test_run_with_a_skip_equals_replay_of_applied_steps(orc):
    # power-of-two loss scales are exact, so 6 steps with step 3 skipped give the same bits
    # as the 5 applied steps run with loss scale 1 on the unscaled gradients
    n, S = 10_000, 2048
    sc = orc.ScalerCfg(65536.0, 2.0, 0.5, 2000, 1)
    h = hp()
    p = synth.normal_16(synth.SEED_PARAMS, 0, 0, 0, n, 0.02, torch.float16, "cpu")

    def init():
        return p.float().numpy().copy(), np.zeros(n, np.float32), np.zeros(n, np.float32), synth.as_u16(p).copy()

    w, m, v, p16 = init()
    st = orc.new_state(sc)
    applied = []
    for s in range(1, 7):
        sigma = st.loss_scale
        g = _fp16_grads(n, s, sigma)
        if s == 3:
            g[synth.pick_element(synth.SEED_INF, 3, n)] = 0x7C00
        r = orc.step(h, sc, st, g, w, m, v, p16, S, orc.FP16)
        if not r.found_inf:
            applied.append((g, sigma))
    assert st.t == 5 and st.loss_scale == 32768.0 and len(applied) == 5
    w2, m2, v2, p2 = init()
    st2 = orc.new_state(None)
    for g, sigma in applied:
        # the same gradient values, unscaled exactly in fp32 (values stay fp32 here, so the
        # replay feeds them through grad_mult rather than re-rounding them to fp16)
        rep = O.Report()
        sq = orc.sqnorm(g, orc.FP16, loss_scale=sigma, block=S)
        gm = orc.clip_coef(math.sqrt(sq), 1.0) / sigma
        st2.t += 1
        orc.adamw_f64(h, st2.t, gm, g, w2, m2, v2, p2, orc.FP16)
    for a, b in zip((w, m, v, p16), (w2, m2, v2, p2)):
        assert np.array_equal(a, b)


def test_scale_grows_after_interval_and_never_drops_below_one(orc):
    n, S = 256, 64
    sc = orc.ScalerCfg(4.0, 2.0, 0.5, 3, 1)
    st = orc.new_state(sc)
    w = np.zeros(n, np.float32); m = w.copy(); v = w.copy(); p16 = np.zeros(n, np.uint16)
    g = np.zeros(n, np.uint16)
    scales = []
    for _ in range(7):
        orc.step(hp(), sc, st, g, w, m, v, p16, S, orc.FP16)
        scales.append(st.loss_scale)
    assert scales == [4.0, 4.0, 8.0, 8.0, 8.0, 16.0, 16.0]
    bad = g.copy(); bad[3] = 0xFC00
    for want in (8.0, 4.0, 2.0, 1.0, 1.0):
        orc.step(hp(), sc, st, bad, w, m, v, p16, S, orc.FP16)
        assert st.loss_scale == want and st.good_steps == 0
    assert st.t == 7


def test_resume_from_the_same_bytes_gives_the_same_bits(orc):
    n, S = 5000, 1024
    g16, w, m, v, p16 = fresh(n)
    h = hp()
    st = orc.new_state(None)
    gs = [synth.as_u16(synth.normal_16(synth.SEED_GRADS, s, 0, 0, n, 1e-3, torch.bfloat16, "cpu")).copy()
          for s in range(1, 5)]
    for g in gs[:2]:
        orc.step(h, None, st, g, w, m, v, p16, S, orc.BF16)
    w2, m2, v2, p2 = w.copy(), m.copy(), v.copy(), p16.copy()
    st2 = orc.State(st.t, st.good_steps, st.loss_scale)
    for g in gs[2:]:
        orc.step(h, None, st, g, w, m, v, p16, S, orc.BF16)
        orc.step(h, None, st2, g, w2, m2, v2, p2, S, orc.BF16)
    assert all(np.array_equal(a, b) for a, b in zip((w, m, v, p16), (w2, m2, v2, p2)))


def test_chunk_size_does_not_change_the_update(orc):
    # with the multiplier shared, the update is elementwise: any S gives the same bits
    n = 30_000
    g16, w, m, v, p16 = fresh(n)
    outs = []
    for S in (1024, 4096, 30_000):
        a = [x.copy() for x in (w, m, v, p16)]
        st = orc.new_state(None)
        r = orc.step(hp(), None, st, g16, *a, S, orc.BF16)
        outs.append((r.norm, a))
    assert abs(outs[0][0] - outs[2][0]) <= 1e-12 * outs[2][0]


# ------------------------------------------------------------- weight-decay groups (no-decay mask)

def test_no_decay_mask_closed_form_and_library_pin(orc):
    n, S = 6000, 2048
    g16, w, m, v, p16 = fresh(n, std_g=0.1)
    mask = np.zeros(n, np.uint8)
    mask[100:1100] = 1; mask[4000] = 1; mask[n - 7:] = 1
    w0 = w.astype(np.float64)
    g = orc.decode16(g16, orc.BF16).astype(np.float64) * 0.5
    a = [x.copy() for x in (w, m, v, p16)]
    orc.adamw_f64(hp(), 1, 0.5, g16, *a, orc.BF16, no_decay=mask)
    # step 1 from zero state: decayed elements lose lr*wd*w, masked ones do not
    want = w0 - 1e-4 * g / (np.abs(g) + 1e-8) - np.where(mask, 0.0, 1e-4 * 0.1 * w0)
    assert np.all(np.abs(a[0] - want) <= 0.5 * ulp32(a[0]) * 1.0001 + 1e-17)
    # the fp32 sequence with the mask stays at the fp64 evaluation; without a mask nothing changed
    b = [x.copy() for x in (w, m, v, p16)]
    orc.adamw_f32seq(orc.consts_f32(hp(), 1, 0.5), g16, *b, orc.BF16, no_decay=mask)
    assert np.all(np.abs(b[0].astype(np.float64) - a[0]) <= 2e-7 * (np.abs(w0) + 1e-4))
    c0 = [x.copy() for x in (w, m, v, p16)]; c1 = [x.copy() for x in (w, m, v, p16)]
    orc.adamw_f64(hp(), 1, 0.5, g16, *c0, orc.BF16)
    orc.adamw_f64(hp(), 1, 0.5, g16, *c1, orc.BF16, no_decay=np.zeros(n, np.uint8))
    assert all(np.array_equal(x, y) for x, y in zip(c0, c1))
    # library pin: torch.optim.AdamW with two parameter groups (wd 0.1 / wd 0), clipped together, fp64
    steps = 3
    gs16 = [synth.as_u16(synth.normal_16(synth.SEED_GRADS, s + 1, 0, 0, n, 0.1, torch.bfloat16, "cpu")).copy()
            for s in range(steps)]
    wa, ma, va, pa = w.copy(), m.copy(), v.copy(), p16.copy()
    st = orc.new_state(None)
    trk = ScaleTracker(w, m, HP)
    for s in range(steps):
        r = orc.step(hp(), None, st, gs16[s], wa, ma, va, pa, S, orc.BF16, threads=2, no_decay=mask)
        trk.advance(s + 1, orc.decode16(gs16[s], orc.BF16).astype(np.float64) * r.grad_mult, va)
    idx_d, idx_n = np.flatnonzero(mask == 0), np.flatnonzero(mask)
    pd = torch.nn.Parameter(torch.tensor(w[idx_d], dtype=torch.float64))
    pn = torch.nn.Parameter(torch.tensor(w[idx_n], dtype=torch.float64))
    opt = torch.optim.AdamW([{"params": [pd], "weight_decay": 0.1}, {"params": [pn], "weight_decay": 0.0}],
                            lr=1e-4, betas=(0.9, 0.95), eps=1e-8)
    for s in range(steps):
        gf = orc.decode16(gs16[s], orc.BF16).astype(np.float64)
        pd.grad = torch.tensor(gf[idx_d]); pn.grad = torch.tensor(gf[idx_n])
        torch.nn.utils.clip_grad_norm_([pd, pn], 1.0)
        opt.step()
    wt = np.empty(n); wt[idx_d] = pd.detach().numpy(); wt[idx_n] = pn.detach().numpy()
    assert np.all(np.abs(wa - wt) <= 1e-6 * trk.W)


def test_f32_sequence_is_exact_where_every_operation_is_exact(orc):
    """A case built so that no operation of the fp32 sequence rounds: powers of two for the
    hyper-parameters, gradients of one magnitude equal to eps, small dyadic weights, first step.
    Then the sequence, the fp64 evaluation and exact rational arithmetic must agree bit for bit;
    a dropped, doubled or mis-signed term anywhere in the sequence breaks the equality."""
    from fractions import Fraction as F
    n = 4096
    rng = np.random.default_rng(7)
    h = hp(lr=2.0 ** -10, beta1=0.5, beta2=0.75, eps=2.0 ** -10, weight_decay=0.5, max_norm=0.0)
    gm = 2.0 ** -3
    sign = rng.choice([-1.0, 1.0], n)
    g16 = bf16w(sign * 2.0 ** -7)                                   # g = +-2^-7 * 2^-3 = +-2^-10 = +-eps
    j = rng.integers(-1000, 1001, n)
    w0 = (j * 2.0 ** -6).astype(np.float32)
    states = []
    for fn in ("f64", "f32"):
        w, m, v, p16 = w0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32), np.zeros(n, np.uint16)
        if fn == "f64":
            orc.adamw_f64(h, 1, gm, g16, w, m, v, p16, orc.BF16)
        else:
            c = orc.consts_f32(h, 1, gm)
            # the nine constants themselves are exact here
            assert [F(float(x)) for x in c] == [F(1, 2), F(3, 4), F(1, 2), F(1, 4), 1 - F(1, 2 ** 11), F(1, 2 ** 9), F(2),
                                                F(1, 2 ** 10), F(1, 8)]
            orc.adamw_f32seq(c, g16, w, m, v, p16, orc.BF16)
        states.append((w, m, v, p16))
    for a, b in zip(*states):
        assert a.tobytes() == b.tobytes()
    w, m, v, p16 = states[1]
    for i in range(0, n, 37):                                        # exact rationals, element by element
        g = F(float(sign[i])) * F(1, 2 ** 10)
        assert F(float(m[i])) == g / 2                                # (1 - beta1) g
        assert F(float(v[i])) == g * g / 4                            # (1 - beta2) g^2
        d = abs(g) / 2 * 2 + F(1, 2 ** 10)                            # sqrt(v) / sqrt(1 - beta2) + eps = 2^-9
        want = F(int(j[i]), 64) * (1 - F(1, 2 ** 11)) - F(1, 2 ** 9) * ((g / 2) / d)
        assert F(float(w[i])) == want
    assert np.array_equal(p16, orc.encode16_rne(w, orc.BF16))


# ------------------------------------------------ the fp32 sequence against exact rational arithmetic
# An independent referee for orc_adamw_f32seq in the general case (operations that DO round): every
# operation of the sequence is carried out exactly on rationals and then rounded once to binary32 by a
# value-domain nearest / ties-to-even rule written here (no float type, no C compiler, no libm takes part:
# Python integers and fractions only), the square root through integer square roots with the result
# proven by exact squares of the neighbouring midpoints.

from fractions import Fraction as Fr
from math import isqrt


def _floor_log2(a: Fr) -> int:
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fr(2) ** e > a:
        e -= 1
    if Fr(2) ** (e + 1) <= a:
        e += 1
    assert Fr(2) ** e <= a < Fr(2) ** (e + 1)
    return e


def _quantum(a: Fr, p: int, emin: int) -> Fr:
    """spacing of the format (p significand bits, smallest normal exponent emin) at magnitude a > 0"""
    return Fr(2) ** (max(_floor_log2(a), emin) - (p - 1))


def rn(x: Fr, p: int = 24, emin: int = -126, emax: int = 127) -> Fr:
    """nearest value of the binary format, ties to the even significand; subnormals included"""
    if x == 0:
        return x
    a = abs(x)
    q = _quantum(a, p, emin)
    k = a / q
    n = k.numerator // k.denominator
    r = k - n
    if r > Fr(1, 2) or (r == Fr(1, 2) and n % 2 == 1):
        n += 1
    out = n * q
    assert out < Fr(2) ** (emax + 1), "overflow is not part of these cases"
    return out if x > 0 else -out


def rn_sqrt(x: Fr) -> Fr:
    """correctly rounded binary32 square root of a non-negative rational"""
    if x == 0:
        return x
    K = 160
    y = Fr(isqrt((x.numerator << (2 * K)) // x.denominator), 1 << K)      # floor(sqrt(x) * 2^K) / 2^K
    r = rn(y)
    for cand in (r, r - _quantum(r, 24, -126), r + _quantum(r, 24, -126)):
        if cand <= 0:
            continue
        q = _quantum(cand, 24, -126)
        lo_q = q / 2 if cand == Fr(2) ** _floor_log2(cand) and _floor_log2(cand) > -126 else q
        lo, hi = cand - lo_q / 2, cand + q / 2
        if lo * lo < x < hi * hi:             # a square root of a binary32 value never sits on a midpoint
            return cand
    raise AssertionError("no candidate brackets the square root")


def decode_word(w: int, fbits: int, ebits: int) -> Fr:
    """IEEE definition of a 16-bit word: 1 sign bit, ebits exponent bits, fbits fraction bits"""
    sign = -1 if (w >> 15) & 1 else 1
    E = (w >> fbits) & ((1 << ebits) - 1)
    f = w & ((1 << fbits) - 1)
    bias = (1 << (ebits - 1)) - 1
    assert E != (1 << ebits) - 1, "finite words only"
    if E == 0:
        return sign * Fr(f, 1 << fbits) * Fr(2) ** (1 - bias)
    return sign * (1 + Fr(f, 1 << fbits)) * Fr(2) ** (E - bias)


def word16_of(x: Fr, fp16: bool) -> int:
    """bit pattern of the 16-bit value nearest to x (ties to even), from the value alone"""
    p, emin, fbits, ebits = (11, -14, 10, 5) if fp16 else (8, -126, 7, 8)
    r = rn(x, p, emin, 15 if fp16 else 127)
    if r == 0:
        return 0x8000 if x < 0 else 0
    a = abs(r)
    e = _floor_log2(a)
    bias = (1 << (ebits - 1)) - 1
    if e < emin:
        E, f = 0, a / Fr(2) ** (emin - fbits)
    else:
        E, f = e + bias, (a / Fr(2) ** e - 1) * (1 << fbits)
    assert f.denominator == 1
    return (0x8000 if r < 0 else 0) | (E << fbits) | int(f)


def seq_exact(c, g, w, m, v, decay_on):
    """the fp32 operation sequence, every operation rounded once from its exact result"""
    b1, b2, omb1, omb2, decay, step_size, rsb2, eps, gm = c
    gg = rn(g * gm)
    t1 = rn(omb1 * gg)
    mn = rn(b1 * m + t1)
    t2 = rn(omb2 * gg)
    t2 = rn(t2 * gg)
    vn = rn(b2 * v + t2)
    d = rn(rn_sqrt(vn) * rsb2 + eps)
    u = rn(mn / d)
    t3 = rn(w * (decay if decay_on else 1))
    wn = rn(-step_size * u + t3)
    return wn, mn, vn


@pytest.mark.parametrize("fp16", [False, True])
def test_f32_sequence_against_correctly_rounded_rational_arithmetic(orc, fp16):
    n, steps = 700, 3
    dt, odt = (torch.float16, orc.FP16) if fp16 else (torch.bfloat16, orc.BF16)
    fbits, ebits = (10, 5) if fp16 else (7, 8)
    sigma = 65536.0 if fp16 else 1.0
    h = hp()
    p = synth.normal_16(synth.SEED_PARAMS + 3, 0, 0, 0, n, 0.02, dt, "cpu")
    p16 = synth.as_u16(p).copy()
    w = p.float().numpy().copy()
    m, v = np.zeros(n, np.float32), np.zeros(n, np.float32)
    mask = (np.arange(n) % 5 == 0).astype(np.uint8)                     # every fifth element is not decayed
    W = [Fr(float(x)) for x in w]
    M = [Fr(0)] * n
    V = [Fr(0)] * n
    for t in range(1, steps + 1):
        g = synth.normal_16(synth.SEED_GRADS + 3, t, 0, 0, n, 1e-3, dt, "cpu", scale=sigma)
        g16 = synth.as_u16(g).copy()
        # a few special gradients: zero, the smallest subnormal word, and (bf16) values whose square is subnormal in fp32
        g16[0], g16[1], g16[2] = 0, 1, 0x8001
        if not fp16:
            g16[3:9] = bf16w(np.array([3e-18, -7e-19, 2.5e-20, -1e-21, 6e-17, 1e-30], np.float32))
        gm = 0.0123 / sigma * (1.0 + 0.1 * t)
        c = orc.consts_f32(h, t, gm)
        cF = [Fr(float(x)) for x in c]
        orc.adamw_f32seq(c, g16, w, m, v, p16, odt, threads=2, no_decay=mask)
        for i in range(n):
            W[i], M[i], V[i] = seq_exact(cF, decode_word(int(g16[i]), fbits, ebits), W[i], M[i], V[i], not mask[i])
        assert [Fr(float(x)) for x in w] == W, f"master weights, step {t}"
        assert [Fr(float(x)) for x in m] == M, f"momentum, step {t}"
        assert [Fr(float(x)) for x in v] == V, f"variance, step {t}"
        assert [int(x) for x in p16] == [word16_of(x, fp16) for x in W], f"16-bit parameters, step {t}"
    if not fp16:
        assert any(0 < x < Fr(2) ** -126 for x in V), "the case must reach subnormal variances"


def test_f32_sequence_on_fp32_gradients_against_rational_arithmetic(orc):
    """the same referee for the fp32-gradient variant: gradients that no 16-bit word holds"""
    n = 400
    rng = np.random.default_rng(11)
    g32 = (rng.standard_normal(n) * 4e-3).astype(np.float32)
    g32[:4] = [0.0, 1e-30, -3e-39, 1.5e-19]                              # zero, tiny, subnormal, subnormal square
    w = (rng.standard_normal(n) * 0.02).astype(np.float32)
    m = (rng.standard_normal(n) * 1e-5).astype(np.float32)
    v = (rng.random(n) * 1e-10).astype(np.float32)
    p16 = np.zeros(n, np.uint16)
    c = orc.consts_f32(hp(), 7, 0.0371)
    cF = [Fr(float(x)) for x in c]
    want = [seq_exact(cF, Fr(float(g32[i])), Fr(float(w[i])), Fr(float(m[i])), Fr(float(v[i])), True) for i in range(n)]
    orc.adamw_f32seq_g32(c, g32, w, m, v, p16, orc.BF16, threads=1)
    assert [Fr(float(x)) for x in w] == [x[0] for x in want]
    assert [Fr(float(x)) for x in m] == [x[1] for x in want]
    assert [Fr(float(x)) for x in v] == [x[2] for x in want]
    assert [int(x) for x in p16] == [word16_of(x[0], False) for x in want]


def test_the_rational_referee_itself():
    """rn / rn_sqrt / word16_of on values whose rounding is known by hand"""
    assert rn(Fr(1) + Fr(1, 2 ** 24)) == 1                               # tie -> even
    assert rn(Fr(1) + Fr(3, 2 ** 24)) == 1 + Fr(1, 2 ** 22)              # tie -> even (upwards)
    assert rn(Fr(1) + Fr(1, 2 ** 24) + Fr(1, 2 ** 60)) == 1 + Fr(1, 2 ** 23)
    assert rn(Fr(3, 2 ** 151)) == Fr(1, 2 ** 149)                        # 0.75 of the smallest subnormal
    assert rn(Fr(1, 2 ** 150)) == 0 and rn(Fr(3, 2 ** 150)) == Fr(2, 2 ** 149)   # subnormal ties -> even
    assert rn_sqrt(Fr(4)) == 2 and rn_sqrt(Fr(2)) == Fr(11863283, 2 ** 23)        # 1.41421354...
    assert rn_sqrt(Fr(1, 2 ** 149)) == rn(Fr(isqrt(2 << 300), 1 << 150) * Fr(1, 2 ** 75))
    assert word16_of(Fr(1) + Fr(1, 256), False) == 0x3F80                # bf16 tie -> even
    assert word16_of(Fr(1) + Fr(3, 256), False) == 0x3F82
    assert word16_of(Fr(1, 2 ** 24), True) == 0x0001 and word16_of(Fr(-1, 2 ** 25), True) == 0x8000
    assert word16_of(Fr(65504), True) == 0x7BFF
