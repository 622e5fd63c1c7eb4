"""Pins for the oracle's fp32 gradient-accumulation variant (micro-batches summed into an
fp32 array of the chunk layout; norm, clipping and update read that array).

Pinned against what the arithmetic fixes: numpy's float32 addition and Python's exact
rationals for the accumulation, math.fsum for the norm, the already pinned 16-bit-gradient
update where the two must coincide, a closed form where they must not, and
torch.optim.AdamW + clip_grad_norm_ in fp64 on fp32 gradients.
"""
import math
from fractions import Fraction

import numpy as np
import torch

import oracle as O
from paper_2406_08334_amd import synth

HP = dict(lr=1e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, max_norm=1.0)


def hp(**kw):
    d = dict(HP); d.update(kw)
    return O.Hparams(**d)


def words(seed, n, dtype):
    """random 16-bit patterns: every exponent, both signs, NaNs and infinities included"""
    return np.random.default_rng(seed).integers(0, 1 << 16, n, dtype=np.uint16)


def draws(seed, step, n, std, dtype=torch.bfloat16):
    return synth.as_u16(synth.normal_16(synth.SEED_GRADS + seed, step, 0, 0, n, std, dtype, "cpu")).copy()


def test_accumulation_is_float32_addition_of_the_decoded_words(orc):
    for dtype in (orc.BF16, orc.FP16):
        a, b, c = (words(s, 70_000, dtype) for s in (1, 2, 3))
        acc = np.full(a.size, 7.0, np.float32)
        orc.accum_f32(a, acc, dtype, overwrite=True)              # the old content is gone
        da, db, dc = (orc.decode16(x, dtype) for x in (a, b, c))
        assert acc.tobytes() == da.tobytes()
        orc.accum_f32(b, acc, dtype)
        orc.accum_f32(c, acc, dtype)
        with np.errstate(invalid="ignore", over="ignore"):
            want = (da + db) + dc                                  # numpy float32: IEEE single additions
        same = (acc.view(np.uint32) == want.view(np.uint32)) | (np.isnan(acc) & np.isnan(want))
        assert same.all()


def test_accumulation_rounds_the_exact_sum_once(orc):
    """brute force with exact rationals: each addition is the exact sum rounded to nearest even"""
    rng = np.random.default_rng(5)
    a = rng.integers(0, 1 << 16, 400, dtype=np.uint16)
    b = rng.integers(0, 1 << 16, 400, dtype=np.uint16)
    for dtype in (orc.BF16, orc.FP16):
        da, db = orc.decode16(a, dtype), orc.decode16(b, dtype)
        acc = da.copy()
        orc.accum_f32(b, acc, dtype)
        for x, y, got in zip(da, db, acc):
            if not (math.isfinite(x) and math.isfinite(y)):
                assert not math.isfinite(got)                      # inf and NaN never turn finite
                continue
            exact = Fraction(float(x)) + Fraction(float(y))
            if not math.isfinite(got):
                assert abs(exact) >= Fraction(2) ** 128 - Fraction(2) ** 103      # overflow threshold of binary32
                continue
            g = Fraction(float(got))
            lo, hi = np.nextafter(got, np.float32(-np.inf)), np.nextafter(got, np.float32(np.inf))
            for nb in (lo, hi):
                if math.isfinite(nb):
                    assert abs(exact - g) <= abs(exact - Fraction(float(nb)))      # no neighbour is nearer


def test_opposite_infinities_and_nan_are_found(orc):
    acc = np.zeros(8, np.float32)
    a = np.zeros(8, np.uint16); b = np.zeros(8, np.uint16)
    a[2], b[2] = 0x7F80, 0xFF80                                   # +inf then -inf (bf16) -> NaN
    a[5] = 0x7F80                                                 # +inf stays
    orc.accum_f32(a, acc, orc.BF16, overwrite=True)
    orc.accum_f32(b, acc, orc.BF16)
    assert math.isnan(acc[2]) and math.isinf(acc[5]) and orc.found_nonfinite_f32(acc)
    assert not orc.found_nonfinite_f32(np.array([0.0, -0.0, 1e-45, 3.4e38], np.float32))
    for bad in (np.inf, -np.inf, np.nan):
        x = np.zeros(1000, np.float32); x[999] = bad
        assert orc.found_nonfinite_f32(x)


def test_sqnorm_f32_against_fsum_and_closed_forms(orc):
    rng = np.random.default_rng(11)
    g = (rng.standard_normal(100_003) * 1e-3).astype(np.float32)
    for sigma in (1.0, 65536.0):
        want = math.fsum((float(x) / sigma) ** 2 for x in g)
        for block, threads in ((0, 1), (4096, 1), (4096, 5), (100_003, 3)):
            got = orc.sqnorm_f32(g, loss_scale=sigma, block=block, threads=threads)
            assert abs(got - want) <= 1e-12 * want
    assert orc.sqnorm_f32(np.ones(1 << 22, np.float32)) == float(1 << 22)
    assert orc.sqnorm_f32(np.zeros(100, np.float32)) == 0.0
    one = np.zeros(77, np.float32); one[33] = -3.0
    assert orc.sqnorm_f32(one) == 9.0
    assert orc.sqnorm_f32(g * np.float32(8.0), block=4096) == 64.0 * orc.sqnorm_f32(g, block=4096)
    # thread count never changes the bits
    assert orc.sqnorm_f32(g, block=1000, threads=1) == orc.sqnorm_f32(g, block=1000, threads=7)
    # a value that 16 bits cannot hold really enters with all its bits
    x = np.array([1.0 + 2.0 ** -20], np.float32)
    assert orc.sqnorm_f32(x) == (1.0 + 2.0 ** -20) ** 2


def _state(n, seed=0):
    p = synth.normal_16(synth.SEED_PARAMS + seed, 0, 0, 0, n, 0.02, torch.bfloat16, "cpu")
    return p.float().numpy().copy(), np.zeros(n, np.float32), np.zeros(n, np.float32), synth.as_u16(p).copy()


def test_update_from_fp32_gradients_equals_the_16_bit_update_on_decoded_words(orc):
    """where the fp32 gradient IS a decoded 16-bit word the two entry points must give the same bits"""
    n = 30_000
    for dtype, tdt in ((orc.BF16, torch.bfloat16), (orc.FP16, torch.float16)):
        g16 = draws(0, 1, n, 1e-3, tdt)
        g32 = orc.decode16(g16, dtype)
        nd = (np.arange(n) % 7 == 0).astype(np.uint8)
        a, b = _state(n), _state(n)
        orc.adamw_f64(hp(), 3, 0.37, g16, *a, dtype, no_decay=nd)
        orc.adamw_f64_g32(hp(), 3, 0.37, g32, *b, dtype, no_decay=nd)
        for x, y in zip(a, b):
            assert x.tobytes() == y.tobytes()
        c = orc.consts_f32(hp(), 3, 0.37)
        a, b = _state(n), _state(n)
        orc.adamw_f32seq(c, g16, *a, dtype, no_decay=nd)
        orc.adamw_f32seq_g32(c, g32, *b, dtype, no_decay=nd)
        for x, y in zip(a, b):
            assert x.tobytes() == y.tobytes()
        # whole step, with the norm and clipping in it
        a, b = _state(n), _state(n)
        sa, sb = orc.new_state(None), orc.new_state(None)
        ra = orc.step(hp(), None, sa, g16, *a, 4096, dtype)
        rb = orc.step_g32(hp(), None, sb, g32, *b, 4096, dtype)
        assert (ra.sqnorm, ra.norm, ra.clip_coef, ra.grad_mult, ra.found_inf) == \
               (rb.sqnorm, rb.norm, rb.clip_coef, rb.grad_mult, rb.found_inf) and sa.t == sb.t == 1
        for x, y in zip(a, b):
            assert x.tobytes() == y.tobytes()


def test_first_step_closed_form_with_gradients_no_16_bit_word_holds(orc):
    n = 4000
    rng = np.random.default_rng(3)
    g32 = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    assert not np.array_equal(orc.decode16(orc.encode16_rne(g32, orc.BF16), orc.BF16), g32)
    w, m, v, p16 = _state(n)
    w0 = w.astype(np.float64)
    gm = 0.0123
    g = g32.astype(np.float64) * gm
    orc.adamw_f64_g32(hp(), 1, gm, g32, w, m, v, p16, orc.BF16)
    ulp = lambda x: np.spacing(np.abs(x).astype(np.float32)).astype(np.float64)
    assert np.all(np.abs(m - 0.1 * g) <= 0.5 * ulp(m) * 1.0001)
    assert np.all(np.abs(v - (1 - 0.95) * g * g) <= 0.5 * ulp(v) * 1.0001)
    want = w0 - 1e-4 * g / (np.abs(g) + 1e-8) - 1e-4 * 0.1 * w0
    assert np.all(np.abs(w - want) <= 0.5 * ulp(w) * 1.0001 + 1e-17)
    assert np.array_equal(p16, orc.encode16_rne(w, orc.BF16))


def test_three_accumulated_steps_against_torch_adamw_in_fp64(orc):
    """library pin: micro-batches accumulated in fp32, clipped by the global norm, AdamW"""
    n, S, K = 20_000, 4096, 3
    w, m, v, p16 = _state(n)
    ost = orc.new_state(None)
    p = torch.nn.Parameter(torch.tensor(w, dtype=torch.float64))
    opt = torch.optim.AdamW([p], lr=HP["lr"], betas=(HP["beta1"], HP["beta2"]), eps=HP["eps"],
                            weight_decay=HP["weight_decay"])
    for step in (1, 2, 3):
        acc = np.zeros(n, np.float32)
        for k in range(K):
            orc.accum_f32(draws(step, k, n, 1.0), acc, orc.BF16, overwrite=(k == 0))
        assert np.abs(acc).max() > 3.0                              # really a sum of three draws
        rep = orc.step_g32(hp(), None, ost, acc, w, m, v, p16, S, orc.BF16)
        p.grad = torch.tensor(acc, dtype=torch.float64)
        norm = torch.nn.utils.clip_grad_norm_([p], HP["max_norm"])
        assert abs(rep.norm - float(norm)) <= 1e-12 * float(norm) and rep.clip_coef < 0.01
        opt.step()
        ref = p.detach().numpy()
        # the oracle rounds its fp64 result to fp32 once per step; torch keeps fp64 throughout
        assert np.abs(w - ref).max() <= step * 2.0 ** -24 * np.abs(ref).max() * 1.01
    assert ost.t == 3


def test_skipped_step_on_accumulated_nonfinite_leaves_state(orc):
    n = 3000
    w, m, v, p16 = _state(n)
    before = [x.copy() for x in (w, m, v, p16)]
    sc = orc.ScalerCfg(65536.0, 2.0, 0.5, 2000, 1)
    ost = orc.new_state(sc)
    acc = (np.random.default_rng(0).standard_normal(n)).astype(np.float32)
    acc[1234] = np.inf
    rep = orc.step_g32(hp(), sc, ost, acc, w, m, v, p16, 1024, orc.BF16)
    assert rep.found_inf == 1 and ost.t == 0 and ost.loss_scale == 32768.0
    for x, y in zip((w, m, v, p16), before):
        assert x.tobytes() == y.tobytes()
