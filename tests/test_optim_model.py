"""The OPTIM-phase cost model and n_persist chooser (paper, Appendix A.1 Eq. 2 restricted to the
optimizer phase; Appendix A.2 model-state memory term): library against the plain-Python oracle,
and the oracle against closed forms."""
import random

import pytest

from oracle import optim_model as OM
from paper_2406_08334_amd import binding as B

RATES = dict(gpu_s_fixed=2e-5, gpu_s_per_elem=5.1e-12, link_s_fixed=4e-3, link_s_per_elem=3.1e-10,
             host_s_fixed=1e-4, host_s_per_elem=7.3e-11, stream_contention=0.5, gpu_serial_share=0.0)
S, C = 1 << 26, 194


def lib_rates(r):
    return B.pt_optim_rates(*[r[k] for k in ("gpu_s_fixed", "gpu_s_per_elem", "link_s_fixed", "link_s_per_elem",
                                              "host_s_fixed", "host_s_per_elem", "stream_contention", "gpu_serial_share")])


def test_oracle_closed_forms():
    # everything resident: only the GPU part; nothing resident: only the other part
    assert OM.predict(RATES, S, C, C, OM.HOST) == (2e-5 + 5.1e-12 * S * C, 0.0, 2e-5 + 5.1e-12 * S * C)
    assert OM.predict(RATES, S, C, 0, OM.STREAM)[2] == 4e-3 + 3.1e-10 * S * C
    # host mode is a plain max; streamed mode adds the contention share of the shorter part
    tg, to, t = OM.predict(RATES, S, C, 100, OM.HOST)
    assert t == max(tg, to)
    tg, to, t = OM.predict(RATES, S, C, 100, OM.STREAM)
    assert t == max(tg, to) + 0.5 * min(tg, to)
    # the part of the resident work that comes before the norm (share s) is served first, the rest runs beside
    # the other part: host part longer -> s*tg + to; resident part longer -> tg; s = 0 -> the plain max
    for s_ in (0.0, 0.125, 0.5, 1.0):
        r = dict(RATES, gpu_serial_share=s_)
        tg, to, t = OM.predict(r, S, C, 100, OM.HOST)                 # 100 resident, 94 on the host: host part longer
        assert to > tg and t == s_ * tg + to
        tg, to, t = OM.predict(r, S, C, 190, OM.HOST)                 # 4 on the host: resident part longer ...
        assert tg > to
        if (1 - s_) * tg > to:
            assert abs(t - tg) <= 1e-18                               # ... and still longer without its serial share
        else:
            assert abs(t - (s_ * tg + to)) <= 1e-18
        assert OM.predict(r, S, C, C, OM.HOST)[2] == OM.predict(RATES, S, C, C, OM.HOST)[2]    # all resident: no share
        assert OM.predict(r, S, C, 0, OM.STREAM)[2] == OM.predict(RATES, S, C, 0, OM.STREAM)[2]  # nothing resident
        tg, to, t = OM.predict(r, S, C, 100, OM.STREAM)
        assert abs(t - (s_ * tg + max((1 - s_) * tg, to) + 0.5 * min((1 - s_) * tg, to))) <= 1e-15
    prev = 0.0
    for s_ in (0.0, 0.1, 0.3, 0.9):                                   # more serial work never makes a step shorter
        t = OM.predict(dict(RATES, gpu_serial_share=s_), S, C, 150, OM.HOST)[2]
        assert t >= prev
        prev = t
    # balanced point with a serial share: (1-s) * gpu rate * resident elements = host rate * host elements
    r = dict(RATES, gpu_s_fixed=0.0, host_s_fixed=0.0, gpu_serial_share=0.25)
    n, t, need, buffers = OM.choose(r, S, 1000, 1 << 62, OM.HOST, 0)
    g_, h_ = 0.75 * r["gpu_s_per_elem"], r["host_s_per_elem"]
    assert abs((1000 - n) / 1000 - g_ / (g_ + h_)) <= 2e-3
    # balanced point of the host mode: with zero fixed costs the best split makes both parts equal,
    # n*/C = host rate / (host rate + gpu rate) of the ELEMENTS go to the host
    r = dict(RATES, gpu_s_fixed=0.0, host_s_fixed=0.0)
    n, t, need, buffers = OM.choose(r, S, 1000, 1 << 62, OM.HOST, 0)
    frac_host = r["gpu_s_per_elem"] / (r["gpu_s_per_elem"] + r["host_s_per_elem"])
    assert abs((1000 - n) / 1000 - frac_host) <= 1e-3 and buffers == 0
    assert t <= OM.predict(r, S, 1000, 1000, OM.HOST)[2]          # never worse than all-resident
    # streamed mode with a slow link: as many resident chunks as the budget holds, buffers counted
    budget = 16 * S * (50 + 3)
    n, t, need, buffers = OM.choose(RATES, S, C, budget, OM.STREAM, 3)
    assert (n, buffers, need) == (50, 3, budget)
    n, t, need, buffers = OM.choose(RATES, S, C, 16 * S * C, OM.STREAM, 3)
    assert (n, buffers) == (C, 0)                                  # all resident needs no buffers
    assert OM.choose(RATES, S, C, 16 * S * 2, OM.STREAM, 3) is None


def test_library_matches_the_oracle():
    rng = random.Random(4)
    for _ in range(300):
        r = {k: v * rng.uniform(0.2, 5.0) for k, v in RATES.items()}
        r["stream_contention"] = rng.uniform(0.0, 1.0)
        r["gpu_serial_share"] = rng.choice([0.0, 1.0, rng.uniform(0.0, 1.0)])
        s = 8 * rng.randint(1, 1 << 20)
        c = rng.randint(1, 300)
        mode = rng.choice([OM.STREAM, OM.HOST])
        n = rng.randint(0, c)
        got = B.pt_optim_predict(lib_rates(r), s, c, n, mode)
        want = OM.predict(r, s, c, n, mode)
        assert all(abs(a - b) <= 1e-12 * max(abs(b), 1e-30) for a, b in zip(got, want))
        slots = rng.randint(2, 8)
        budget = 16 * s * rng.randint(0, c + 10)
        want = OM.choose(r, s, c, budget, mode, slots)
        if want is None:
            with pytest.raises(B.PtError):
                B.pt_optim_choose(lib_rates(r), s, c, budget, mode, slots)
            continue
        ch = B.pt_optim_choose(lib_rates(r), s, c, budget, mode, slots)
        assert (ch.n_persist, ch.hbm_bytes, ch.n_slots) == (want[0], want[2], want[3])
        assert abs(ch.t_step - want[1]) <= 1e-12 * want[1]
    neg = dict(RATES, gpu_s_fixed=-1.0)                            # a fitted intercept below zero never gives a negative time
    assert B.pt_optim_predict(lib_rates(neg), S, C, 1, OM.HOST)[0] == 0.0 == OM.predict(neg, S, C, 1, OM.HOST)[0]
    for bad in (-0.1, 1.5, float("nan")):
        with pytest.raises(B.PtError):
            B.pt_optim_predict(lib_rates(dict(RATES, gpu_serial_share=bad)), S, C, 1, OM.HOST)
    with pytest.raises(B.PtError):
        B.pt_optim_predict(lib_rates(RATES), S, C, C + 1, OM.HOST)
    with pytest.raises(B.PtError):
        B.pt_optim_choose(lib_rates(RATES), S, C, 1 << 40, 7, 3)
