"""Pins for the oracle's 16-bit conversions (bf16 / fp16, round-to-nearest-even).

The method stores parameters and gradients in a 16-bit format and updates in
fp32 (paper, Background: mixed-precision training); the recast is RNE.
Pins: library conversions (numpy float16, torch bfloat16/float16) on all 2^16
patterns and on random fp32 inputs; the value-domain nearest/ties-even definition
(tests/pins/nearest16.c) on ALL 2^32 fp32 inputs; explicit tie cases.
"""
import ctypes as C
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def pinlib(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("pins") / "libnearest16.so")
    subprocess.run(["gcc", "-O2", "-fPIC", "-shared", "-o", out,
                    os.path.join(HERE, "pins", "nearest16.c"), "-lm"], check=True)
    L = C.CDLL(out)
    L.pin_count_mismatch.restype = C.c_uint64
    L.pin_count_mismatch.argtypes = [C.POINTER(C.c_float), C.POINTER(C.c_float), C.c_uint64, C.c_int]
    return L


def test_decode_all_patterns_against_libraries(orc):
    words = np.arange(1 << 16, dtype=np.uint16)
    # fp16: numpy's own binary16
    got = orc.decode16(words, orc.FP16)
    want = words.view(np.float16).astype(np.float32)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    # bf16: torch's bfloat16
    got = orc.decode16(words, orc.BF16)
    want = torch.from_numpy(words.view(np.int16)).view(torch.bfloat16).float().numpy()
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got.view(np.uint32)[~nan], want.view(np.uint32)[~nan])


def test_every_16bit_pattern_survives_a_round_trip(orc):
    words = np.arange(1 << 16, dtype=np.uint16)
    for dt, expmask in ((orc.BF16, 0x7F80), (orc.FP16, 0x7C00)):
        back = orc.encode16_rne(orc.decode16(words, dt), dt)
        frac = words & np.uint16(~np.uint16(expmask | 0x8000) & 0xFFFF)
        nan = ((words & expmask) == expmask) & (frac != 0)
        assert np.array_equal(back[~nan], words[~nan])
        # NaN stays NaN (quieted), sign kept
        bnan = ((back & expmask) == expmask) & ((back & np.uint16(~np.uint16(expmask | 0x8000) & 0xFFFF)) != 0)
        assert np.array_equal(bnan, nan)
        assert np.array_equal(back[nan] & 0x8000, words[nan] & 0x8000)


def test_encode_matches_library_conversions_on_random_bits(orc):
    rng = np.random.default_rng(7)
    bits = rng.integers(0, 1 << 32, size=4_000_000, dtype=np.uint64).astype(np.uint32)
    x = bits.view(np.float32)
    finite = np.isfinite(x)
    with np.errstate(over="ignore"):
        want16 = x.astype(np.float16).view(np.uint16)
    got16 = orc.encode16_rne(x, orc.FP16)
    assert np.array_equal(got16[finite], want16[finite])
    wantbf = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    gotbf = orc.encode16_rne(x, orc.BF16)
    assert np.array_equal(gotbf[finite], wantbf[finite])


def test_explicit_ties_round_to_even(orc):
    def f(bits):
        return np.array([bits], dtype=np.uint32).view(np.float32)
    # bf16: 1.0 + 2^-8 is halfway between 0x3F80 and 0x3F81 -> even 0x3F80
    assert orc.encode16_rne(f(0x3F808000), orc.BF16)[0] == 0x3F80
    # 1.0 + 3*2^-8 is halfway between 0x3F81 and 0x3F82 -> even 0x3F82
    assert orc.encode16_rne(f(0x3F818000), orc.BF16)[0] == 0x3F82
    assert orc.encode16_rne(f(0x3F808001), orc.BF16)[0] == 0x3F81
    # largest finite fp32 overflows to +inf in bf16
    assert orc.encode16_rne(f(0x7F7FFFFF), orc.BF16)[0] == 0x7F80
    # fp16: 1 + 2^-11 tie -> 0x3C00 ; 1 + 3*2^-11 tie -> 0x3C02
    assert orc.encode16_rne(np.array([1 + 2.0 ** -11], np.float32), orc.FP16)[0] == 0x3C00
    assert orc.encode16_rne(np.array([1 + 3 * 2.0 ** -11], np.float32), orc.FP16)[0] == 0x3C02
    # 65520 is the tie between 65504 and 2^16 -> inf ; just below stays 65504
    assert orc.encode16_rne(np.array([65520.0], np.float32), orc.FP16)[0] == 0x7C00
    assert orc.encode16_rne(np.array([65519.996], np.float32), orc.FP16)[0] == 0x7BFF
    # 2^-25 is the tie between 0 and the smallest subnormal -> 0 ; above it -> 1
    assert orc.encode16_rne(np.array([2.0 ** -25], np.float32), orc.FP16)[0] == 0x0000
    assert orc.encode16_rne(np.array([2.0 ** -25 * 1.0001], np.float32), orc.FP16)[0] == 0x0001
    assert orc.encode16_rne(np.array([-0.0], np.float32), orc.FP16)[0] == 0x8000


@pytest.mark.parametrize("dt", [0, 1])
def test_encode_is_nearest_even_for_all_2pow32_inputs(orc, pinlib, dt):
    block = 1 << 24

    def run(b):
        bits = np.arange(b * block, (b + 1) * block, dtype=np.uint64).astype(np.uint32)
        x = bits.view(np.float32)
        back = orc.decode16(orc.encode16_rne(x, dt), dt)
        return int(pinlib.pin_count_mismatch(x.ctypes.data_as(C.POINTER(C.c_float)),
                                             back.ctypes.data_as(C.POINTER(C.c_float)), x.size, dt))

    with ThreadPoolExecutor(max_workers=8) as ex:
        bad = sum(ex.map(run, range(256)))
    assert bad == 0
