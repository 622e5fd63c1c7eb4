"""Scale-aware reading of "relative 1e-6" for the fp32 state arrays.

m, v and w are sums of terms; where terms of opposite sign cancel, the plain
relative error of a correctly computed fp32 value is unbounded.  The tolerance is
therefore applied against the accumulated MAGNITUDE of the terms that formed the
value, tracked in fp64 beside the trajectory:

  A_t = beta1 A_{t-1} + (1-beta1) |g_t|          (scale of m;  A_0 = |m_0|)
  v itself                                        (scale of v: all terms >= 0)
  W_t = W_{t-1} (1 - lr wd) + step_t A_t / d_t    (scale of w;  W_0 = |w_0|)

with g_t the clipped, unscaled gradient, step_t = lr/(1-beta1^t) and
d_t = sqrt(v_t)/sqrt(1-beta2^t) + eps.  Away from cancellation A = |m| and
W ~ |w|, i.e. this is the plain relative error.
"""
import os

import numpy as np


class ScaleTracker:
    def __init__(self, w0, m0, hp):
        self.A = np.abs(np.asarray(m0, dtype=np.float64))
        self.W = np.abs(np.asarray(w0, dtype=np.float64))
        self.hp = hp

    def advance(self, t, g_eff, v_new):
        """g_eff: fp64 clipped+unscaled gradient of update t; v_new: v after update t."""
        hp = self.hp
        self.A = hp["beta1"] * self.A + (1.0 - hp["beta1"]) * np.abs(g_eff)
        step = hp["lr"] / (1.0 - hp["beta1"] ** t)
        d = np.sqrt(np.asarray(v_new, dtype=np.float64)) / np.sqrt(1.0 - hp["beta2"] ** t) + hp["eps"]
        self.W = self.W * (1.0 - hp["lr"] * hp["weight_decay"]) + step * self.A / d

    def check(self, got, want, tol=1e-6):
        """got/want: (w, m, v) triples.  Returns the worst error/scale ratio per array."""
        out = {}
        for name, a, b, scale in (("w", got[0], want[0], self.W), ("m", got[1], want[1], self.A),
                                  ("v", got[2], want[2], np.abs(np.asarray(want[2], dtype=np.float64)))):
            err = np.abs(np.asarray(a, dtype=np.float64) - np.asarray(b, dtype=np.float64))
            bad = err > tol * scale
            ratio = float(np.max(err / np.maximum(scale, 1e-300))) if err.size else 0.0
            out[name] = ratio
            assert not bad.any(), f"{name}: {int(bad.sum())} elements beyond {tol} x scale (worst {ratio:.3e})"
        return out


def ulp16_distance(a, b):
    """Distance in units in the last place between two arrays of 16-bit sign-magnitude patterns."""
    def order(x):
        x = np.asarray(x, dtype=np.uint16).astype(np.int32)
        return np.where(x & 0x8000, -(x & 0x7FFF), x & 0x7FFF)
    return np.abs(order(a) - order(b))


def ulp16(x, fp16: bool):
    """Spacing of the 16-bit format at magnitude |x| (bf16: 8 significand bits; fp16: 11, emin -14)."""
    ax = np.abs(np.asarray(x, dtype=np.float64))
    _, e = np.frexp(np.where(ax > 0, ax, 1.0))
    e = e - 1
    if fp16:
        return np.ldexp(1.0, np.maximum(e, -14) - 10)
    return np.ldexp(1.0, np.maximum(e, -126) - 7)


def check_p16(got_p_val, want_p_val, want_w, W, fp16: bool, tol=1e-6):
    """16-bit parameters: "within one ulp" read in the value domain as
    |p_got - p_want| <= ulp16(w) + tol * W: both sides round their own fp32 master weight
    (half an ulp each) and the master weights themselves may differ by tol * W (see
    ScaleTracker).  Away from cancellation in w this is the plain one-ulp bar.
    Returns the number of elements whose patterns differ by more than one ulp."""
    gp = np.asarray(got_p_val, dtype=np.float64)
    wp = np.asarray(want_p_val, dtype=np.float64)
    d = np.abs(gp - wp)
    u = ulp16(want_w, fp16)
    bad = d > u * 1.0000001 + tol * W
    assert not bad.any(), f"p16: {int(bad.sum())} elements beyond ulp16 + {tol} x scale"
    far = int((d > u * 1.0000001).sum())
    log = os.environ.get("PT_P16_LOG")           # a run that wants the counts on record names a file
    if log:
        with open(log, "a") as f:
            f.write(f"{far} of {d.size} elements beyond a plain one-ulp distance ({far / max(d.size, 1):.3e})\n")
    return far


def far_cap(n: int) -> int:
    """How many of n elements may lie beyond a plain one-ulp distance of the oracle's 16-bit parameter (while
    still inside ulp16 + tol * W): they are the elements where the two terms of w cancel.  Seen on the GPU: at
    most 1.4e-7 of the elements (6 of 2^26, 1 of 7.3 M); the cap is ten times that, and at least 2 elements."""
    return max(2, int(2e-6 * n))
