"""The oracle reproduces its stored tiny run bit for bit (tests/golden/adamw_tiny_bf16.txt,
written by tests/golden/make_golden.py from the oracle alone)."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "adamw_tiny_bf16.txt")


def load_golden():
    rec = {}
    with open(GOLDEN) as f:
        for line in f:
            if line.startswith("#"):
                continue
            k, hx = line.split()
            rec[k] = bytes.fromhex(hx)
    return rec


def test_oracle_reproduces_golden(orc):
    rec = load_golden()
    p16 = np.frombuffer(rec["p16_0"], dtype=np.uint16).copy()
    n, S = p16.size, 16
    w = orc.decode16(p16, orc.BF16).copy()
    m = np.zeros(n, np.float32); v = np.zeros(n, np.float32)
    hp = orc.Hparams(1e-4, 0.9, 0.95, 1e-8, 0.1, 1.0)
    st = orc.new_state(None)
    for s in (1, 2, 3):
        g = np.frombuffer(rec[f"g16_{s}"], dtype=np.uint16).copy()
        rep = orc.step(hp, None, st, g, w, m, v, p16, S, orc.BF16)
        assert np.float64(rep.norm).tobytes() == rec[f"norm_{s}"]
    assert w.tobytes() == rec["w_final"] and m.tobytes() == rec["m_final"]
    assert v.tobytes() == rec["v_final"] and p16.tobytes() == rec["p16_final"]
    assert not w[-3:].any() and not p16[-3:].any()      # padding stayed zero
