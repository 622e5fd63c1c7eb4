"""Writes tests/golden/adamw_tiny_bf16.txt: a 40-element, 3-step bf16 run of the CPU oracle.

Calls only oracle/ (numpy's seeded generator supplies the input bits, which are
stored in the file, so the fixture does not depend on any generator afterwards).
The expected values are the oracle's own: the fixture guards the oracle against
drifting between machines/compilers and gives the GPU tests a tiny fixed case.
Hyper-parameters: lr 1e-4, betas (0.9, 0.95), eps 1e-8, wd 0.1, clip 1.0 (the
AdamW setting of the benchmark configurations).

Run from the repository root:  python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
import oracle as O  # noqa: E402

N, S, STEPS = 40, 16, 3


def main():
    rng = np.random.default_rng(20240608)
    p16 = O.encode16_rne(rng.normal(0, 0.02, N).astype(np.float32), O.BF16)
    p16[N - 3:] = 0                                      # stands for chunk padding
    w = O.decode16(p16, O.BF16).copy()
    m = np.zeros(N, np.float32)
    v = np.zeros(N, np.float32)
    grads = [O.encode16_rne(rng.normal(0, 0.3, N).astype(np.float32), O.BF16) for _ in range(STEPS)]
    for g in grads:
        g[N - 3:] = 0
    hp = O.Hparams(1e-4, 0.9, 0.95, 1e-8, 0.1, 1.0)
    st = O.new_state(None)
    lines = [f"# n={N} chunk_elems={S} steps={STEPS} dtype=bf16 ; hex words, one array per line",
             "p16_0 " + p16.tobytes().hex()]
    for s, g in enumerate(grads):
        rep = O.step(hp, None, st, g, w, m, v, p16, S, O.BF16)
        lines.append(f"g16_{s + 1} " + g.tobytes().hex())
        lines.append(f"norm_{s + 1} " + np.float64(rep.norm).tobytes().hex())
    for name, a in (("w", w), ("m", m), ("v", v), ("p16", p16)):
        lines.append(f"{name}_final " + a.tobytes().hex())
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "adamw_tiny_bf16.txt")
    with open(out, "w") as f:
        f.write("\n".join(lines) + "\n")
    print("wrote", out)


if __name__ == "__main__":
    main()
