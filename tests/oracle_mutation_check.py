"""Are the oracle's pins sharp?  Plants one mistake at a time in a COPY of oracle/oracle.cpp
(on the CPU, in a temporary directory), runs the oracle's pin tests against that copy and
expects them to fail.  Not collected by pytest; run it by hand:

    python tests/oracle_mutation_check.py

Exit status 0 when every planted mistake is caught.
"""
import os
import subprocess
import sys
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

MUTATIONS = [
    ("variance uses g once instead of g squared", "(1.0 - b2) * g * g", "(1.0 - b2) * g"),
    ("no bias correction of the variance", "std::sqrt(vn) / sqrt_bc2 + eps", "std::sqrt(vn) + eps"),
    ("momentum weight beta1 instead of 1 - beta1", "b1 * double(m[i]) + (1.0 - b1) * g", "b1 * double(m[i]) + b1 * g"),
    ("decay applied with the wrong sign of the step", "- step_size * (mn / denom)", "+ step_size * (mn / denom)"),
    ("fp32 sequence: 1/sqrt(1 - beta2^t) dropped", "std::fmaf(std::sqrt(vn), rsb2, eps)", "std::sqrt(vn) + eps"),
    ("fp32 sequence: (1 - beta1) replaced by beta1", "float t1 = omb1 * g;", "float t1 = b1 * g;"),
    ("fp32 sequence: decay also on undecayed elements",
     "float t3 = w[i] * ((no_decay && no_decay[i]) ? 1.0f : decay);", "float t3 = w[i] * decay;"),
    # last-bit variations of the fp32 sequence: only a correctly rounded referee can tell them apart
    ("fp32 sequence: momentum with two roundings instead of one fused multiply-add",
     "float mn = std::fmaf(b1, m[i], t1);", "float mn = b1 * m[i] + t1;"),
    ("fp32 sequence: (1 - beta2) * (g * g) instead of ((1 - beta2) * g) * g",
     "float t2 = omb2 * g;\n      t2 = t2 * g;", "float t2 = g * g;\n      t2 = omb2 * t2;"),
    ("fp32 sequence: denominator with two roundings", "float d = std::fmaf(std::sqrt(vn), rsb2, eps);",
     "float d = std::sqrt(vn) * rsb2 + eps;"),
    ("fp32 sequence: weight update with two roundings", "float wn = std::fmaf(-step_size, u, t3);",
     "float wn = t3 - step_size * u;"),
    ("fp32 sequence: multiplies by the reciprocal of the denominator instead of dividing", "float u = mn / d;",
     "float u = mn * (1.0f / d);"),
    ("norm ignores the loss scale", "double x = double(decode16(g[i], dtype)) / loss_scale;",
     "double x = double(decode16(g[i], dtype));"),
    ("clip coefficient without its epsilon", "max_norm / (norm + 1e-6)", "max_norm / norm"),
    ("pack: position off by one", "uint64_t c = e / S, pos = e % S;", "uint64_t c = e / S, pos = (e + 1) % S;"),
    ("accumulate: first micro-batch adds instead of overwriting", "acc[i] = overwrite ? x : acc[i] + x;",
     "acc[i] = acc[i] + x;"),
    ("skipped step still counts as an update", "    rep->t_after = st->t;\n    return false;",
     "    st->t += 1;\n    rep->t_after = st->t;\n    return false;"),
    ("bf16 recast truncates instead of rounding to nearest even",
     "u += 0x7fffu + keep_lsb;", "u += 0;"),
    ("bf16 recast rounds ties away from zero", "u += 0x7fffu + keep_lsb;", "u += 0x8000u;"),
    ("loss scale does not back off", "st->loss_scale = std::max(sigma * sc->backoff, 1.0);", "st->loss_scale = sigma;"),
    ("fp32 norm squares without unscaling", "double x = double(g[i]) / loss_scale;", "double x = double(g[i]);"),
]


def main() -> int:
    src = open(os.path.join(ROOT, "oracle", "oracle.cpp")).read()
    survived = []
    with tempfile.TemporaryDirectory() as tmp:
        for k, (name, old, new) in enumerate(MUTATIONS):
            if src.count(old) < 1:
                print(f"[{k:2d}] {name}: the text to replace is gone from oracle.cpp - update this list")
                survived.append(name)
                continue
            path = os.path.join(tmp, f"mutant_{k}.cpp")
            with open(path, "w") as f:
                f.write(src.replace(old, new, 1))
            env = dict(os.environ, ORACLE_SRC_OVERRIDE=path)
            res = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests"), "-q", "-x", "-m", "not gpu",
                                  "-k", "oracle", "-p", "no:cacheprovider"], env=env, capture_output=True, text=True, cwd=ROOT)
            tail = (res.stdout.strip().splitlines() or ["?"])[-1]
            caught = res.returncode != 0
            print(f"[{k:2d}] {name}: {'caught' if caught else 'SURVIVED'}  ({tail})", flush=True)
            if not caught:
                survived.append(name)
    print(f"{len(MUTATIONS) - len(survived)} of {len(MUTATIONS)} planted mistakes caught")
    return 1 if survived else 0


if __name__ == "__main__":
    raise SystemExit(main())
