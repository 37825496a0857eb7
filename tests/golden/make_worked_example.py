"""Writes tests/golden/worked_example_n3k4m2.txt.

The paper prints no numeric worked example, so this one is derived here from
Eq. 1-5, 7, 11 and 12 of Section 2.1 with exact rational arithmetic (Python
Fraction / int); numpy float32 scalars stand in for the single IEEE fp32
operations the equations leave (128/gamma, x*scale, beta*gamma/128, acc*scale).
It imports neither the oracle nor the GPU library: it is an independent
derivation that the oracle is pinned against.

Run:  python tests/golden/make_worked_example.py
"""
from fractions import Fraction
from pathlib import Path
import math

import numpy as np

f32 = np.float32

W = [[0.02, -0.01, 0.03, -0.04], [0.00, 0.05, -0.02, 0.01], [-0.03, 0.02, 0.01, 0.01]]
X = [[1.0, -0.5, 0.25, 2.0], [-1.5, 0.3, 0.7, -0.1]]
EPS = 1e-5


def exact(v):
    return Fraction(float(f32(v)))


def to_f32(fr: Fraction):
    # nearest fp32 of an exact rational (via nearest fp64; inputs here are far from ties)
    return f32(float(fr))


def round_half_even(v: np.float32) -> int:
    return round(Fraction(float(v)))  # Python rounds exact halves to even


def derive(skip_ln: bool):
    N, K, M = len(W), len(W[0]), len(X)
    Wf = [[exact(v) for v in row] for row in W]
    alpha = to_f32(sum(sum(r) for r in Wf) / (N * K))                      # Eq. 3
    beta = to_f32(sum(sum(abs(v) for v in r) for r in Wf) / (N * K))       # Eq. 12
    sign = [[1 if v > exact(alpha) else -1 for v in r] for r in Wf]        # Eq. 1-2
    words = [sum((1 << k) for k in range(K) if sign[n][k] > 0) for n in range(N)]
    xhat = []
    for row in X:
        xs = [float(f32(v)) for v in row]
        if skip_ln:
            xhat.append([f32(v) for v in xs])
            continue
        mu = math.fsum(xs) / K                                             # Eq. 12, LN
        var = math.fsum((v - mu) ** 2 for v in xs) / K
        rstd = 1.0 / math.sqrt(var + EPS)
        xhat.append([f32((v - mu) * rstd) for v in xs])
    gamma = [max(abs(v) for v in row) for row in xhat]                     # Eq. 5
    codes = []
    for row, g in zip(xhat, gamma):
        scale = f32(128.0) / g
        codes.append([max(-128, min(127, round_half_even(v * scale))) for v in row])  # Eq. 4
    acc = [[sum(codes[m][k] * sign[n][k] for k in range(K)) for n in range(N)] for m in range(M)]
    y = [[f32(acc[m][n]) * ((beta * gamma[m]) / f32(128.0)) for n in range(N)] for m in range(M)]
    return alpha, beta, sign, words, xhat, gamma, codes, acc, y


def fmt(vals):
    return " ".join(repr(float(v)) if isinstance(v, (np.floating, float)) else str(int(v))
                    for v in vals)


def main():
    out = ["# Worked example for BitLinear, N=3 K=4 M=2, derived from Eq. 1-5, 7, 11, 12",
           "# (Section 2.1) by tests/golden/make_worked_example.py with exact rationals.",
           "# Readings: round-half-even + clamp [-128,127]; beta = mean|W|; Sign(0) = -1.",
           "W " + fmt(v for r in W for v in r),
           "X " + fmt(v for r in X for v in r),
           f"eps {EPS!r}"]
    for tag, skip in (("noln", True), ("ln", False)):
        alpha, beta, sign, words, xhat, gamma, codes, acc, y = derive(skip)
        if skip:
            out += ["alpha " + fmt([alpha]), "beta " + fmt([beta]),
                    "sign " + fmt(v for r in sign for v in r), "words " + fmt(words)]
        out += [f"{tag}.xhat " + fmt(v for r in xhat for v in r),
                f"{tag}.gamma " + fmt(gamma),
                f"{tag}.codes " + fmt(v for r in codes for v in r),
                f"{tag}.acc " + fmt(v for r in acc for v in r),
                f"{tag}.y " + fmt(v for r in y for v in r)]
    path = Path(__file__).with_name("worked_example_n3k4m2.txt")
    path.write_text("\n".join(out) + "\n")
    print(path.read_text())


if __name__ == "__main__":
    main()
