"""Writes fma_discriminator.txt: one (b, s, c) triple per element type on which
Triad computed with two roundings, fl(b + fl(s*c)), differs from the fused
fl(b + s*c).  Every value is derived with exact rational arithmetic
(fractions.Fraction) and Python's correctly rounded int/int division; nothing
here calls the oracle or the GPU library.

Triad is defined with a separately rounded multiply and add (Table 1 lists it
as a 3-line kernel a = b + s*c; both sides are built with contraction off), so
an implementation that fuses them must fail on these vectors.

Run from the repository root:  python tests/golden/make_fma_discriminator.py
"""
import os
from fractions import Fraction

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))


def rn64(q: Fraction) -> float:
    return q.numerator / q.denominator  # correctly rounded to binary64


def rn32(q: Fraction) -> float:
    # round-to-nearest-even to binary32, done on the exact rational
    if q == 0:
        return 0.0
    sign = -1 if q < 0 else 1
    q = abs(q)
    e = 0
    while q >= 2:
        q /= 2
        e += 1
    while q < 1:
        q *= 2
        e -= 1
    scaled = q * (1 << 23)
    fl = scaled.numerator // scaled.denominator
    rem = scaled - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return sign * float(Fraction(fl, 1 << 23) * Fraction(2) ** e)


def find(rn, to_type, seed):
    rng = np.random.RandomState(seed)
    while True:
        b, c = (to_type(x) for x in rng.uniform(0.5, 1.5, size=2))
        s = to_type(0.4)
        fb, fs, fc = Fraction(float(b)), Fraction(float(s)), Fraction(float(c))
        two_step = rn(fb + Fraction(rn(fs * fc)))
        fused = rn(fb + fs * fc)
        if two_step != fused:
            return float(b), float(s), float(c), two_step, fused


def main():
    lines = [
        "# Triad a = b + s*c (Table 1), two roundings vs one fused rounding.",
        "# columns: type  b  s  c  two_step=fl(b+fl(s*c))  fused=fl(b+s*c)   (C99 hex floats)",
        "# written by tests/golden/make_fma_discriminator.py from exact rational arithmetic",
    ]
    for name, rn, to_type, seed in (("f64", rn64, np.float64, 7), ("f32", rn32, np.float32, 11)):
        vals = find(rn, to_type, seed)
        lines.append(name + " " + " ".join(float(v).hex() for v in vals))
    with open(os.path.join(HERE, "fma_discriminator.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")
    print("\n".join(lines))


if __name__ == "__main__":
    main()
