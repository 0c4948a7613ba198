"""Writes zo_ln_table.hip.h: the 512 (inv_i, l_i) pivot pairs of the logarithm inside the normal transform
(zo_rng.hip.h), as hex-float literals.

    python paper_2507_03211_amd/csrc/gen_ln_table.py

Definition.  Interval i = 256 lb + j (lb = 0: significands m in [0.5, 1); lb = 1: m in [1, 2); j = the top 8 fraction
bits) has the pivot p_i = (1 + (j + 1/2) / 256) * (lb ? 1 : 1/2), its midpoint, except p_255 = 1.
inv_i = the fp32 number nearest to 1 / p_i; l_i = the fp32 number nearest to 2 ln(inv_i), inv_i taken exactly.
Computed here with exact rationals and a 60-digit logarithm, each rounding decided by comparing the two fp32
neighbours exactly (no double rounding through fp64).
"""
import os
import struct
from decimal import Decimal, getcontext
from fractions import Fraction

getcontext().prec = 60


def _f32_bits(x):
    return struct.unpack("<I", struct.pack("<f", x))[0]


def _f32_from_bits(b):
    return struct.unpack("<f", struct.pack("<I", b))[0]


def nearest_f32(exact):
    """exact: Fraction.  The fp32 number nearest to it (ties do not occur for these values; asserted)."""
    guess = struct.unpack("<f", struct.pack("<f", float(exact)))[0]
    b = _f32_bits(guess)
    cands = [guess]
    for nb in (b - 1, b + 1):
        if nb & 0x7FFFFFFF < 0x7F800000:
            cands.append(_f32_from_bits(nb))
    if guess == 0.0:
        cands = [0.0]
    dist = sorted((abs(Fraction(c) - exact), c) for c in cands)
    assert len(dist) == 1 or dist[0][0] != dist[1][0], "tie"
    return dist[0][1]


def table():
    out = []
    for i in range(512):
        lb, j = i >> 8, i & 255
        p = Fraction(1) if i == 255 else (1 + Fraction(2 * j + 1, 512)) * (1 if lb else Fraction(1, 2))
        inv = nearest_f32(1 / p)
        if inv == 1.0:
            l = 0.0
        else:
            fr = Fraction(inv)
            ln = (Decimal(fr.numerator) / Decimal(fr.denominator)).ln() * 2
            l = nearest_f32(Fraction(ln))
        out.append((inv, l))
    return out


def main():
    here = os.path.dirname(os.path.abspath(__file__))
    rows = table()
    with open(os.path.join(here, "zo_ln_table.hip.h"), "w") as f:
        f.write("// Pivot table of the logarithm in the normal transform (zo_rng.hip.h): entry i = {inv_i, l_i} with\n"
                "// inv_i = fl32(1 / p_i), l_i = fl32(2 ln inv_i), p_i the midpoint of significand interval i (p_255 = 1).\n"
                "// Written by gen_ln_table.py (exact rationals, 60-digit logarithm); do not edit by hand.\n"
                "#pragma once\n\nnamespace zo {\n\n"
                "__device__ __constant__ const float2 kLnPivot[512] = {\n")
        for i, (inv, l) in enumerate(rows):
            f.write("    {%s, %s},%s" % (float(inv).hex() + "f", float(l).hex() + "f", "\n" if i % 2 else " "))
        f.write("};\n\n}  // namespace zo\n")
    print("wrote", len(rows), "entries")


if __name__ == "__main__":
    main()
