"""Writes zo_rayleigh_table.hip.h: the piecewise-cubic table of the Rayleigh quantile that the normal transform
(zo_rng.hip.h) draws its radius from, as hex-float literals.

    python paper_2507_03211_amd/csrc/gen_rayleigh_table.py

Definition.  A cell is (h, E, jj): h = 0 the lower half of the distribution (F = q, rho = sqrt(-2 ln(1 - q))), h = 1
the upper half (1 - F = q, rho = sqrt(-2 ln q)); q = qf 2^-32 where qf is an fp32 number with biased exponent E in
134..157 whose top five fraction bits are jj.  The cell's pivot pf is its midpoint (fraction = jj, then a one, then
zeros) and its four entries are the fp32 numbers nearest to the Taylor coefficients of rho_h at the pivot with respect
to d = qf - pf:  rho ~ a0 + d (a1 + d (a2 + d a3)).
Computed here in 60-digit decimal arithmetic; every rounding to fp32 is decided by comparing the two neighbouring
fp32 numbers exactly (no double rounding through fp64).
Layout: entry (2 c + h) of 2048, c = (32 E + jj) mod 1024 (192 .. 959), which is where the kernel's address
arithmetic lands; the other entries are zero and never read.
"""
import os
import struct
from decimal import Decimal, getcontext
from fractions import Fraction

getcontext().prec = 60


def nearest_f32(x):
    """x: Decimal.  The fp32 number nearest to it."""
    exact = Fraction(x)
    guess = struct.unpack("<f", struct.pack("<f", float(x)))[0]
    b = struct.unpack("<I", struct.pack("<f", guess))[0]
    cands = {guess}
    for nb in (b - 1, b + 1):
        if 0 <= nb and (nb & 0x7FFFFFFF) < 0x7F800000:
            cands.add(struct.unpack("<f", struct.pack("<I", nb))[0])
    dist = sorted((abs(Fraction(c) - exact), c) for c in cands)
    assert dist[0][0] != dist[1][0], "tie"
    return dist[0][1]


def cell(h, E, jj):
    q = (Decimal(1) + (Decimal(jj) + Decimal("0.5")) / 32) * Decimal(2) ** (E - 127 - 32)
    g, dg = (q, Decimal(1)) if h else (1 - q, Decimal(-1))
    t = -2 * g.ln()
    t1, t2, t3 = -2 * dg / g, 2 / (g * g), -4 * dg / (g * g * g)
    rho = t.sqrt()
    r1 = t1 / (2 * rho)
    r2 = t2 / (2 * rho) - t1 * t1 / (4 * rho ** 3)
    r3 = t3 / (2 * rho) - 3 * t1 * t2 / (4 * rho ** 3) + 3 * t1 ** 3 / (8 * rho ** 5)
    s = Decimal(2) ** -32
    return [nearest_f32(v) for v in (rho, r1 * s, r2 / 2 * s * s, r3 / 6 * s * s * s)]


def table():
    out = [[0.0, 0.0, 0.0, 0.0] for _ in range(2048)]
    for h in (0, 1):
        for E in range(134, 158):
            for jj in range(32):
                out[2 * ((32 * E + jj) % 1024) + h] = cell(h, E, jj)
    return out


def main():
    here = os.path.dirname(os.path.abspath(__file__))
    rows = table()
    with open(os.path.join(here, "zo_rayleigh_table.hip.h"), "w") as f:
        f.write("// Piecewise-cubic table of the Rayleigh quantile for the normal transform (zo_rng.hip.h): entry 2 c + h holds\n"
                "// {a0, a1, a2, a3} of cell c = (32 E + jj) mod 1024 in half h, the fp32 roundings of the Taylor coefficients of\n"
                "// rho_h at the cell's pivot.  Entries of cells that do not occur are zero.\n"
                "// Written by gen_rayleigh_table.py (60-digit decimal arithmetic); do not edit by hand.\n"
                "#pragma once\n\nnamespace zo {\n\n"
                "constexpr int kRayleighFirst = 2 * 192, kRayleighLast = 2 * 960;   // the entries that are used: [first, last)\n"
                "__device__ __constant__ const float4 kRayleighCell[2048] = {\n")
        for i, a in enumerate(rows):
            if all(v == 0.0 for v in a):
                f.write("    {0.0f, 0.0f, 0.0f, 0.0f},\n")
            else:
                f.write("    {%s},\n" % ", ".join(float(v).hex() + "f" for v in a))
        f.write("};\n\n}  // namespace zo\n")
    print("wrote", sum(1 for a in rows if any(a)), "cells")


if __name__ == "__main__":
    main()
