"""Writes exp_table.h: 2^(j/128), j = 0..127, as pairs (hi, lo) of doubles with hi the double
nearest to the value and lo the double nearest to the remainder, computed with 60 decimal digits.
Run from this directory: python make_exp_table.py > exp_table.h"""
from decimal import Decimal, getcontext

getcontext().prec = 60
N = 128
LN2 = Decimal(2).ln()

print("// 2^(j/128) for j = 0..127 as hi + lo, hi the nearest double and lo the nearest double to the")
print("// remainder (written by make_exp_table.py; the table of a table-driven fp64 exponential).")
print("#pragma once")
print("")
print("namespace lantern {")
print("")
print("constexpr int EXP_TABLE_N = %d;" % N)
print("#if defined(__HIPCC__)")
print("#define LANTERN_EXP_TABLE_QUAL __device__")
print("#else")
print("#define LANTERN_EXP_TABLE_QUAL")
print("#endif")
print("static const LANTERN_EXP_TABLE_QUAL double EXP_TABLE_HILO[2 * EXP_TABLE_N] = {")
for j in range(N):
    v = (LN2 * Decimal(j) / Decimal(N)).exp()
    hi = float(v)
    lo = float(v - Decimal(hi))
    print("    %s, %s," % (hi.hex(), lo.hex()))
print("};")
print("")
print("}  // namespace lantern")
