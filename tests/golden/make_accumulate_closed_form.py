"""Writes accumulate_closed_form.txt: exact values of the momentum-corrected
accumulation (Alg. 1/2, first line of the layer loop, with DGC's momentum
correction named in Sec. V-A) for m = 1/2, g = 2^-10 at every iteration.

Uses exact rational arithmetic only (no oracle, no GPU code): every value is
checked to be exactly representable in fp32, so the fp32 recurrence must
reproduce it bit for bit whatever the rounding mode.
Closed form: u_t = g(2 - 2^(1-t)),  v_t = sum_{s<=t} u_s = g(2t - 2 + 2^(1-t)).
"""
import os
import struct
from fractions import Fraction

m, g = Fraction(1, 2), Fraction(1, 1024)
u = v = Fraction(0)
rows = []
for t in range(1, 17):
    u = m * u + g
    v = v + u
    assert u == g * (2 - Fraction(2) ** (1 - t))
    assert v == g * (2 * t - 2 + Fraction(2) ** (1 - t))
    for x in (u, v):
        f = struct.unpack("<f", struct.pack("<f", float(x)))[0]
        assert Fraction(f) == x, "not exactly representable in fp32"
    ub = struct.unpack("<I", struct.pack("<f", float(u)))[0]
    vb = struct.unpack("<I", struct.pack("<f", float(v)))[0]
    rows.append((t, ub, vb))

out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "accumulate_closed_form.txt")
with open(out, "w") as f:
    f.write("# u <- m*u + g ; v <- v + u  with m = 0.5, g = 2^-10, u0 = v0 = 0 (Alg. 1/2 accumulation line,\n")
    f.write("# momentum correction of Sec. V-A).  Exact rational values, all representable in fp32.\n")
    f.write("# t  bits(u_t)  bits(v_t)   (IEEE-754 binary32, hex)\n")
    for t, ub, vb in rows:
        f.write(f"{t} {ub:08x} {vb:08x}\n")
print("wrote", out)
