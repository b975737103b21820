"""Writes softmax_two_keys.txt from the closed form, in 50-digit arithmetic (mpmath).

Independent of both the oracle and the GPU library: it evaluates
p1 = e^s/(1+e^s), LSE = ln(1+e^s), O = p0*v0 + p1*v1 for one fixed tiny case.
"""
import os

from mpmath import exp, log, mp, mpf, nstr

mp.dps = 50
s = mpf("0.693359375")  # ln 2 rounded to fp16
p1 = exp(s) / (1 + exp(s))
p0 = 1 - p1
v0 = [3, 0, -6, 1]
v1 = [0, 3, 6, 1]
o = [p0 * a + p1 * b for a, b in zip(v0, v1)]
HEADER = """\
# Hand-derived closed form, not a value printed by the paper (it prints none).
# Semantics pinned: start_generate(prompt, begin) prefills prompt[begin:] over the
# cached prompt[:begin] (Sec. 3.1); here begin = 1, one new token, one head,
# head_dim = 4, scale = 1, page size 2 (the new token sits in slot 1 of page 0 of the table).
#   q  = (1, 0, 0, 0)
#   k0 = (0, 0, 0, 0)                      -> score 0
#   k1 = (0.693359375, 0, 0, 0)            -> score s = fp16(ln 2)
#   v0 = (3, 0, -6, 1), v1 = (0, 3, 6, 1)
# p1 = e^s/(1+e^s), p0 = 1-p1, lse = ln(1+e^s), o = p0*v0 + p1*v1.
"""
path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "softmax_two_keys.txt")
with open(path, "w") as f:
    f.write(HEADER)
    f.write(f"s {nstr(s, 20)}\n")
    f.write(f"p0 {nstr(p0, 20)}\n")
    f.write(f"p1 {nstr(p1, 20)}\n")
    f.write(f"lse {nstr(log(1 + exp(s)), 20)}\n")
    f.write("o " + " ".join(nstr(x, 20) for x in o) + "\n")
print(open(path).read())
