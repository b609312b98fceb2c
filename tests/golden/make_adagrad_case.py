"""Writes tests/golden/adagrad_two_rows_two_steps.txt: a hand-sized worked case of the embedding update
(equation (2) with Omega^emb = row-wise Adagrad, optimizer state stored beside the row as in section 4.2.2),
computed here from the closed form with 60-digit decimal arithmetic.  This script imports nothing from
oracle/ or from the HIP package: the file it writes is an expectation that is independent of both.

The case: one fp32 table of 2 rows x 4 columns, identity hash, one slot, sum pooling; lr, eps and the initial
accumulator are the fp32 values nearest 0.05, 1e-8 and 0.1.  Two steps:

  step 1: three samples, bags {0, 0}, {1}, {0}       row 0 occurs three times (twice inside one bag), row 1 once
  step 2: two samples,  bags {1, 0}, {1}             row 1 occurs twice, row 0 once

Per step and per row that occurs:   G   = sum over the row's occurrences of the bag's upstream gradient
                                    a'  = a + mean_d(G_d^2)                   stored as fp32
                                    w_d' = w_d - lr * G_d / (sqrt(a') + eps)   stored as fp32
with the exact a' (not its fp32 rounding) inside the square root, and step 2 starting from the stored fp32 values.
Every stored quantity is the exact result rounded once to fp32 (nearest, ties to even).

    python tests/golden/make_adagrad_case.py          # rewrites the file
"""
import os
from decimal import Decimal, getcontext
from fractions import Fraction

getcontext().prec = 60
PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "adagrad_two_rows_two_steps.txt")

D = 4


def f32(x, exact=True) -> float:
    """The fp32 value nearest to x (ties to even), by integer arithmetic on the exact rational value of x.
    exact=False marks a 60-digit approximation of an irrational result (it went through a square root): such a
    value must not sit within 1e-30 of a tie, where the digits beyond the 60th would decide."""
    q = Fraction(x)
    if q == 0:
        return 0.0
    a = abs(q)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1                                   # 2^e <= a < 2^(e+1)
    sp = max(e - 23, -149)                       # spacing 2^sp of fp32 values around a
    scaled = a / Fraction(2) ** sp
    m = scaled.numerator // scaled.denominator
    rest = scaled - m
    if not exact:
        assert abs(rest - Fraction(1, 2)) > Fraction(1, 10 ** 30), "too close to an fp32 tie to decide from 60 digits"
    if rest > Fraction(1, 2) or (rest == Fraction(1, 2) and m % 2 == 1):
        m += 1
    v = float(m * Fraction(2) ** sp)             # exact: m < 2^24 + 1
    return -v if q < 0 else v


LR, EPS, ACC0 = f32(Decimal("0.05")), f32(Decimal("1e-8")), f32(Decimal("0.1"))
W0 = [[f32(Decimal(v)) for v in row] for row in (("0.5", "-0.25", "0.125", "1.0"), ("-0.75", "0.0625", "0.3", "-0.01"))]
STEPS = [
    dict(ids=[0, 0, 1, 0], offsets=[0, 2, 3, 4],
         d_pooled=[["1.5", "-2.0", "0.25", "3.0"], ["-0.5", "0.75", "1.0", "-1.25"], ["2.0", "0.5", "-1.5", "0.125"]]),
    dict(ids=[1, 0, 1], offsets=[0, 2, 3],
         d_pooled=[["0.3", "-0.7", "1.1", "0.9"], ["-1.75", "2.5", "0.0", "-0.6"]]),
]


def run():
    w = [[Decimal(v) for v in row] for row in W0]
    a = [Decimal(ACC0), Decimal(ACC0)]
    out = []
    for st in STEPS:
        dp = [[Decimal(f32(Decimal(v))) for v in row] for row in st["d_pooled"]]     # upstream gradients are fp32
        pooled = []
        G = {}
        for bag in range(len(st["offsets"]) - 1):
            acc = [Decimal(0)] * D
            for i in range(st["offsets"][bag], st["offsets"][bag + 1]):
                r = st["ids"][i]
                acc = [x + y for x, y in zip(acc, w[r])]
                g = G.setdefault(r, [Decimal(0)] * D)
                G[r] = [x + y for x, y in zip(g, dp[bag])]
            pooled.append([f32(x) for x in acc])
        for r in sorted(G):
            a_new = a[r] + sum(g * g for g in G[r]) / D
            denom = a_new.sqrt() + Decimal(EPS)
            w[r] = [Decimal(f32(wd - Decimal(LR) * g / denom, exact=False)) for wd, g in zip(w[r], G[r])]
            a[r] = Decimal(f32(a_new))
        out.append(dict(pooled=pooled, dp=[[float(x) for x in row] for row in dp], w=[[float(x) for x in row] for row in w],
                        a=[float(x) for x in a]))
    return out


def hexf(vals):
    return " ".join(float(v).hex() for v in vals)


def lines():
    L = ["# written by tests/golden/make_adagrad_case.py (closed form, decimal arithmetic; no oracle, no HIP code)",
         "# fp32 values as exact hex literals",
         f"dim {D}", f"lr {LR.hex()}", f"eps {EPS.hex()}", f"acc_init {ACC0.hex()}"]
    for r, row in enumerate(W0):
        L.append(f"w0 {r} " + hexf(row))
    for s, (st, res) in enumerate(zip(STEPS, run())):
        L.append(f"step {s} ids " + " ".join(map(str, st["ids"])))
        L.append(f"step {s} offsets " + " ".join(map(str, st["offsets"])))
        for b, row in enumerate(res["dp"]):
            L.append(f"step {s} d_pooled {b} " + hexf(row))
        for b, row in enumerate(res["pooled"]):
            L.append(f"step {s} pooled {b} " + hexf(row))
        for r in range(2):
            L.append(f"step {s} row {r} acc {res['a'][r].hex()} w " + hexf(res["w"][r]))
    return L


if __name__ == "__main__":
    with open(PATH, "w") as f:
        f.write("\n".join(lines()) + "\n")
    print("wrote", PATH)
