"""Writes tests/golden/small_case.txt from the CPU oracle alone (never from the HIP path).

The paper prints no worked numeric example of the embedding path (no hash, table or gradient values), so there is
nothing of the paper's to store here.  What is stored is the oracle's own output on one tiny, fully specified
case, as a fixed point: a later change to the oracle's arithmetic shows up as a diff of this file and has to be
justified, and the GPU tests compare against the same numbers.  Floats are written as C99 hex literals (exact).

    python tests/golden/make_golden.py          # rewrites the file
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import oracle as O  # noqa: E402

PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "small_case.txt")

# The case: two tables (37 rows x 8 fp32; 64 rows x 16 bf16), three slots (tables 0, 1, 0), mixing hash, row-wise
# Adagrad lr 0.25 eps 1e-8 accumulator 0.5, init U(-0.5, 0.25) seed 2021; batch of 3 samples.
TABLES = [(37, 8, 0), (64, 16, 1)]
SLOTS = [(0, 0x1111), (1, 0x2222), (0, 0x3333)]
ARGS = dict(hash_kind=1, opt=1, lr=0.25, eps=1e-8, acc_init=0.5, init_seed=2021, init_lo=-0.5, init_hi=0.25)
IDS = np.array([5, 5, 900, 17, 0xFFFFFFFFFFFFFFFF, 5, 17, 31, 31, 31, 2 ** 40], dtype=np.uint64)
OFFSETS = np.array([0, 3, 4, 4, 5, 7, 8, 10, 11, 11], dtype=np.int32)   # bags of sample 0: [0,3) [3,4) [4,4) ...


def d_pooled():
    w = 8 + 16 + 8
    return ((np.arange(3 * w, dtype=np.float32).reshape(3, w) % 7) - 3.0) * np.float32(0.125)


def hexf(a):
    return " ".join(float(x).hex() for x in np.asarray(a, dtype=np.float64).ravel())


def lines():
    out = ["# written by tests/golden/make_golden.py from oracle/ only; floats are exact hex literals"]
    out.append("mix64 " + " ".join(f"{O.mix64(x):016x}" for x in (0, 1, 2 ** 63, 0xDEADBEEFCAFEF00D)))
    orc = O.Oracle(TABLES, SLOTS, **ARGS)
    out.append("rows " + " ".join(str(int(r)) for r in orc.hash_rows(IDS, OFFSETS)))
    for t, (rows, _, _) in enumerate(TABLES):
        w, a = orc.read_rows(t, np.array([0, 1, rows - 1]))
        out.append(f"init{t} " + hexf(w))
    out.append("pooled " + hexf(orc.lookup_pool(IDS, OFFSETS)))
    keys, seg_off, seg_bags = orc.backward_update(IDS, OFFSETS, d_pooled())
    out.append("keys " + " ".join(f"{int(k):x}" for k in keys))
    out.append("seg_off " + " ".join(str(int(x)) for x in seg_off))
    out.append("seg_bags " + " ".join(str(int(x)) for x in seg_bags))
    for k in keys:
        t, r = int(k) >> 32, int(k) & 0xFFFFFFFF
        w, a = orc.read_rows(t, np.array([r]))
        out.append(f"row {t} {r} acc {hexf(a)} w {hexf(w)}")
    out.append("pooled_after " + hexf(orc.lookup_pool(IDS, OFFSETS)))
    return out


if __name__ == "__main__":
    with open(PATH, "w") as f:
        f.write("\n".join(lines()) + "\n")
    print("wrote", PATH)
