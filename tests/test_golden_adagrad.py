"""The worked two-row, two-step row-wise Adagrad case (tests/golden/adagrad_two_rows_two_steps.txt, written by
tests/golden/make_adagrad_case.py from the closed form in decimal arithmetic, without the oracle and without the HIP
code): equation (2) with the optimizer state beside the row (section 4.2.2).  The oracle must reproduce it, and so
must the HIP path."""
import os

import numpy as np
import pytest

from oracle import oracle as O

PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "adagrad_two_rows_two_steps.txt")


def _case():
    c = {"w0": {}, "steps": {}}
    for line in open(PATH):
        f = line.split()
        if not f or f[0] == "#":
            continue
        if f[0] in ("lr", "eps", "acc_init"):
            c[f[0]] = float.fromhex(f[1])
        elif f[0] == "dim":
            c["dim"] = int(f[1])
        elif f[0] == "w0":
            c["w0"][int(f[1])] = [float.fromhex(x) for x in f[2:]]
        elif f[0] == "step":
            st = c["steps"].setdefault(int(f[1]), {"d_pooled": {}, "pooled": {}, "row": {}})
            if f[2] in ("ids", "offsets"):
                st[f[2]] = [int(x) for x in f[3:]]
            elif f[2] in ("d_pooled", "pooled"):
                st[f[2]][int(f[3])] = [float.fromhex(x) for x in f[4:]]
            elif f[2] == "row":
                st["row"][int(f[3])] = (float.fromhex(f[5]), [float.fromhex(x) for x in f[7:]])
    return c


def _arrays(st):
    ids = np.array(st["ids"], np.uint64)
    off = np.array(st["offsets"], np.int32)
    dp = np.array([st["d_pooled"][b] for b in range(len(off) - 1)], np.float32)
    pooled = np.array([st["pooled"][b] for b in range(len(off) - 1)], np.float32)
    return ids, off, dp, pooled


def test_the_case_file_is_what_its_script_writes():
    import importlib.util
    spec = importlib.util.spec_from_file_location("make_adagrad_case", os.path.join(os.path.dirname(PATH), "make_adagrad_case.py"))
    m = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(m)
    assert m.lines() == open(PATH).read().splitlines()


def test_oracle_reproduces_the_worked_adagrad_case_bit_for_bit():
    c = _case()
    orc = O.Oracle([(2, c["dim"], 0)], [(0, 0)], hash_kind=0, opt=1, lr=c["lr"], eps=c["eps"], acc_init=c["acc_init"],
                   init_seed=1, init_lo=0.0, init_hi=0.0)
    orc.write_rows(0, np.array([0, 1], np.uint64), np.array([c["w0"][0], c["w0"][1]], np.float32))
    for s in sorted(c["steps"]):
        st = c["steps"][s]
        ids, off, dp, pooled = _arrays(st)
        np.testing.assert_array_equal(orc.lookup_pool(ids, off), pooled)
        orc.backward_update(ids, off, dp)
        w, a = orc.read_rows(0, np.array([0, 1], np.uint64))
        for r in (0, 1):
            np.testing.assert_array_equal(w[r], np.array(st["row"][r][1], np.float32), err_msg=f"step {s} row {r}")
            assert a[r] == np.float32(st["row"][r][0]), f"step {s} accumulator {r}"


@pytest.mark.gpu
def test_hip_path_reproduces_the_worked_adagrad_case():
    import torch
    from paper_2111_05897_amd import binding as B
    B.load_library()
    c = _case()
    D = c["dim"]
    # the library's smallest row is 8 wide: the case's 4 columns are laid twice side by side, which leaves the mean of
    # the squared gradient -- and with it every number of the case -- unchanged
    ctx = B.EmbContext([(2, 2 * D, 0)], [(0, 0)], hash_kind=0, opt=1, lr=c["lr"], eps=c["eps"], acc_init=c["acc_init"],
                       init_seed=1, init_lo=0.0, init_hi=0.0, max_batch=4, max_ids=8)
    ctx.emb_write_rows(0, np.array([0, 1], np.uint64), np.tile(np.array([c["w0"][0], c["w0"][1]], np.float32), (1, 2)))
    for s in sorted(c["steps"]):
        st = c["steps"][s]
        ids, off, dp, pooled = _arrays(st)
        db = B.DeviceBatch(len(off) - 1, ids, off)
        got = ctx.emb_lookup_pool(db).cpu().numpy()
        np.testing.assert_allclose(got, np.tile(pooled, (1, 2)), rtol=1e-5, atol=1e-6)
        ctx.emb_backward_update(db, torch.from_numpy(np.tile(dp, (1, 2))).cuda())
        w, a = ctx.emb_read_rows(0, np.array([0, 1], np.uint64))
        for r in (0, 1):
            np.testing.assert_allclose(w[r], np.tile(np.array(st["row"][r][1], np.float32), 2), rtol=1e-5, atol=1e-6)
            np.testing.assert_allclose(a[r], st["row"][r][0], rtol=1e-5, atol=1e-6)
    ctx.close()
