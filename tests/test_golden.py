"""The stored small case (tests/golden/small_case.txt, written by tests/golden/make_golden.py from the oracle
alone).  It is a change detector, not a pin: the oracle reproducing its own stored output proves nothing about the
oracle (the independent expectation is tests/test_golden_adagrad.py and the pins of tests/test_oracle_pins.py); it
only makes a change of the oracle's arithmetic show up as a diff that has to be justified.  The HIP path is
compared with the same numbers -- integers bit for bit, floats within the tolerance of the table's storage type."""
import importlib.util
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
_spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
G = importlib.util.module_from_spec(_spec)
_spec.loader.exec_module(G)


def _stored():
    out = {}
    rows = []
    for line in open(G.PATH):
        if line.startswith("#"):
            continue
        f = line.split()
        if f[0] == "row":
            rows.append((int(f[1]), int(f[2]), float.fromhex(f[4]), np.array([float.fromhex(x) for x in f[6:]])))
        else:
            out[f[0]] = f[1:]
    out["row"] = rows
    return out


def test_oracle_output_on_the_stored_case_has_not_changed():
    want = [l for l in open(G.PATH).read().splitlines()]
    assert G.lines() == want


def test_stored_case_is_internally_consistent():
    s = _stored()
    seg_off = [int(x) for x in s["seg_off"]]
    assert seg_off[0] == 0 and seg_off[-1] == len(G.IDS) == len(s["seg_bags"])
    keys = [int(k, 16) for k in s["keys"]]
    assert keys == sorted(set(keys)) and len(keys) + 1 == len(seg_off)
    rows = [int(r) for r in s["rows"]]
    # every (table, row) of the batch appears among the keys, with its multiplicity
    lens = np.diff(G.OFFSETS)
    slot = np.repeat(np.tile(np.arange(3), 3), lens)
    table = np.array([t for t, _ in G.SLOTS])[slot]
    got = sorted((int(t) << 32) | r for t, r in zip(table, rows))
    want = sorted(k for k, a, b in zip(keys, seg_off[:-1], seg_off[1:]) for _ in range(b - a))
    assert got == want
    assert len(s["row"]) == len(keys)


@pytest.mark.gpu
def test_hip_path_matches_the_stored_case():
    import torch
    from paper_2111_05897_amd import binding as B
    B.load_library()
    s = _stored()
    ctx = B.EmbContext(G.TABLES, G.SLOTS, max_batch=3, max_ids=len(G.IDS), **G.ARGS)
    db = B.DeviceBatch(3, G.IDS, G.OFFSETS)
    np.testing.assert_array_equal(ctx.emb_hash_rows(db).cpu().numpy().view(np.uint32), [int(r) for r in s["rows"]])
    # columns: slot 0 (fp32, 8) | slot 1 (bf16 table, 16) | slot 2 (fp32, 8)
    rtol = np.concatenate([np.full(8, 1e-5), np.full(16, 2e-2), np.full(8, 1e-5)])
    want = np.array([float.fromhex(x) for x in s["pooled"]]).reshape(3, 32)
    got = ctx.emb_lookup_pool(db).cpu().numpy()
    assert (np.abs(got - want) <= rtol * np.abs(want) + 1e-6).all()
    ctx.emb_backward_update(db, torch.from_numpy(G.d_pooled()).cuda())
    keys, seg_off, seg_bags = ctx.emb_read_dedup()
    np.testing.assert_array_equal(keys, [int(k, 16) for k in s["keys"]])
    np.testing.assert_array_equal(seg_off, [int(x) for x in s["seg_off"]])
    np.testing.assert_array_equal(seg_bags, [int(x) for x in s["seg_bags"]])
    for t, r, acc, w in s["row"]:
        gw, ga = ctx.emb_read_rows(t, np.array([r]))
        tol = 2e-2 if G.TABLES[t][2] == 1 else 1e-5
        np.testing.assert_allclose(gw[0], w, rtol=tol, atol=1e-6)
        np.testing.assert_allclose(ga[0], acc, rtol=1e-5, atol=1e-6)
    want = np.array([float.fromhex(x) for x in s["pooled_after"]]).reshape(3, 32)
    got = ctx.emb_lookup_pool(db).cpu().numpy()
    assert (np.abs(got - want) <= rtol * np.abs(want) + 2e-6).all()
    ctx.close()
