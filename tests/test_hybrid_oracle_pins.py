"""Pins of the hybrid-loop oracle (oracle/hybrid_oracle.py) -- CPU only.

The oracle defers the training of a batch with a queue.  The pins state the same semantics in other terms:
explicit versions of the table (lookup t reads version max(0, t - tau)), the limit tau >= run length (every
lookup reads the initial table), frozen embeddings (tau cannot matter), and a deliberately wrong oracle
(staleness tau + 1) that the version pin must reject.
"""
from collections import deque

import numpy as np
import pytest

from oracle import hybrid_oracle as HO
from oracle import mlp_oracle as MO
from oracle.oracle import Oracle
from paper_2111_05897_amd import workload as W

ROWS, DIM, SLOTS, DENSE, BATCH, STEPS = 96, 8, 4, 32, 64, 7
WIDTHS = [SLOTS * DIM + DENSE, 64, 1]


def _emb(lr=0.5, opt=0):
    return Oracle([(ROWS, DIM, 0)], [(0, W.default_salt(s)) for s in range(SLOTS)], hash_kind=1, opt=opt, lr=lr, eps=1e-8,
                  acc_init=0.1, init_seed=77, init_lo=-0.5, init_hi=0.5)


def _mlp():
    Ws, bs = W.make_mlp_params(WIDTHS, 5)
    return MO.MLP(Ws, bs, lr=0.2, loss_mean=True, rounding=False)


def _batches():
    out = []
    for t in range(STEPS):
        b = W.random_batch(900 + t, BATCH, SLOTS, 3, 40)          # 40 ids over 96 rows: every batch hits the same rows
        dense, labels = W.make_dense_and_labels(31, t, BATCH, DENSE, positive_rate=0.4)
        out.append((b.ids, b.offsets, dense, labels))
    return out


def _all_rows(emb):
    return emb.read_rows(0, np.arange(ROWS))


def _versions_run(batches, tau, opt=0):
    """The same loop written with explicit table versions: version v = the table after the updates of batches
    0 .. v-1; the lookup of batch t reads version max(0, t - tau)."""
    mlp = _mlp()
    work = _emb(opt=opt)
    versions = [_all_rows(work)]
    pooled, losses = [], []
    for t, (ids, offsets, dense, labels) in enumerate(batches):
        v = max(0, t - tau)
        while len(versions) <= v:                                   # make version len(versions) from the one before
            k = len(versions) - 1
            work.write_rows(0, np.arange(ROWS), *versions[k])
            loss, d_pooled, _ = mlp.step(pooled[k], batches[k][2], batches[k][3])
            work.backward_update(batches[k][0], batches[k][1], d_pooled)
            versions.append(_all_rows(work))
            losses.append(float(loss))
        reader = _emb(opt=opt)
        reader.write_rows(0, np.arange(ROWS), *versions[v])
        pooled.append(reader.lookup_pool(ids, offsets))
    return pooled, np.array(losses)


@pytest.mark.parametrize("tau,opt", [(0, 0), (1, 0), (2, 1), (3, 0)])
def test_lookup_reads_the_version_tau_updates_back(tau, opt):
    batches = _batches()
    losses, pooled = HO.run(_emb(opt=opt), _mlp(), batches, tau, record_pooled=True)
    want_pooled, want_losses = _versions_run(batches, tau, opt=opt)
    for t in range(STEPS):
        np.testing.assert_array_equal(pooled[t], want_pooled[t], err_msg=f"batch {t}")
    np.testing.assert_array_equal(losses[:len(want_losses)], want_losses)
    assert len(losses) == STEPS


def test_staleness_changes_what_a_lookup_sees():
    """Not vacuous: with shared hot rows, tau = 1 and tau = 0 differ from the second batch on, and only there."""
    batches = _batches()
    _, p0 = HO.run(_emb(), _mlp(), batches, 0, record_pooled=True)
    _, p1 = HO.run(_emb(), _mlp(), batches, 1, record_pooled=True)
    np.testing.assert_array_equal(p0[0], p1[0])
    assert np.abs(p0[1] - p1[1]).max() > 1e-4


def test_tau_beyond_the_run_reads_the_initial_table():
    batches = _batches()
    _, pooled = HO.run(_emb(), _mlp(), batches, STEPS + 3, record_pooled=True)
    for t, (ids, offsets, _, _) in enumerate(batches):
        np.testing.assert_array_equal(pooled[t], _emb().lookup_pool(ids, offsets))


def test_frozen_embeddings_make_tau_irrelevant():
    """The dense side takes the batches in the same order whatever tau is; with a zero embedding step size the
    whole run (losses, final weights) cannot depend on tau."""
    batches = _batches()
    ref_mlp = _mlp()
    ref, _ = HO.run(_emb(lr=0.0), ref_mlp, batches, 0)
    for tau in (1, 4):
        mlp = _mlp()
        got, _ = HO.run(_emb(lr=0.0), mlp, batches, tau)
        np.testing.assert_array_equal(got, ref)
        for a, b in zip(mlp.W, ref_mlp.W):
            np.testing.assert_array_equal(a, b)


def test_all_batches_are_trained_once_in_order():
    class Rec:
        def __init__(self):
            self.log = []

        def lookup_pool(self, ids, offsets):
            self.log.append(("L", int(ids[0])))
            return np.zeros((1, 1), dtype=np.float32)

        def backward_update(self, ids, offsets, d):
            self.log.append(("U", int(ids[0])))

    class Net:
        def step(self, pooled, dense, labels):
            return 0.0, pooled, None

    rec = Rec()
    HO.run(rec, Net(), [(np.array([t]), None, None, None) for t in range(5)], 2)
    assert rec.log == [("L", 0), ("L", 1), ("L", 2), ("U", 0), ("L", 3), ("U", 1), ("L", 4), ("U", 2), ("U", 3), ("U", 4)]


def test_version_pin_rejects_an_off_by_one_loop():
    """A loop that trains one batch later than it should (staleness tau + 1) must fail the version pin."""
    def late_run(emb, mlp, batches, tau):
        q, pooled_log = deque(), []
        for ids, offsets, dense, labels in batches:
            pooled = emb.lookup_pool(ids, offsets)
            pooled_log.append(pooled)
            q.append((ids, offsets, dense, labels, pooled))
            if len(q) > tau + 1:
                i, o, d, y, p = q.popleft()
                emb.backward_update(i, o, mlp.step(p, d, y)[1])
        return pooled_log
    batches = _batches()
    wrong = late_run(_emb(), _mlp(), batches, 1)
    want, _ = _versions_run(batches, 1)
    assert any(np.abs(wrong[t] - want[t]).max() > 1e-4 for t in range(STEPS))
