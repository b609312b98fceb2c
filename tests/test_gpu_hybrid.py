"""GPU tests of the hybrid step loop (hyb_*): lookups run tau batches ahead of the dense step and the
embedding update, on a second stream.

Two things are checked.  (1) The schedule: every kernel of the path is deterministic, so the loop must give
bit for bit what the same entry points give when called one after the other, on one stream, in the order the
oracle of the loop (oracle/hybrid_oracle.py) prescribes -- any lookup that saw one update too many or too few,
or an input buffer read after its slot was reused, changes bits.  (2) The composite against the oracles: losses
and the movement of the embedding rows, to the tolerance of the bf16 dense step (2e-2)."""
import numpy as np
import pytest

from oracle import hybrid_oracle as HO
from oracle import mlp_oracle as MO
from oracle.oracle import Oracle
from paper_2111_05897_amd import workload as W

pytestmark = pytest.mark.gpu

ROWS, DIM, SLOTS, DENSE = 4096, 16, 4, 64
WIDTHS = [SLOTS * DIM + DENSE, 128, 64, 1]
SIZES = [128, 64, 192, 128, 128, 64, 192, 128, 64]       # batch sizes, so that a reused slot changes shape


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_2111_05897_amd import binding
    binding.load_library()
    return binding


def _emb_args(opt):
    return dict(tables=[(ROWS, DIM, 0)], slots=[(0, W.default_salt(s)) for s in range(SLOTS)], hash_kind=1, opt=opt, lr=0.3,
                eps=1e-8, acc_init=0.1, init_seed=4242, init_lo=-0.3, init_hi=0.3)


def _contexts(B, opt, max_batch=192, max_ids=192 * SLOTS * 6):
    emb = B.EmbContext(max_batch=max_batch, max_ids=max_ids, **_emb_args(opt))
    Ws, bs = W.make_mlp_params(WIDTHS, 11)
    mlp = B.MlpContext(WIDTHS, SLOTS * DIM, DENSE, max_batch, 0.1, Ws, bs, loss_mean=True)
    return emb, mlp


def _host_batches():
    out = []
    for t, bsz in enumerate(SIZES):
        b = W.random_batch(7000 + t, bsz, SLOTS, 5, 300)       # 300 ids: the same rows come back every batch
        dense, labels = W.make_dense_and_labels(17, t, bsz, DENSE, positive_rate=0.3)
        out.append((b, dense, labels))
    return out


def _serial(B, emb, mlp, batches, tau):
    """The entry points one after the other on the default stream, in the order of the loop's oracle."""
    import torch
    pending, losses = [], []

    def train(item):
        db, dense, labels, pooled = item
        d_pooled, loss = mlp.mlp_step(pooled, dense, labels)
        emb.emb_backward_update(db, d_pooled)
        losses.append(loss)

    for b, dense, labels in batches:
        db = B.DeviceBatch(b.batch_size, b.ids, b.offsets)
        pooled = emb.emb_lookup_pool(db)
        pending.append((db, torch.from_numpy(dense).cuda(), torch.from_numpy(labels).cuda(), pooled))
        if len(pending) > tau:
            train(pending.pop(0))
    while pending:
        train(pending.pop(0))
    torch.cuda.synchronize()
    return np.array([l.item() for l in losses], dtype=np.float32)


def _state(emb, mlp):
    w, acc = emb.emb_read_rows(0, np.arange(ROWS))
    return [w, acc] + [x for l in range(len(WIDTHS) - 1) for x in mlp.mlp_read_weights(l)]


@pytest.mark.parametrize("tau,opt", [(0, 0), (1, 1), (3, 0), (12, 1)])
def test_loop_equals_the_serial_order_bit_for_bit(B, tau, opt):
    import torch
    batches = _host_batches()
    emb_s, mlp_s = _contexts(B, opt)
    want_losses = _serial(B, emb_s, mlp_s, batches, tau)
    want = _state(emb_s, mlp_s)

    emb, mlp = _contexts(B, opt)
    loop = B.HybridLoop(emb, mlp, tau)
    # one set of staging buffers, overwritten for every batch once the loop has taken its copy
    ids_buf = torch.zeros(192 * SLOTS * 6, dtype=torch.int64, device="cuda")
    off_buf = torch.zeros(192 * SLOTS + 1, dtype=torch.int32, device="cuda")
    dense_buf = torch.zeros(192 * DENSE, dtype=torch.float32, device="cuda")
    label_buf = torch.zeros(192, dtype=torch.float32, device="cuda")
    for t, (b, dense, labels) in enumerate(batches):
        loop.hyb_wait_inputs()
        n, bsz = len(b.ids), b.batch_size
        ids_buf[:n] = torch.from_numpy(b.ids.view(np.int64)).cuda()
        off_buf[:bsz * SLOTS + 1] = torch.from_numpy(b.offsets).cuda()
        dense_buf[:bsz * DENSE] = torch.from_numpy(dense.reshape(-1)).cuda()
        label_buf[:bsz] = torch.from_numpy(labels).cuda()
        torch.cuda.synchronize()                                  # the fills ran on torch's stream
        db = B.DeviceBatch.__new__(B.DeviceBatch)
        db.batch_size, db.num_ids, db.ids, db.offsets = bsz, n, ids_buf, off_buf
        db.c = B.emb_batch(bsz, 0, n, ids_buf.data_ptr(), off_buf.data_ptr())
        loop.hyb_submit(db, dense_buf[:bsz * DENSE].view(bsz, DENSE), label_buf[:bsz])
        submitted, trained = loop.hyb_counts()
        assert submitted == t + 1 and trained == max(0, t + 1 - tau)
    loop.hyb_drain()
    assert loop.hyb_counts() == (len(batches), len(batches))
    got_losses = loop.hyb_read_losses(0, len(batches))
    np.testing.assert_array_equal(got_losses, want_losses)
    for g, w_ in zip(_state(emb, mlp), want):
        np.testing.assert_array_equal(g, w_)
    loop.close()


@pytest.mark.parametrize("tau", [0, 2])
def test_loop_tracks_the_oracle(B, tau):
    import torch
    batches = _host_batches()
    emb, mlp = _contexts(B, 0)
    loop = B.HybridLoop(emb, mlp, tau)
    keep = []
    for b, dense, labels in batches:
        db = B.DeviceBatch(b.batch_size, b.ids, b.offsets)
        d, y = torch.from_numpy(dense).cuda(), torch.from_numpy(labels).cuda()
        keep.append((db, d, y))
        loop.hyb_submit(db, d, y)
    loop.hyb_drain()
    got_losses = loop.hyb_read_losses(0, len(batches))

    orc_emb = Oracle(**{k: v for k, v in _emb_args(0).items()})
    Ws, bs = W.make_mlp_params(WIDTHS, 11)
    orc_mlp = MO.MLP(Ws, bs, lr=0.1, loss_mean=True, rounding=True)
    want_losses, _ = HO.run(orc_emb, orc_mlp, [(b.ids, b.offsets, d, y) for b, d, y in batches], tau)
    np.testing.assert_allclose(got_losses, want_losses, rtol=2e-2)
    # movement of the embedding rows away from their initial values, in norm
    init, _ = Oracle(**_emb_args(0)).read_rows(0, np.arange(ROWS))
    got_w, _ = emb.emb_read_rows(0, np.arange(ROWS))
    want_w, _ = orc_emb.read_rows(0, np.arange(ROWS))
    moved = np.linalg.norm(want_w - init)
    assert moved > 0
    assert np.linalg.norm(got_w - want_w) <= 2e-2 * moved
    # untouched rows are still bit-identical to the initial table
    untouched = np.all(want_w == init, axis=1)
    assert untouched.any() and np.array_equal(got_w[untouched], init[untouched])
    loop.close()


@pytest.mark.parametrize("tau,opt", [(0, 1), (2, 0), (3, 1)])
def test_embedding_side_of_the_loop_follows_the_oracle_element_by_element(B, tau, opt):
    """The loop equals the serial order of its entry points bit for bit (test above).  Here that serial order runs
    with the embedding oracle beside it, fed at every training step with the GPU network's own gradient of the
    pooled activations (stage isolation: the bf16 noise of the dense step never enters the comparison): every
    lookup of the loop -- stale by tau updates -- and the rows and accumulators at the end must match the oracle
    element by element on the fp32 bar."""
    import torch
    from tests import util
    batches = _host_batches()
    emb, mlp = _contexts(B, opt)
    orc = Oracle(**_emb_args(opt))
    cfg = W.EmbConfig(tables=[W.TableDesc(ROWS, DIM, 0)], slots=[W.SlotDesc(0, W.default_salt(s)) for s in range(SLOTS)])
    pending = []

    def train(item):
        b, db, dense, labels, pooled = item
        d_pooled, _ = mlp.mlp_step(pooled, dense, labels)
        emb.emb_backward_update(db, d_pooled)
        orc.backward_update(b.ids, b.offsets, d_pooled.cpu().numpy())

    for b, dense, labels in batches:
        db = B.DeviceBatch(b.batch_size, b.ids, b.offsets)
        pooled = emb.emb_lookup_pool(db)
        torch.cuda.synchronize()
        util.compare_pooled(pooled.cpu().numpy(), orc.lookup_pool(b.ids, b.offsets), cfg)
        pending.append((b, db, torch.from_numpy(dense).cuda(), torch.from_numpy(labels).cuda(), pooled))
        if len(pending) > tau:
            train(pending.pop(0))
    while pending:
        train(pending.pop(0))
    gw, ga = emb.emb_read_rows(0, np.arange(ROWS))
    ow, oa = orc.read_rows(0, np.arange(ROWS))
    util.assert_close(gw, ow, rtol=1e-5, atol=1e-6, err_msg="rows")
    util.assert_close(ga, oa, rtol=1e-5, atol=1e-6, err_msg="accumulators")
    assert (ow != Oracle(**_emb_args(opt)).read_rows(0, np.arange(ROWS))[0]).any()


def test_loop_validation(B):
    import torch
    emb, mlp = _contexts(B, 0)
    Ws, bs = W.make_mlp_params([128 + 64, 64, 1], 3)
    other = B.MlpContext([128 + 64, 64, 1], 128, 64, 64, 0.1, Ws, bs)
    with pytest.raises(B.EmbError):
        B.HybridLoop(emb, other, 1)                               # pooled widths differ
    loop = B.HybridLoop(emb, mlp, 1)
    b = W.random_batch(1, 96, SLOTS, 3, 50)                       # 96 is not a multiple of 64
    db = B.DeviceBatch(b.batch_size, b.ids, b.offsets)
    with pytest.raises(B.EmbError):
        loop.hyb_submit(db, torch.zeros(96, DENSE, device="cuda"), torch.zeros(96, device="cuda"))
    with pytest.raises(B.EmbError):
        loop.hyb_read_losses(0, 1)                                # nothing trained yet
    assert loop.hyb_counts() == (0, 0)
    loop.hyb_drain()                                              # nothing to do
    loop.hyb_sync()
    loop.close()


def test_small_staleness_trains_like_synchronous(B):
    """The qualitative claim of section 5 / Table 2 on the synthetic click task: the student learns (the
    progressive-validation loss falls well below the base-rate entropy) and a staleness of a few batches
    leaves the loss it reaches within 2 % of fully synchronous training."""
    from paper_2111_05897_amd import staleness_study as SS
    task = SS.Task(3)
    out = {}
    for tau in (0, 4):
        losses, bayes, base = SS.run(tau, 240, batch_size=2048, seed=3, task=task)
        assert np.isfinite(losses).all()
        out[tau] = SS.summarize(tau, losses, bayes, base, 40)
    assert out[0]["loss_last"] < 0.93 * out[0]["base_rate_entropy"], out
    assert out[0]["loss_last"] > out[0]["teacher_entropy"], out
    assert abs(out[4]["loss_last"] - out[0]["loss_last"]) <= 0.02 * out[0]["loss_last"], out
    # the comparison the hybrid algorithm is defined against: with the dense network's gradients arriving 4 steps
    # late as well (fully asynchronous), the same run ends clearly worse, or diverges
    losses, bayes, base = SS.run(4, 240, batch_size=2048, seed=3, task=task, dense_delay=4)
    worse = SS.summarize(4, losses, bayes, base, 40, "fully asynchronous")
    assert (not np.isfinite(worse["loss_last"])) or worse["loss_last"] > out[4]["loss_last"] + 0.02, (worse, out)
