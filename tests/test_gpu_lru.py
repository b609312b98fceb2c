"""GPU tests of tables kept in host memory behind the LRU cache (emb_create_cached).

(1) Transparency: a context whose table sits in host memory with a small cache must give, bit for bit, what a
context with the table resident gives -- pooled activations at every step, every row and accumulator at the
end (read through the cache and again after a flush) -- while rows are being evicted and brought back.
(2) Policy: after every call the row -> slot map and the statistics equal the CPU model's
(oracle/lru_oracle.py).  (3) The usual parity against the embedding oracle, run through the cached context.
"""
import numpy as np
import pytest

from oracle import oracle as ORC
from oracle.lru_oracle import LruCache
from paper_2111_05897_amd import workload as W
from tests import util

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_2111_05897_amd import binding
    binding.load_library()
    return binding


def _args(tables, slots, opt):
    return dict(tables=tables, slots=[(t, W.default_salt(s)) for s, t in enumerate(slots)], hash_kind=1, opt=opt, lr=0.1,
                eps=1e-8, acc_init=0.1, init_seed=909, init_lo=-0.2, init_hi=0.2)


def _table_rows(orc, b, slots, table, S):
    """Unique rows of `table` that batch b touches (from the CPU oracle's hash)."""
    rows = orc.hash_rows(b.ids, b.offsets)
    lens = np.diff(b.offsets.astype(np.int64))
    slot_of = np.repeat(np.tile(np.arange(S), b.batch_size), lens)
    return np.unique(rows[np.asarray(slots)[slot_of] == table])


@pytest.mark.parametrize("dim,dtype,opt,cache", [(16, 0, 0, 1024), (64, 1, 1, 800), (128, 0, 1, 768)])
def test_cached_table_is_transparent_and_follows_the_lru_model(B, dim, dtype, opt, cache):
    import torch
    rows, S, bsz, steps = 1 << 14, 3, 64, 14
    a = _args([(rows, dim, dtype)], [0] * S, opt)
    max_ids = bsz * S * 4
    ref = B.EmbContext(max_batch=bsz, max_ids=max_ids, **a)
    ctx = B.EmbContext(max_batch=bsz, max_ids=max_ids, cache_rows=[cache], **a)
    orc = ORC.Oracle(**a)
    model = LruCache(cache)
    rng = np.random.default_rng(dim)
    for t in range(steps):
        # the id space moves slowly, so some rows come back after having been evicted
        b = W.random_batch(500 + t, bsz, S, 4, 900)
        b.ids[:] = b.ids + np.uint64(150 * (t % 5))
        db = B.DeviceBatch(b.batch_size, b.ids, b.offsets)
        touched = _table_rows(orc, b, [0] * S, 0, S)
        got = ctx.emb_lookup_pool(db)
        want = ref.emb_lookup_pool(db)
        torch.cuda.synchronize()
        assert torch.equal(got, want), f"pooled differs at step {t}"
        model.access(touched)
        where = ctx.emb_cache_where(0)
        want_where = np.full(rows, -1, dtype=np.int32)
        for r, s in model.where.items():
            want_where[r] = s
        np.testing.assert_array_equal(where, want_where, err_msg=f"lookup {t}")
        dp = torch.from_numpy(rng.standard_normal((bsz, S * dim)).astype(np.float32)).cuda()
        ctx.emb_backward_update(db, dp)
        ref.emb_backward_update(db, dp)
        model.access(touched)
        st = ctx.emb_cache_stats(0)
        assert (st["requested"], st["misses"], st["written_back"], st["overflows"]) == \
            (model.requested, model.misses, model.written_back, 0), f"update {t}"
        g, r_ = ctx.emb_read_dedup(), ref.emb_read_dedup()
        for x, y in zip(g, r_):
            np.testing.assert_array_equal(x, y)
    assert model.written_back > 0 and model.misses > cache          # the test did evict
    all_rows = np.arange(rows)
    want_w, want_acc = ref.emb_read_rows(0, all_rows)
    got_w, got_acc = ctx.emb_read_rows(0, all_rows)
    np.testing.assert_array_equal(got_w, want_w)
    np.testing.assert_array_equal(got_acc, want_acc)
    ctx.emb_cache_flush()
    got_w, got_acc = ctx.emb_read_rows(0, all_rows)
    np.testing.assert_array_equal(got_w, want_w)
    np.testing.assert_array_equal(got_acc, want_acc)
    np.testing.assert_array_equal(ctx.emb_cache_where(0), where)          # a flush moves nothing
    # writing through the cache reaches a row wherever it is
    some = np.array([int(next(iter(model.where))), int(np.setdiff1d(all_rows, list(model.where))[0])])
    new_w = np.full((2, dim), 0.5, dtype=np.float32)
    ctx.emb_write_rows(0, some, new_w, np.array([3.0, 4.0], dtype=np.float32))
    back_w, back_a = ctx.emb_read_rows(0, some)
    np.testing.assert_array_equal(back_w, new_w)
    np.testing.assert_array_equal(back_a, [3.0, 4.0])
    ctx.close()
    ref.close()


def test_cached_and_resident_tables_side_by_side(B):
    """Table 0 (dim 32) behind a cache, table 1 (dim 8, bf16) resident, slots interleaved: same results as both
    resident, and the oracle agrees with either."""
    import torch
    tables = [(1 << 13, 32, 0), (1 << 10, 8, 1)]
    slots = [0, 1, 0, 1, 0]
    S, bsz = len(slots), 64
    a = _args(tables, slots, 1)
    max_ids = bsz * S * 3
    ref = B.EmbContext(max_batch=bsz, max_ids=max_ids, **a)
    ctx = B.EmbContext(max_batch=bsz, max_ids=max_ids, cache_rows=[max_ids, 0], **a)
    width = sum(tables[t][1] for t in slots)
    rng = np.random.default_rng(1)
    for t in range(8):
        b = W.random_batch(40 + t, bsz, S, 3, 5000)
        db = B.DeviceBatch(b.batch_size, b.ids, b.offsets)
        got, want = ctx.emb_lookup_pool(db), ref.emb_lookup_pool(db)
        torch.cuda.synchronize()
        assert torch.equal(got, want)
        dp = torch.from_numpy(rng.standard_normal((bsz, width)).astype(np.float32)).cuda()
        ctx.emb_backward_update(db, dp)
        ref.emb_backward_update(db, dp)
    for tb, (r, _, _) in enumerate(tables):
        gw, ga = ctx.emb_read_rows(tb, np.arange(r))
        ww, wa = ref.emb_read_rows(tb, np.arange(r))
        np.testing.assert_array_equal(gw, ww)
        np.testing.assert_array_equal(ga, wa)
    assert ctx.emb_cache_stats(0)["written_back"] > 0
    with pytest.raises(B.EmbError):
        ctx.emb_cache_stats(1)                                     # table 1 has no cache
    with pytest.raises(B.EmbError):
        ctx.emb_table_ptr(0)                                       # no flat device array behind a cache
    ctx.close()
    ref.close()


def test_cached_context_against_the_oracle(B):
    """The ordinary parity run (hash, pooled, index form, rows after each step) through a cached context."""
    w = W.make_workload(1, scale=1.0 / 64)                         # 2^16 rows, dim 32, 26 slots
    batches = [W.make_batch(w, s) for s in range(3)]
    need = max(b.num_ids for b in batches)
    util.run_steps(B, W, ORC, w, steps=3, batches=batches, cache_rows=[min(need, w.cfg.tables[0].rows - 1)])


def test_cache_validation(B):
    a = _args([(1 << 12, 16, 0)], [0, 0], 0)
    with pytest.raises(B.EmbError):                                # smaller than a batch's worst case
        B.EmbContext(max_batch=64, max_ids=1000, cache_rows=[999], **a)
    ctx = B.EmbContext(max_batch=64, max_ids=1000, cache_rows=[1 << 12], **a)   # >= rows: simply resident
    with pytest.raises(B.EmbError):
        ctx.emb_cache_stats(0)
    ctx.close()


@pytest.mark.parametrize("tau", [0, 2])
def test_hybrid_loop_over_a_cached_table(B, tau):
    """The staleness loop (lookups ahead of updates, second stream) driving a table behind the cache: losses,
    network weights and every embedding row equal those of the same loop over a resident table, bit for bit."""
    import torch
    rows, dim, S, dense_w, bsz = 1 << 15, 16, 4, 64, 128
    widths = [S * dim + dense_w, 128, 64, 1]
    a = _args([(rows, dim, 0)], [0] * S, 1)
    max_ids = bsz * S * 5
    Ws, bs = W.make_mlp_params(widths, 21)
    out = []
    for cache in (None, [max_ids]):
        emb = B.EmbContext(max_batch=bsz, max_ids=max_ids, cache_rows=cache, **a)
        mlp = B.MlpContext(widths, S * dim, dense_w, bsz, 0.1, Ws, bs, loss_mean=True)
        loop = B.HybridLoop(emb, mlp, tau)
        keep = []
        for t in range(10):
            b = W.random_batch(3000 + t, bsz, S, 5, 20000)
            d, y = W.make_dense_and_labels(5, t, bsz, dense_w, positive_rate=0.3)
            item = (B.DeviceBatch(b.batch_size, b.ids, b.offsets), torch.from_numpy(d).cuda(), torch.from_numpy(y).cuda())
            keep.append(item)
            loop.hyb_submit(*item)
        loop.hyb_drain()
        losses = loop.hyb_read_losses(0, 10)
        w_, acc = emb.emb_read_rows(0, np.arange(rows))
        out.append((losses, w_, acc, [mlp.mlp_read_weights(l)[0] for l in range(3)]))
        if cache:
            st = emb.emb_cache_stats(0)
            assert st["written_back"] > 0 and st["overflows"] == 0
        loop.close()
        mlp.close()
        emb.close()
    np.testing.assert_array_equal(out[0][0], out[1][0])
    np.testing.assert_array_equal(out[0][1], out[1][1])
    np.testing.assert_array_equal(out[0][2], out[1][2])
    for x, y in zip(out[0][3], out[1][3]):
        np.testing.assert_array_equal(x, y)


def test_cached_table_is_transparent_at_full_size(B):
    """Config 1 at its real size (2^22 rows, 2.2 M ids per batch) with the smallest cache the size rule allows:
    hundreds of thousands of rows are replaced per call, the scans span thousands of workgroups.  Pooled
    activations at every step and a sample of rows at the end equal those of the resident table bit for bit."""
    import torch
    w = W.make_workload(1)
    cfg = w.cfg
    batches = [W.make_batch(w, s) for s in range(5)]
    max_ids = max(b.num_ids for b in batches)
    ref = B.EmbContext.from_config(cfg, max_batch=w.batch, max_ids=max_ids)
    ctx = B.EmbContext.from_config(cfg, max_batch=w.batch, max_ids=max_ids, cache_rows=[max_ids])
    gen = torch.Generator(device="cuda")
    gen.manual_seed(7)
    for t in (0, 1, 2, 3, 4, 0, 2):
        b = batches[t]
        db = B.DeviceBatch(b.batch_size, b.ids, b.offsets)
        got, want = ctx.emb_lookup_pool(db), ref.emb_lookup_pool(db)
        torch.cuda.synchronize()
        assert torch.equal(got, want), f"pooled differs at batch {t}"
        dp = torch.randn((w.batch, cfg.pooled_width), generator=gen, device="cuda", dtype=torch.float32)
        ctx.emb_backward_update(db, dp)
        ref.emb_backward_update(db, dp)
    st = ctx.emb_cache_stats(0)
    assert st["written_back"] > 100000 and st["overflows"] == 0, st
    rows = np.unique(np.random.default_rng(0).integers(0, cfg.tables[0].rows, size=200000).astype(np.uint64))
    gw, ga = ctx.emb_read_rows(0, rows)
    ww, wa = ref.emb_read_rows(0, rows)
    np.testing.assert_array_equal(gw, ww)
    np.testing.assert_array_equal(ga, wa)
    ctx.close()
    ref.close()


def test_cached_context_orders_calls_that_arrive_on_different_streams(B):
    """A context with cached tables has one admission state; the library makes a hot call that arrives on another
    stream wait for the one before it, so a two-stream caller without events of its own gets what one stream gives."""
    import torch
    rows, S, bsz, steps, cache = 1 << 13, 4, 128, 6, 2048
    a = _args([(rows, 64, 0)], [0] * S, 1)
    max_ids = bsz * S * 4
    one = B.EmbContext(max_batch=bsz, max_ids=max_ids, cache_rows=[cache], **a)
    two = B.EmbContext(max_batch=bsz, max_ids=max_ids, cache_rows=[cache], **a)
    s_a, s_b = torch.cuda.Stream(), torch.cuda.Stream()      # default priority, both
    rng = np.random.default_rng(2)
    batches = [W.random_batch(900 + t, bsz, S, 4, 3000) for t in range(steps)]
    dbs = [B.DeviceBatch(b.batch_size, b.ids, b.offsets) for b in batches]
    grads = [torch.from_numpy(rng.standard_normal((bsz, S * 64)).astype(np.float32)).cuda() for _ in range(steps)]
    p_one = [torch.empty((bsz, S * 64), device="cuda") for _ in range(steps)]
    p_two = [torch.empty((bsz, S * 64), device="cuda") for _ in range(steps)]
    torch.cuda.synchronize()
    for t in range(steps):
        one.emb_lookup_pool(dbs[t], p_one[t])
        one.emb_backward_update(dbs[t], grads[t])
    for t in range(steps):                                    # lookups on one stream, updates on the other, no events
        two.emb_lookup_pool(dbs[t], p_two[t], stream=s_a)
        two.emb_backward_update(dbs[t], grads[t], stream=s_b)
    torch.cuda.synchronize()
    for t in range(steps):
        assert torch.equal(p_one[t], p_two[t]), f"lookup {t}"
    allrows = np.arange(rows, dtype=np.uint64)
    w1, a1 = one.emb_read_rows(0, allrows)
    w2, a2 = two.emb_read_rows(0, allrows)
    np.testing.assert_array_equal(w1, w2)
    np.testing.assert_array_equal(a1, a2)
    assert one.emb_cache_stats(0) == two.emb_cache_stats(0)
    one.close()
    two.close()
