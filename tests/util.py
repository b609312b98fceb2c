"""Shared helpers of the GPU parity tests: run one batch through the HIP library and through the
CPU oracle on the same seeded inputs and compare element by element."""
import numpy as np

# spec tolerances: fp32 tables 1e-5 relative + 1e-6 absolute; bf16 storage 2e-2 relative
TOL = {0: dict(rtol=1e-5, atol=1e-6), 1: dict(rtol=2e-2, atol=1e-6)}
LOW32 = np.uint64(0xFFFFFFFF)
# How close the two sides really are.  Both evaluate the same definitions in fp64 (sums of fp32 terms, the optimizer)
# and round each stored quantity once, so they differ only where the order of the fp64 additions moved a result across
# an fp32 (or bf16) rounding boundary: a difference of one unit in the last place, at a rate of order 1e-8 per
# element.  Besides the spec bar above, the comparisons below therefore require that all but MAX_DIFFERING of
# the elements are identical bit for bit.
MAX_DIFFERING = 1e-3


def tol_for(cfg):
    return TOL[1] if any(t.dtype == 1 for t in cfg.tables) else TOL[0]


def assert_close(got, want, rtol, atol, err_msg=""):
    """|got - want| <= atol + rtol |want| for every element, and at most MAX_DIFFERING of them differ at all."""
    got, want = np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64)
    bound = atol + rtol * np.abs(want)
    differing = float((got != want).mean()) if got.size else 0.0
    assert differing <= max(MAX_DIFFERING, 2.0 / max(got.size, 1)), \
        f"{err_msg}: {differing:.2e} of {got.size} elements are not bit-identical"
    bad = ~(np.abs(got - want) <= bound)       # NaNs count as bad
    if bad.any():
        i = np.unravel_index(np.argmax(np.where(bad, np.abs(got - want) - bound, -np.inf)), got.shape)
        raise AssertionError(f"{err_msg}: {int(bad.sum())} of {bad.size} elements outside the bound; worst at {i}: "
                             f"got {got[i]!r}, want {want[i]!r}, bound {bound[i] if np.ndim(bound) else bound!r}")


def compare_pooled(got, want, cfg):
    assert_close(got, want, **tol_for(cfg), err_msg="pooled")


def compare_dedup(gpu, orc):
    """Index form of the batch: integers, bit-exact."""
    gk, go, gb = gpu
    ok, oo, ob = orc
    assert len(gk) == len(ok), f"U differs: gpu {len(gk)} oracle {len(ok)}"
    np.testing.assert_array_equal(gk, ok)
    np.testing.assert_array_equal(go, oo)
    np.testing.assert_array_equal(gb, ob)


def compare_rows(ctx, orc, cfg, keys, extra_rows=64, seed=0, all_touched=None):
    """Touched rows (and their accumulators) within tolerance; a sample of other rows bit-exact.
    all_touched: every key the GPU batch touched, when `keys` is only a sample of them."""
    tables = (keys >> np.uint64(32)).astype(np.int64)
    rows = keys & LOW32
    if all_touched is None:
        all_touched = keys
    at_tables = (all_touched >> np.uint64(32)).astype(np.int64)
    at_rows = all_touched & LOW32
    rng = np.random.default_rng(seed)
    for t, td in enumerate(cfg.tables):
        r = rows[tables == t]
        tol = TOL[td.dtype]
        if len(r):
            gw, ga = ctx.emb_read_rows(t, r)
            ow, oa = orc.read_rows(t, r)
            assert_close(gw, ow, **tol, err_msg=f"table {t} rows")
            assert_close(ga, oa, rtol=1e-5, atol=1e-6, err_msg=f"table {t} accumulators")
        probe = rng.integers(0, td.rows, size=extra_rows, dtype=np.uint64)
        probe = np.setdiff1d(probe, at_rows[at_tables == t])
        if len(probe):
            gw, ga = ctx.emb_read_rows(t, probe)
            ow, oa = orc.read_rows(t, probe)
            np.testing.assert_array_equal(gw, ow, err_msg=f"table {t}: a row outside the batch changed")
            np.testing.assert_array_equal(ga, oa)


def run_steps(binding, workload_mod, oracle_mod, w, steps=1, dense=None, batches=None, grads=None, check_hash=True,
              cache_rows=None):
    """Runs `steps` forward+backward steps of workload w on both sides, each side on its own trajectory (the state
    of one side is never copied into the other), and compares everything after every step."""
    cfg = w.cfg
    if batches is None:
        batches = [workload_mod.make_batch(w, s) for s in range(steps)]
    if grads is None:
        grads = [workload_mod.make_d_pooled(w, s) for s in range(steps)]
    max_ids = max(b.num_ids for b in batches)
    max_b = max(b.batch_size for b in batches)
    if dense is None:
        dense = sum(t.rows * t.dim for t in cfg.tables) <= (1 << 24)
    orc = oracle_mod.Oracle.from_config(cfg, dense=dense)
    ctx = binding.EmbContext.from_config(cfg, max_batch=max(max_b, 1), max_ids=max_ids, cache_rows=cache_rows)
    import torch
    touched = []
    for b, dp in zip(batches, grads):
        db = binding.DeviceBatch(b.batch_size, b.ids, b.offsets)
        if check_hash and b.num_ids:
            np.testing.assert_array_equal(ctx.emb_hash_rows(db).cpu().numpy().view(np.uint32),
                                          orc.hash_rows(b.ids, b.offsets))
        pooled = ctx.emb_lookup_pool(db)
        torch.cuda.synchronize()
        compare_pooled(pooled.cpu().numpy(), orc.lookup_pool(b.ids, b.offsets), cfg)
        ctx.emb_backward_update(db, torch.from_numpy(dp).cuda())
        gd = ctx.emb_read_dedup()
        od = orc.backward_update(b.ids, b.offsets, dp)
        compare_dedup(gd, od)
        touched.append(od[0])
        compare_rows(ctx, orc, cfg, np.unique(np.concatenate(touched)))   # every row touched so far
    ctx.close()
    orc.close()


class Trajectory:
    """The HIP library and the oracle side by side over several steps of one workload, each on its own state (no
    value of one side ever enters the other).  step(t) runs lookup + backward/update of batch t on both sides and
    compares the pooled activations and the index form; final_check() compares rows and accumulators."""

    def __init__(self, binding, workload_mod, oracle_mod, w, max_ids):
        self.B, self.W, self.w, self.cfg = binding, workload_mod, w, w.cfg
        self.orc = oracle_mod.Oracle.from_config(w.cfg, dense=False)
        self.ctx = binding.EmbContext.from_config(w.cfg, max_batch=w.batch, max_ids=max_ids)
        self.touched = []
        self.steps_done = 0

    def step(self, t):
        import torch
        b = self.W.make_batch(self.w, t)
        dp = self.W.make_d_pooled(self.w, t)
        db = self.B.DeviceBatch(b.batch_size, b.ids, b.offsets)
        pooled = self.ctx.emb_lookup_pool(db)
        torch.cuda.synchronize()
        compare_pooled(pooled.cpu().numpy(), self.orc.lookup_pool(b.ids, b.offsets), self.cfg)
        del pooled
        self.ctx.emb_backward_update(db, torch.from_numpy(dp).cuda())
        od = self.orc.backward_update(b.ids, b.offsets, dp)
        compare_dedup(self.ctx.emb_read_dedup(), od)
        self.touched.append(od[0])
        self.steps_done += 1

    def final_check(self, max_rows=1 << 20, seed=0):
        """Rows and accumulators: every row of the last step, and a sample of the rows touched in earlier steps."""
        allk = np.unique(np.concatenate(self.touched))
        earlier = np.setdiff1d(allk, self.touched[-1])
        if len(earlier) > max_rows:
            earlier = np.random.default_rng(seed).choice(earlier, size=max_rows, replace=False)
        compare_rows(self.ctx, self.orc, self.cfg, np.union1d(self.touched[-1], earlier), extra_rows=256, seed=seed,
                     all_touched=allk)

    def close(self):
        self.ctx.close()
        self.orc.close()


def bag_of_occurrence(offsets):
    lens = np.diff(offsets).astype(np.int64)
    return np.repeat(np.arange(len(lens), dtype=np.uint32), lens)


def sub_batch(b, keep_occ, bag_of=None):
    """(ids, offsets) of the CSR batch with the same bags that holds only the occurrences flagged in keep_occ."""
    if bag_of is None:
        bag_of = bag_of_occurrence(b.offsets)
    n_bags = len(b.offsets) - 1
    kept_per_bag = np.bincount(bag_of[keep_occ], minlength=n_bags)
    off = np.zeros(n_bags + 1, dtype=np.int64)
    np.cumsum(kept_per_bag, out=off[1:])
    return b.ids[keep_occ], off.astype(np.int32)


def sampled_step_check(binding, workload_mod, oracle_mod, w, n_bags=4096, n_rows=2048, seed=0, dense_step=None):
    """Full-size parity on sampled outputs (for workloads whose full oracle run would take minutes).

    One forward + backward step of workload w on the GPU; the oracle then recomputes, from the paper's
    definitions, (a) the pooled vectors of `n_bags` sampled bags, (b) the updated rows, accumulators and
    bag lists of `n_rows` sampled unique rows -- a row's gradient depends only on its own occurrences, so
    a sub-batch that keeps exactly those occurrences gives the exact update -- and (c) the whole set of
    unique keys and segment offsets, which numpy derives from the oracle's hash of every id.
    dense_step (optional): called with the pooled activations (device tensor) between the lookup and the update,
    returns the gradient of the pooled activations (device tensor) that the update is fed with -- the dense network's
    step; the embedding update is then checked against the oracle fed with that same gradient (stage isolation).
    Without it the gradient is N(0, 1).
    """
    import torch
    cfg = w.cfg
    S = cfg.num_slots
    b = workload_mod.make_batch(w, 0)
    ctx = binding.EmbContext.from_config(cfg, max_batch=b.batch_size, max_ids=b.num_ids)
    db = binding.DeviceBatch(b.batch_size, b.ids, b.offsets)
    pooled_dev = ctx.emb_lookup_pool(db)
    torch.cuda.synchronize()
    if dense_step is None:
        gen = torch.Generator(device="cuda")
        gen.manual_seed(1234 + w.index)
        dp_dev = torch.randn((b.batch_size, cfg.pooled_width), generator=gen, device="cuda", dtype=torch.float32)
    else:
        dp_dev = dense_step(pooled_dev)
    pooled = pooled_dev.cpu().numpy()
    del pooled_dev
    ctx.emb_backward_update(db, dp_dev)
    gk, go, gb = ctx.emb_read_dedup()
    dp = dp_dev.cpu().numpy()
    del dp_dev

    rng = np.random.default_rng(seed)
    lens = np.diff(b.offsets).astype(np.int64)
    n_all_bags = len(lens)
    bag_of = np.repeat(np.arange(n_all_bags, dtype=np.uint32), lens)

    # (c) the whole index form's keys and offsets
    orc = oracle_mod.Oracle.from_config(cfg, dense=False)
    rows = orc.hash_rows(b.ids, b.offsets)
    slot_table = np.array([s.table for s in cfg.slots], dtype=np.uint64)
    keys_occ = (slot_table[bag_of % S] << np.uint64(32)) | rows.astype(np.uint64)
    uk, cnt = np.unique(keys_occ, return_counts=True)
    assert len(gk) == len(uk)
    np.testing.assert_array_equal(gk, uk)
    np.testing.assert_array_equal(go[1:].astype(np.int64), np.cumsum(cnt))
    assert go[0] == 0
    np.testing.assert_array_equal(np.bincount(gb, minlength=n_all_bags), lens)   # every occurrence listed once

    # (a) pooled vectors of sampled bags
    pick = rng.choice(n_all_bags, size=min(n_bags, n_all_bags), replace=False)
    keep = np.zeros(n_all_bags, dtype=bool)
    keep[pick] = True
    ids_s, off_s = sub_batch(b, keep[bag_of], bag_of)
    want = orc.lookup_pool(ids_s, off_s)
    cols = np.array(cfg.slot_cols())
    dims = np.array(cfg.slot_dims())
    tol = tol_for(cfg)
    for bag in pick[:512]:
        bb, s = divmod(int(bag), S)
        sl = slice(cols[s], cols[s] + dims[s])
        np.testing.assert_allclose(pooled[bb, sl], want[bb, sl], **tol, err_msg=f"bag {bag}")
    mask = np.zeros_like(want, dtype=bool)
    for bag in pick:
        bb, s = divmod(int(bag), S)
        mask[bb, cols[s]:cols[s] + dims[s]] = True
    np.testing.assert_allclose(pooled[mask], want[mask], **tol)
    orc.close()

    # (b) sampled unique rows: hot ones (longest segments) and random ones
    order = np.argsort(cnt)
    sample_u = np.unique(np.concatenate([order[-64:], rng.choice(len(uk), size=min(n_rows, len(uk)), replace=False)]))
    sample_keys = uk[sample_u]
    keep_occ = np.isin(keys_occ, sample_keys)
    ids_s, off_s = sub_batch(b, keep_occ, bag_of)
    orc2 = oracle_mod.Oracle.from_config(cfg, dense=False)
    ok, oo, ob = orc2.backward_update(ids_s, off_s, dp)
    np.testing.assert_array_equal(ok, sample_keys)
    for j, u in enumerate(sample_u):                      # bag list of each sampled key, bit-exact
        np.testing.assert_array_equal(gb[go[u]:go[u + 1]], ob[oo[j]:oo[j + 1]])
    compare_rows(ctx, orc2, cfg, sample_keys, extra_rows=256, seed=seed, all_touched=uk)
    orc2.close()
    ctx.close()
