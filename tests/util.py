"""Shared helpers of the GPU parity tests: run one batch through the HIP library and through the
CPU oracle on the same seeded inputs and compare element by element."""
import numpy as np

# spec tolerances: fp32 tables 1e-5 relative + 1e-6 absolute; bf16 storage 2e-2 relative
TOL = {0: dict(rtol=1e-5, atol=1e-6), 1: dict(rtol=2e-2, atol=1e-6)}
LOW32 = np.uint64(0xFFFFFFFF)


def tol_for(cfg):
    return TOL[1] if any(t.dtype == 1 for t in cfg.tables) else TOL[0]


def compare_pooled(got, want, cfg):
    np.testing.assert_allclose(got, want, **tol_for(cfg))


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
            np.testing.assert_allclose(gw, ow, **tol, err_msg=f"table {t} rows")
            np.testing.assert_allclose(ga, oa, rtol=1e-5, atol=1e-6, err_msg=f"table {t} accumulators")
        probe = rng.integers(0, td.rows, size=extra_rows, dtype=np.uint64)
        probe = np.setdiff1d(probe, at_rows[at_tables == t])
        if len(probe):
            gw, ga = ctx.emb_read_rows(t, probe)
            ow, oa = orc.read_rows(t, probe)
            np.testing.assert_array_equal(gw, ow, err_msg=f"table {t}: a row outside the batch changed")
            np.testing.assert_array_equal(ga, oa)


def sync_rows(ctx, orc, cfg, keys):
    """bf16 tables only: after a step has been compared, copy the oracle's rows into the GPU table.
    A row that the two sides rounded to neighbouring bf16 values (within the 2e-2 bar) would otherwise
    show up in the next step's pooled sums, where cancellation can magnify it beyond any relative bound;
    with the state re-aligned every step is judged on its own arithmetic."""
    tables = (keys >> np.uint64(32)).astype(np.int64)
    rows = keys & LOW32
    for t in range(len(cfg.tables)):
        r = rows[tables == t]
        if len(r):
            ow, oa = orc.read_rows(t, r)
            ctx.emb_write_rows(t, r, ow, oa)


def run_steps(binding, workload_mod, oracle_mod, w, steps=1, dense=None, batches=None, grads=None, check_hash=True,
              cache_rows=None):
    """Runs `steps` forward+backward steps of workload w on both sides and compares everything."""
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
        compare_rows(ctx, orc, cfg, np.unique(np.concatenate(touched)))
        if any(t.dtype == 1 for t in cfg.tables):
            sync_rows(ctx, orc, cfg, od[0])
    ctx.close()
    orc.close()


def sampled_step_check(binding, workload_mod, oracle_mod, w, n_bags=4096, n_rows=2048, seed=0):
    """Full-size parity on sampled outputs (for workloads whose full oracle run would take minutes).

    One forward + backward step of workload w on the GPU; the oracle then recomputes, from the paper's
    definitions, (a) the pooled vectors of `n_bags` sampled bags, (b) the updated rows, accumulators and
    bag lists of `n_rows` sampled unique rows -- a row's gradient depends only on its own occurrences, so
    a sub-batch that keeps exactly those occurrences gives the exact update -- and (c) the whole set of
    unique keys and segment offsets, which numpy derives from the oracle's hash of every id.
    """
    import torch
    cfg = w.cfg
    S = cfg.num_slots
    b = workload_mod.make_batch(w, 0)
    ctx = binding.EmbContext.from_config(cfg, max_batch=b.batch_size, max_ids=b.num_ids)
    db = binding.DeviceBatch(b.batch_size, b.ids, b.offsets)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1234 + w.index)
    dp_dev = torch.randn((b.batch_size, cfg.pooled_width), generator=gen, device="cuda", dtype=torch.float32)
    pooled = ctx.emb_lookup_pool(db)
    torch.cuda.synchronize()
    pooled = pooled.cpu().numpy()
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

    def sub_batch(keep_occ):
        """CSR with the same bags, holding only the occurrences flagged in keep_occ."""
        kept_per_bag = np.bincount(bag_of[keep_occ], minlength=n_all_bags)
        off = np.zeros(n_all_bags + 1, dtype=np.int64)
        np.cumsum(kept_per_bag, out=off[1:])
        return b.ids[keep_occ], off.astype(np.int32)

    # (a) pooled vectors of sampled bags
    pick = rng.choice(n_all_bags, size=min(n_bags, n_all_bags), replace=False)
    keep = np.zeros(n_all_bags, dtype=bool)
    keep[pick] = True
    ids_s, off_s = sub_batch(keep[bag_of])
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
    ids_s, off_s = sub_batch(keep_occ)
    orc2 = oracle_mod.Oracle.from_config(cfg, dense=False)
    ok, oo, ob = orc2.backward_update(ids_s, off_s, dp)
    np.testing.assert_array_equal(ok, sample_keys)
    for j, u in enumerate(sample_u):                      # bag list of each sampled key, bit-exact
        np.testing.assert_array_equal(gb[go[u]:go[u + 1]], ob[oo[j]:oo[j + 1]])
    compare_rows(ctx, orc2, cfg, sample_keys, extra_rows=256, seed=seed, all_touched=uk)
    orc2.close()
    ctx.close()
