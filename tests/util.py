"""Shared helpers of the GPU parity tests: run one batch through the HIP library and through the
CPU oracle on the same seeded inputs and compare element by element."""
import numpy as np

# spec tolerances: fp32 tables 1e-5 relative + 1e-6 absolute; bf16 storage 2e-2 relative
TOL = {0: dict(rtol=1e-5, atol=1e-6), 1: dict(rtol=2e-2, atol=1e-6)}
LOW32 = np.uint64(0xFFFFFFFF)
# A sum of fp32 terms formed in fp32 (in any order, compensated or not) carries an error of a few units in the last
# place of its LARGEST partial sum, which no bound relative to the result covers when the terms cancel.  The
# comparisons below therefore allow, on top of the spec bar, SUM_EPS times the sum of the terms' magnitudes:
# 8 roundings of 2^-24 (the kernels add at most 8 terms before a compensated step).  At the benchmark's value
# ranges (rows of ~1e-2) this is ~1e-8 and plays no part; it matters only in the stress tests, whose rows and
# steps are hundreds of times larger.
SUM_EPS = 8.0 * 2.0 ** -24


def tol_for(cfg):
    return TOL[1] if any(t.dtype == 1 for t in cfg.tables) else TOL[0]


def assert_close(got, want, rtol, atol, slack=None, err_msg=""):
    """|got - want| <= atol + rtol |want| (+ slack, elementwise)."""
    got, want = np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64)
    bound = atol + rtol * np.abs(want)
    if slack is not None:
        bound = bound + slack
    bad = ~(np.abs(got - want) <= bound)       # NaNs count as bad
    if bad.any():
        i = np.unravel_index(np.argmax(np.where(bad, np.abs(got - want) - bound, -np.inf)), got.shape)
        raise AssertionError(f"{err_msg}: {int(bad.sum())} of {bad.size} elements outside the bound; worst at {i}: "
                             f"got {got[i]!r}, want {want[i]!r}, bound {bound[i] if np.ndim(bound) else bound!r}")


def compare_pooled(got, want, cfg, slack=None):
    assert_close(got, want, **tol_for(cfg), slack=slack, err_msg="pooled")


def pooled_magnitudes(orc, cfg, b):
    """Sum of |row| over the rows each pooled element is made of, [B, pooled width] (numpy, for small batches):
    read from the oracle's tables as they stand."""
    S = cfg.num_slots
    cols, dims = np.array(cfg.slot_cols()), np.array(cfg.slot_dims())
    slot_table = np.array([s.table for s in cfg.slots])
    out = np.zeros((b.batch_size, cfg.pooled_width), dtype=np.float64)
    if b.num_ids == 0:
        return out
    rows = orc.hash_rows(b.ids, b.offsets).astype(np.uint64)
    lens = np.diff(b.offsets.astype(np.int64))
    bag_of = np.repeat(np.arange(len(lens)), lens)
    for t in range(len(cfg.tables)):
        sel = np.flatnonzero(slot_table[bag_of % S] == t)
        if not len(sel):
            continue
        ur, inv = np.unique(rows[sel], return_inverse=True)
        w_abs = np.abs(orc.read_rows(t, ur)[0].astype(np.float64))[inv]          # [n_t, D_t]
        bb, ss = bag_of[sel] // S, bag_of[sel] % S
        D = cfg.tables[t].dim
        for d in range(D):
            np.add.at(out, (bb, cols[ss] + d), w_abs[:, d])
    return out


def gradient_magnitudes(cfg, index_form, dp):
    """For each unique key of the index form: max over the row's elements of the sum of |upstream gradient| over
    the key's occurrences (numpy, for small batches)."""
    keys, seg_off, bags = index_form
    S = cfg.num_slots
    cols = np.array(cfg.slot_cols())
    out = np.zeros(len(keys), dtype=np.float64)
    tables = (keys >> np.uint64(32)).astype(np.int64)
    seg_off = seg_off.astype(np.int64)
    absdp = np.abs(dp.astype(np.float64))
    for u in range(len(keys)):
        D = cfg.tables[tables[u]].dim
        bg = bags[seg_off[u]:seg_off[u + 1]].astype(np.int64)
        bb, ss = bg // S, bg % S
        acc = np.zeros(D)
        for b_, s_ in zip(bb, ss):
            acc += absdp[b_, cols[s_]:cols[s_] + D]
        out[u] = acc.max() if D else 0.0
    return out


def compare_dedup(gpu, orc):
    """Index form of the batch: integers, bit-exact."""
    gk, go, gb = gpu
    ok, oo, ob = orc
    assert len(gk) == len(ok), f"U differs: gpu {len(gk)} oracle {len(ok)}"
    np.testing.assert_array_equal(gk, ok)
    np.testing.assert_array_equal(go, oo)
    np.testing.assert_array_equal(gb, ob)


def compare_rows(ctx, orc, cfg, keys, extra_rows=64, seed=0, all_touched=None, grad_mag=None):
    """Touched rows (and their accumulators) within tolerance; a sample of other rows bit-exact.
    all_touched: every key the GPU batch touched, when `keys` is only a sample of them.
    grad_mag: per key (aligned with `keys`), the value gradient_magnitudes gives; widens the bound by what
    SUM_EPS * grad_mag in the summed gradient can do to the row and to its accumulator (tolerances)."""
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
            slack_w = slack_a = None
            if grad_mag is not None:
                gm = grad_mag[tables == t]
                delta = SUM_EPS * gm                                   # error of an element of the summed gradient
                if cfg.opt == 0:                                        # w' = w - lr G
                    slack_w = (cfg.lr * delta)[:, None]
                else:                                                   # a' = a + mean G^2; w' = w - lr G / (sqrt a' + eps)
                    step = cfg.lr / (np.sqrt(oa.astype(np.float64)) + cfg.eps)
                    slack_w = (step * (1.0 + np.sqrt(td.dim)) * delta)[:, None]
                    slack_a = 2.0 * gm * delta + delta * delta
            assert_close(gw, ow, **tol, slack=slack_w, err_msg=f"table {t} rows")
            assert_close(ga, oa, rtol=1e-5, atol=1e-6, slack=slack_a, err_msg=f"table {t} accumulators")
        probe = rng.integers(0, td.rows, size=extra_rows, dtype=np.uint64)
        probe = np.setdiff1d(probe, at_rows[at_tables == t])
        if len(probe):
            gw, ga = ctx.emb_read_rows(t, probe)
            ow, oa = orc.read_rows(t, probe)
            np.testing.assert_array_equal(gw, ow, err_msg=f"table {t}: a row outside the batch changed")
            np.testing.assert_array_equal(ga, oa)


def sync_rows(ctx, orc, cfg, keys):
    """After a step has been compared, copy the oracle's rows into the GPU table.  A row on which the two sides
    differ within the bar (neighbouring bf16 values; a few fp32 units in the last place) would otherwise show up
    in the next step's pooled sums, where cancellation can magnify it beyond any bound relative to the result;
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
        small = b.num_ids <= 50000        # the magnitude terms of the bound are computed in numpy
        pooled = ctx.emb_lookup_pool(db)
        torch.cuda.synchronize()
        compare_pooled(pooled.cpu().numpy(), orc.lookup_pool(b.ids, b.offsets), cfg,
                       slack=SUM_EPS * pooled_magnitudes(orc, cfg, b) if small else None)
        ctx.emb_backward_update(db, torch.from_numpy(dp).cuda())
        gd = ctx.emb_read_dedup()
        od = orc.backward_update(b.ids, b.offsets, dp)
        compare_dedup(gd, od)
        touched.append(od[0])
        if small:   # this step's rows with the widened bound, every row touched so far (re-aligned below) flat
            compare_rows(ctx, orc, cfg, od[0], grad_mag=gradient_magnitudes(cfg, od, dp))
        else:
            compare_rows(ctx, orc, cfg, np.unique(np.concatenate(touched)))
        if small or any(t.dtype == 1 for t in cfg.tables):
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
