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


def compare_rows(ctx, orc, cfg, keys, extra_rows=64, seed=0):
    """Touched rows (and their accumulators) within tolerance; a sample of other rows bit-exact."""
    tables = (keys >> np.uint64(32)).astype(np.int64)
    rows = keys & LOW32
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
        probe = np.setdiff1d(probe, r)
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


def run_steps(binding, workload_mod, oracle_mod, w, steps=1, dense=None, batches=None, grads=None, check_hash=True):
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
    ctx = binding.EmbContext.from_config(cfg, max_batch=max(max_b, 1), max_ids=max_ids)
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
