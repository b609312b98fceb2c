#!/usr/bin/env python3
"""Benchmark of the embedding hot path on one MI355X.

A step = one pass of the whole path (emb_lookup_pool, then emb_backward_update: hash, gather +
sum-pool, key build, radix-sort dedup, segmented gradient reduce, fused row-wise optimizer) over one
synthetic batch that is already resident in HBM.  Prints ONE JSON line with the throughput in
embedding IDs/s, the roofline figure of the dominant kernel (algorithmic bytes per launch / average
launch time from HIP events on the launch stream) and the CPU oracle timed beside it.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth


def algorithmic_bytes(tables):
    """Bytes the method itself must move per step, per kernel stage and for the whole step, under two models.
    `tables`: one dict per table with N (ids hashed into it), bags (bags reading it), U (unique rows), Um (unique
    rows whose segment spans tiles), D (dim), e (bytes per stored element).  Kernels that run once per table sum
    over tables.  Sort passes and partial sums are implementation overhead and are counted in neither model.

    "occurrence": every occurrence of an id reads its table row (forward) and its bag's gradient row (backward) --
    the traffic the kernels request; rows and gradient rows that occur several times are counted every time,
    although caches serve the repeats, so this figure can exceed what HBM delivers (and the 8 TB/s peak).
    "compulsory": every distinct byte once -- each unique row read once in the forward, each gradient row read
    once in the backward: a lower bound of the HBM traffic, hence of the HBM fraction."""
    keys = ("gather_pool", "build_keys", "reduce_update", "fixup", "step")
    occ, comp = dict.fromkeys(keys, 0.0), dict.fromkeys(keys, 0.0)
    for t in tables:
        N, bags, U, Um, D, e = t["N"], t["bags"], t["U"], t["Um"], t["D"], t["e"]
        csr = 8 * N + 4 * (bags + 1)                                  # ids + offsets
        for m, rows_fwd, grads in ((occ, N * D * e, N * D * 4), (comp, U * D * e, bags * D * 4)):
            m["gather_pool"] += csr + rows_fwd + bags * D * 4         # row gathers, pooled write
            m["build_keys"] += csr + 8 * N                            # ids re-read, (key, bag) pairs written
            m["reduce_update"] += 8 * N + grads + (U - Um) * (2 * D * e + 8)   # sorted pairs, gradient rows, row + acc RMW
            m["fixup"] += Um * (2 * D * e + 8)                        # rows of segments that span tiles
            m["step"] += csr + rows_fwd + bags * D * 4 + 4 * N + 8 * N + 8 * U + grads + U * (2 * D * e + 8)
    return occ, comp


def cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown CPU"


def host_mem_available_gb() -> float:
    try:
        for line in open("/proc/meminfo"):
            if line.startswith("MemAvailable"):
                return int(line.split()[1]) / (1 << 20)
    except OSError:
        pass
    return 0.0


def read_traffic_profile(path):
    """The committed rocprofv3 --pmc summary of a workload: ({stage: bytes}, ids, unique rows, launches-per-step note) or None."""
    if not os.path.exists(path):
        return None
    traffic, meta = {}, {}
    for line in open(path):
        f = line.split()
        if len(f) == 3 and f[0] == "traffic_per_step":
            traffic[f[1]] = int(f[2])
        elif len(f) == 3 and f[0] == "workload":
            meta[f[1]] = int(f[2])
    return traffic, meta


def bench_codec(args, w, binding, torch, np) -> int:
    """Compress + decompress of one batch of pooled activations, one block per slot vector (section 4.2.3)."""
    width = w.cfg.pooled_width
    block_len = w.cfg.tables[0].dim
    gen = torch.Generator(device="cuda")
    gen.manual_seed(w.seed)
    v = torch.randn((w.batch, width), generator=gen, device="cuda", dtype=torch.float32) * 0.05
    n = v.numel()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    for _ in range(args.warmup):
        q, norm = binding.emb_codec_compress(v, block_len)
        binding.emb_codec_decompress(q, norm)
    torch.cuda.synchronize()
    t_c = t_d = 0.0
    for _ in range(args.steps):
        ev[0].record()
        q, norm = binding.emb_codec_compress(v, block_len)
        ev[1].record()
        out = binding.emb_codec_decompress(q, norm)
        ev[2].record()
        torch.cuda.synchronize()
        t_c += ev[0].elapsed_time(ev[1])
        t_d += ev[1].elapsed_time(ev[2])
    t_c, t_d = t_c / args.steps, t_d / args.steps
    bytes_c = 4 * n + 2 * n + 4 * (n // block_len)      # fp32 read, fp16 + norm written
    bytes_d = 2 * n + 4 * (n // block_len) + 4 * n      # fp16 + norm read, fp32 written
    out_line = {
        "metric": "value codec throughput (compress + decompress), 1 GPU", "value": round(n / ((t_c + t_d) * 1e-3), 1),
        "unit": "values/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(t_c + t_d, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32->f16", "data": "synthetic",
        "config": {"workload": w.name + "_pooled_codec", "values": n, "block_len": block_len, "kappa": 2.0 ** 15},
        "roofline": {"bound": "hbm", "kernel": "codec_compress", "achieved": round(bytes_c / (t_c * 1e-3) / 1e9, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(bytes_c / (t_c * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                     "traffic": None, "avg_launch_ms": round(t_c, 4), "algorithmic_bytes_per_launch": bytes_c},
        "decompress": {"achieved_GBps": round(bytes_d / (t_d * 1e-3) / 1e9, 1), "avg_launch_ms": round(t_d, 4)},
    }
    print(json.dumps(out_line))
    return 0


def bench_gemm(args, binding, torch) -> int:
    """The bf16 MFMA contraction of the dense step on its own, on the shapes config 3's step is made of
    (batch 32768; C = A * Bt^T, operands already resident in HBM)."""
    shapes = [("forward layer 1", 0, 32768, 4096, 10432), ("forward layer 2", 0, 32768, 2048, 4096),
              ("weight gradient layer 1", 1, 10432, 4096, 32768), ("delta layer 1", 2, 32768, 4096, 2048),
              ("gradient of the pooled activations", 1, 32768, 9920, 4096)]
    out = []
    for name, epi, M, N, K in shapes:
        A = (torch.randn(M, K, device="cuda") * 0.1).to(torch.bfloat16)
        Bt = (torch.randn(N, K, device="cuda") * 0.1).to(torch.bfloat16)
        bias = torch.zeros(N, device="cuda")
        mask = torch.ones(M, N, device="cuda", dtype=torch.bfloat16) if epi == 2 else None
        for _ in range(max(args.warmup, 1)):
            binding.mlp_gemm_nt(epi, A, Bt, bias, mask)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            binding.mlp_gemm_nt(epi, A, Bt, bias, mask)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        # the vendor library's plain product of the same operands (no epilogue), through torch.matmul: a reference
        # beside the figure, not part of the path
        for _ in range(max(args.warmup, 1)):
            torch.matmul(A, Bt.t())
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            torch.matmul(A, Bt.t())
        e1.record()
        torch.cuda.synchronize()
        lib_ms = e0.elapsed_time(e1) / args.steps
        out.append({"product": name, "epilogue": epi, "M": M, "N": N, "K": K, "ms": round(ms, 4),
                    "TFLOPs": round(2.0 * M * N * K / ms / 1e9, 1),
                    "library_reference_TFLOPs": round(2.0 * M * N * K / lib_ms / 1e9, 1)})
        del A, Bt, mask
    best = max(o["TFLOPs"] for o in out)
    print(json.dumps({"metric": "bf16 MFMA contraction C = A * Bt^T (fp32 accumulation), 1 GPU", "unit": "TFLOP/s",
                      "n_gpus": 1, "steps": args.steps, "dtype": "bf16", "data": "synthetic", "products": out,
                      "roofline": {"bound": "mfma", "achieved": best, "peak": 2500.0, "unit": "TFLOP/s",
                                   "frac": round(best / 2500.0, 4), "traffic": None}}))
    return 0


def bench_indexed_forward(args, w, binding, torch, np, W) -> int:
    """The forward two ways on one batch: gather per bag (emb_lookup_pool) and from the index form, each unique
    row read once (emb_lookup_pool_indexed; the index form is built beforehand, outside the timed region, as if
    the batch had arrived compressed)."""
    cfg = w.cfg
    hb = W.make_batch(w, 0)
    b = binding.DeviceBatch(hb.batch_size, hb.ids, hb.offsets)
    ctx = binding.EmbContext.from_config(cfg, max_batch=w.batch, max_ids=b.num_ids)
    pooled = torch.empty((w.batch, cfg.pooled_width), dtype=torch.float32, device="cuda")
    ctx.emb_backward_update(b, torch.zeros_like(pooled))       # zero gradient: builds the index form, changes no row
    keys, seg_off, seg_bags = ctx.emb_read_dedup()
    dk = torch.from_numpy(keys.view(np.int64)).cuda()
    do = torch.from_numpy(seg_off.view(np.int32)).cuda()
    dbg = torch.from_numpy(seg_bags.view(np.int32)).cuda()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    for _ in range(args.warmup):
        ctx.emb_lookup_pool(b, pooled)
        ctx.emb_lookup_pool_indexed(w.batch, dk, do, dbg, pooled)
    torch.cuda.synchronize()
    ev[0].record()
    for _ in range(args.steps):
        ctx.emb_lookup_pool(b, pooled)
    ev[1].record()
    for _ in range(args.steps):
        ctx.emb_lookup_pool_indexed(w.batch, dk, do, dbg, pooled)
    ev[2].record()
    torch.cuda.synchronize()
    t_g, t_i = ev[0].elapsed_time(ev[1]) / args.steps, ev[1].elapsed_time(ev[2]) / args.steps
    print(json.dumps({"metric": "forward, ms per batch", "workload": w.name, "ids": b.num_ids, "unique_rows": int(len(keys)),
                      "gather_per_bag_ms": round(t_g, 4), "from_index_form_ms": round(t_i, 4), "steps": args.steps,
                      "n_gpus": 1, "data": "synthetic"}))
    ctx.close()
    return 0


def bench_hybrid(args, w, binding, torch, np, W) -> int:
    """emb_lookup_pool -> mlp_step -> emb_backward_update(d_pooled from the MLP), one stream, synchronous."""
    cfg = w.cfg
    P = cfg.pooled_width
    widths = [P + W.DENSE_FEATURES] + W.MLP_HIDDEN + [1]
    nb = max(1, min(args.distinct_batches or 2, args.steps, 2))
    host_batches = [W.make_batch(w, s) for s in range(nb)]
    batches = [binding.DeviceBatch(b.batch_size, b.ids, b.offsets) for b in host_batches]
    feats = []
    for s in range(nb):
        d, y = W.make_dense_and_labels(w.seed, s, w.batch)
        feats.append((torch.from_numpy(d).cuda(), torch.from_numpy(y).cuda()))
    Ws, bs = W.make_mlp_params(widths, w.seed)
    ctx = binding.EmbContext.from_config(cfg, max_batch=w.batch, max_ids=max(b.num_ids for b in batches))
    mlp = binding.MlpContext(widths, P, W.DENSE_FEATURES, w.batch, 1e-3, Ws, bs, loss_mean=True)
    pooled = torch.empty((w.batch, P), dtype=torch.float32, device="cuda")
    d_pooled = torch.empty_like(pooled)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    t_emb_f = t_mlp = t_emb_b = 0.0
    ids_done = 0
    torch.cuda.synchronize()

    def step(i, timed):
        nonlocal t_emb_f, t_mlp, t_emb_b
        b = batches[i % nb]
        d, y = feats[i % nb]
        ev[0].record()
        ctx.emb_lookup_pool(b, pooled)
        ev[1].record()
        _, loss = mlp.mlp_step(pooled, d, y, d_pooled)
        ev[2].record()
        ctx.emb_backward_update(b, d_pooled)
        ev[3].record()
        if timed:
            torch.cuda.synchronize()
            t_emb_f += ev[0].elapsed_time(ev[1]); t_mlp += ev[1].elapsed_time(ev[2]); t_emb_b += ev[2].elapsed_time(ev[3])
        return b.num_ids, loss

    for i in range(args.warmup):
        step(i, False)
    torch.cuda.synchronize()
    if args.tau is None:
        t0 = time.perf_counter()
        for i in range(args.steps):
            n, loss = step(args.warmup + i, False)
            ids_done += n
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
    else:
        # the library's step loop: lookups run tau batches ahead of the dense step, on a second stream; the timed
        # region starts with tau lookups in flight and ends with tau in flight, so it holds `steps` whole steps
        loop = binding.HybridLoop(ctx, mlp, args.tau)
        for i in range(args.tau + args.warmup):
            loop.hyb_submit(batches[i % nb], *feats[i % nb])
        loop.hyb_sync()
        t0 = time.perf_counter()
        for i in range(args.steps):
            j = args.tau + args.warmup + i
            loop.hyb_submit(batches[j % nb], *feats[j % nb])
            ids_done += batches[(j - args.tau) % nb].num_ids
        loop.hyb_sync()
        elapsed = time.perf_counter() - t0
        loop.hyb_drain()
        n_trained = loop.hyb_counts()[1]
        loss = torch.tensor(loop.hyb_read_losses(n_trained - 1, 1))
        loop.close()
    for i in range(args.steps):
        step(args.warmup + i, True)
    B = w.batch
    hidden = widths[1:-1]
    flops = 0.0
    prev = widths[0]
    for j, hsz in enumerate(hidden):
        flops += 2.0 * B * prev * hsz            # forward
        flops += 2.0 * B * prev * hsz            # weight gradient
        flops += 2.0 * B * (P if j == 0 else prev) * hsz   # input gradient (first layer: pooled columns only)
        prev = hsz
    flops += 3 * 2.0 * B * prev                  # the logit layer
    mlp_ms = t_mlp / args.steps
    tflops = flops / (mlp_ms * 1e-3) / 1e12
    out = {
        "metric": "embedding IDs/sec (lookup + dense MLP step + bwd + update), 1 GPU", "value": round(ids_done / elapsed, 1),
        "unit": "IDs/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(elapsed * 1e3 / args.steps, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name + "_hybrid", "schedule": "sync" if args.tau is None else f"staleness-{args.tau} loop", "batch": B, "slots": cfg.num_slots, "mlp_widths": widths,
                   "ids_per_step": round(ids_done / args.steps), "last_loss": round(float(loss.item()), 5)},
        "part_ms_per_step": {"emb_lookup_pool": round(t_emb_f / args.steps, 4), "mlp_step": round(mlp_ms, 4),
                             "emb_backward_update": round(t_emb_b / args.steps, 4)},
        "roofline": {"bound": "mfma", "kernel": "mlp_step (all bf16 contractions, transposes and epilogues)",
                     "achieved": round(tflops, 1), "peak": 2500.0, "unit": "TFLOP/s", "frac": round(tflops / 2500.0, 4),
                     "traffic": None, "flop_per_step": flops},
    }
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="benchmark configuration 0..4 (2 = the headline workload: 100 slots, 2^26 rows, fp32 D=64)")
    ap.add_argument("--distinct-batches", type=int, default=0,
                    help="synthetic batches generated and cycled (0 = the workload's own loop length, 10 for the headline workload, else 4)")
    ap.add_argument("--min-seconds", type=float, default=1.0, help="the timed region runs at least this long")
    ap.add_argument("--min-reps", type=int, default=20, help="... and holds at least this many repetitions of --steps steps")
    ap.add_argument("--max-reps", type=int, default=400)
    ap.add_argument("--cpu-dense-gb", type=float, default=40.0,
                    help="the oracle is timed on whole (dense) tables up to this size, on touched-rows-only tables beyond")
    ap.add_argument("--overlap", action="store_true",
                    help="staleness-1 schedule: lookup(t+1) on a second stream while update(t) runs on the first")
    ap.add_argument("--codec", action="store_true",
                    help="instead of the training step, time the scaled-fp16 value codec on this config's pooled shape")
    ap.add_argument("--hybrid", action="store_true",
                    help="full hybrid step: lookup -> dense MLP step (bf16 MFMA) -> embedding update with the MLP's gradient")
    ap.add_argument("--gemm", action="store_true",
                    help="instead of the training step, time the dense step's bf16 MFMA contraction on config 3's shapes")
    ap.add_argument("--indexed-forward", action="store_true",
                    help="instead of the training step, time the forward per bag against the forward from the index form")
    ap.add_argument("--tau", type=int, default=None,
                    help="with --hybrid: run the library's step loop with this staleness (lookups tau batches ahead, second stream)")
    ap.add_argument("--cache-frac", type=float, default=None,
                    help="keep the tables in pinned host memory with this fraction of their rows cached in HBM (LRU)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain 1 GiB device-to-device copies (reference for rocprofv3 byte counters)")
    ap.add_argument("--cpu-samples", type=int, default=0, help="samples of batch 0 the oracle is timed on (0 = all, or as many as hold about 30 M ids)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2111_05897_amd import binding, workload as W

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    binding.load_library()
    w = W.make_workload(args.config)
    cfg = w.cfg
    if args.gemm:
        return bench_gemm(args, binding, torch)
    if args.codec:
        return bench_codec(args, w, binding, torch, np)
    if args.hybrid:
        return bench_hybrid(args, w, binding, torch, np, W)
    if args.indexed_forward:
        return bench_indexed_forward(args, w, binding, torch, np, W)
    if args.overlap and args.cache_frac is not None:
        print("bench.py: --overlap and --cache-frac exclude each other: calls on a context whose tables sit behind the "
              "cache share its admission state and must not overlap", file=sys.stderr)
        return 2
    T = len(cfg.tables)
    e_of = [2 if t.dtype == W.BF16 else 4 for t in cfg.tables]
    slot_table = np.array([s.table for s in cfg.slots])
    # distinct synthetic batches, cycled; the headline workload is a loop over 10 different batches
    want_nb = args.distinct_batches if args.distinct_batches else (w.steps if w.steps > 1 else 4)
    nb = max(1, min(want_nb, max(args.steps, 1)))
    t0 = time.time()
    host_batches = [W.make_batch(w, s) for s in range(nb)]
    batches = [binding.DeviceBatch(b.batch_size, b.ids, b.offsets) for b in host_batches]
    gen = torch.Generator(device="cuda")
    grads = []
    for s in range(nb):
        gen.manual_seed(w.seed * 1000 + s)
        grads.append(torch.randn((w.batch, cfg.pooled_width), generator=gen, device="cuda", dtype=torch.float32))
    max_ids = max(b.num_ids for b in batches)
    cache_rows = None
    if args.cache_frac is not None:
        # tables in pinned host memory, this fraction of their rows cached in HBM (at least one batch's worst case)
        cache_rows = [max(min(t.rows, max_ids), int(args.cache_frac * t.rows)) for t in cfg.tables]
        cache_rows = [c if c < t.rows else 0 for c, t in zip(cache_rows, cfg.tables)]
    ctx = binding.EmbContext.from_config(cfg, max_batch=w.batch, max_ids=max_ids, cache_rows=cache_rows)
    pooled = torch.empty((w.batch, cfg.pooled_width), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    setup_s = time.time() - t0

    def step(i):
        b = batches[i % nb]
        ctx.emb_lookup_pool(b, pooled)
        ctx.emb_backward_update(b, grads[i % nb])
        return b.num_ids

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.overlap:
        s_upd, s_look = torch.cuda.Stream(), torch.cuda.Stream()   # both at the default priority
        pooled2 = [pooled, torch.empty_like(pooled)]

    def run_overlapped(first, count):
        """lookup(t+1) on s_look overlaps update(t) on s_upd; lookup(t+1) waits for update(t-1), update(t) for
        lookup(t): the embedding read is at most one update stale (section 5, tau = 1)."""
        ids = 0
        ev_f = [torch.cuda.Event() for _ in range(count + 1)]
        ev_b = [torch.cuda.Event() for _ in range(count)]
        ctx.emb_lookup_pool(batches[first % nb], pooled2[0], stream=s_look)
        ev_f[0].record(s_look)
        for t in range(count):
            if t + 1 < count:
                if t >= 1:
                    s_look.wait_event(ev_b[t - 1])
                ctx.emb_lookup_pool(batches[(first + t + 1) % nb], pooled2[(t + 1) % 2], stream=s_look)
                ev_f[t + 1].record(s_look)
            s_upd.wait_event(ev_f[t])
            b = batches[(first + t) % nb]
            ctx.emb_backward_update(b, grads[(first + t) % nb], stream=s_upd)
            ev_b[t].record(s_upd)
            ids += b.num_ids
        return ids

    # ---- the timed region.  One repetition = exactly --steps steps (the 10-step loop of the headline workload with
    # the default flags), bracketed by HIP events on the stream the kernels run on; the repetitions follow each other
    # without a gap or a synchronisation until the region has run for at least --min-seconds (and at least
    # --min-reps times), so that the clock has settled to what a sustained run gets.  The figure reported is the
    # MEDIAN repetition; the whole region is bracketed by synchronisations and a wall clock as well.
    K = args.steps
    if args.overlap:
        torch.cuda.synchronize()
        run_overlapped(0, max(args.warmup, 1))
        torch.cuda.synchronize()
    else:
        for i in range(args.warmup):
            step(i)
        torch.cuda.synchronize()
    # one untimed repetition to size the region
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    if args.overlap:
        run_overlapped(args.warmup, K)
        torch.cuda.current_stream().wait_stream(s_upd)
    else:
        for i in range(K):
            step(args.warmup + i)
    e1.record()
    torch.cuda.synchronize()
    est_ms = max(e0.elapsed_time(e1), 1e-3)
    # (+1: the sizing repetition is often a little slower than the settled ones, and the region must not end short)
    reps = int(min(max(args.min_reps, np.ceil(args.min_seconds * 1e3 / est_ms) + 1), args.max_reps))
    cur = torch.cuda.current_stream()
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
    ids_rep = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    evs[0].record(cur)
    for r in range(reps):
        if args.overlap:
            s_look.wait_stream(cur)
            s_upd.wait_stream(cur)
            n_ids = run_overlapped(args.warmup + r * K, K)
            cur.wait_stream(s_upd)
            cur.wait_stream(s_look)
        else:
            n_ids = 0
            for i in range(K):
                n_ids += step(args.warmup + r * K + i)
        ids_rep.append(n_ids)
        evs[r + 1].record(cur)
    torch.cuda.synchronize()
    wall_s = time.perf_counter() - t0
    rep_ms = np.array([evs[r].elapsed_time(evs[r + 1]) for r in range(reps)])
    med = int(np.argsort(rep_ms)[len(rep_ms) // 2])
    ms_per_step = float(rep_ms[med]) / K
    ids_per_s = ids_rep[med] / (float(rep_ms[med]) * 1e-3)
    cache_report = None
    if cache_rows is not None and any(cache_rows):
        cache_report = []
        calls = args.warmup + K * (reps + 1)
        for t, c in enumerate(cache_rows):
            if c:
                st = ctx.emb_cache_stats(t)
                row_bytes = cfg.tables[t].dim * e_of[t] + 4
                cache_report.append({"table": t, "cache_rows": c, "rows": cfg.tables[t].rows, **st,
                                     "hit_rate": round(1.0 - st["misses"] / max(st["requested"], 1), 4),
                                     "host_link_bytes_per_step": round((st["misses"] + st["written_back"]) * row_bytes / calls)})

    # ---- per-kernel timing pass: the same steps once more with every kernel stage bracketed by HIP events on the
    # launch stream inside the library (the events themselves cost a little, so the stages add up to slightly more
    # than a step of the region above)
    ctx.emb_set_profiling(True)
    ctx.emb_reset_stage_ms()
    N_t, U_t, Um_t = np.zeros(T), np.zeros(T), np.zeros(T)
    tile = int(binding.load_library().emb_tile_entries())   # segments crossing a tile edge are finished by the fix-up
    N_sum = 0
    prof_steps = max(K, nb)
    for i in range(prof_steps):
        N_sum += step(args.warmup + i)
        keys, seg_off, _ = ctx.emb_read_dedup()
        s_, en = seg_off[:-1].astype(np.int64), seg_off[1:].astype(np.int64)
        kt = (keys >> np.uint64(32)).astype(np.int64)
        U_t += np.bincount(kt, minlength=T)
        Um_t += np.bincount(kt[s_ // tile != (en - 1) // tile], minlength=T)
        N_t += np.bincount(kt, weights=(en - s_), minlength=T)
    stages = ctx.emb_read_stage_ms()
    ctx.emb_set_profiling(False)
    N_avg, U_avg = N_sum / prof_steps, float(U_t.sum()) / prof_steps
    occ, comp = algorithmic_bytes([{"N": N_t[t] / prof_steps, "bags": w.batch * int((slot_table == t).sum()),
                                    "U": U_t[t] / prof_steps, "Um": Um_t[t] / prof_steps, "D": cfg.tables[t].dim,
                                    "e": e_of[t]} for t in range(T)])
    per_step_ms = {k: ms / prof_steps for k, (ms, c) in stages.items() if c}
    launches = {k: c / prof_steps for k, (ms, c) in stages.items() if c}
    dom = max((k for k in per_step_ms if k in occ), key=lambda k: per_step_ms[k])

    def gbps(nbytes, ms):
        return nbytes / (ms * 1e-3) / 1e9

    # launches of a stage that run once per table are taken together: bytes of all / time of all
    achieved = gbps(occ[dom], per_step_ms[dom])
    achieved_c = gbps(comp[dom], per_step_ms[dom])
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                "avg_launch_ms": round(per_step_ms[dom] / launches[dom], 4),
                "algorithmic_bytes_per_launch": int(occ[dom] / launches[dom]),
                "bytes_model": "occurrence: every id occurrence reads its table row / its bag's gradient row; repeats that "
                               "caches serve are counted, so this is delivered (effective) bandwidth and may exceed HBM's",
                "achieved_compulsory": round(achieved_c, 1), "frac_compulsory": round(achieved_c / HBM_PEAK_GBS, 4),
                "compulsory_bytes_per_launch": int(comp[dom] / launches[dom]),
                "compulsory_model": "every distinct byte once (unique rows, each gradient row once): a lower bound of "
                                    "the HBM traffic and of the HBM fraction"}
    # bytes between L2 and the fabric from the committed rocprofv3 --pmc summary of this workload (FETCH_SIZE and
    # WRITE_SIZE runs of this script, scaled by a plain copy of known size).  They are that earlier run's bytes, not
    # this run's: used only if the summary was taken on the same ids / unique rows per step, else null.
    prof = read_traffic_profile(os.path.join(ROOT, "profiles", f"{w.name}_hbm_traffic.txt"))
    profile_step_bytes = None
    if prof is not None and not args.overlap and cache_report is None:
        traffic, meta = prof
        same = (abs(meta.get("ids_per_step", -1) - N_avg) <= 0.01 * N_avg and
                abs(meta.get("unique_rows_per_step", -1) - U_avg) <= 0.01 * U_avg)
        if same and dom in traffic:
            roofline["traffic"] = int(traffic[dom] / launches[dom])     # per launch, like `achieved`
            profile_step_bytes = sum(traffic.values())

    out = {
        "metric": "embedding IDs/sec (lookup+bwd+update), 1 GPU", "value": round(ids_per_s, 1), "unit": "IDs/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64 sums and optimizer; " + ("f32" if all(x == 4 for x in e_of) else "bf16") + " table storage",
        "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "slots": cfg.num_slots,
                   "rows": [t.rows for t in cfg.tables], "dim": [t.dim for t in cfg.tables],
                   "ids_per_step": round(N_avg), "unique_rows_per_step": round(U_avg),
                   "distinct_batches": nb, "optimizer": "rowwise_adagrad" if cfg.opt else "sgd",
                   "schedule": "staleness-1 overlap, two streams" if args.overlap else "synchronous, one stream"},
        "timing": {"protocol": f"median of {reps} back-to-back repetitions of {K} steps each (HIP events on the launch "
                               f"stream), after {args.warmup} warm-up steps and one untimed repetition",
                   "repetitions": reps, "timed_region_s": round(float(rep_ms.sum()) * 1e-3, 3), "wall_s": round(wall_s, 3),
                   "rep_ms_min": round(float(rep_ms.min()), 4), "rep_ms_median": round(float(rep_ms[med]), 4),
                   "rep_ms_max": round(float(rep_ms.max()), 4),
                   "ms_per_step_mean": round(float(rep_ms.sum()) / (reps * K), 4)},
        "effective_GBps_step": round(gbps(occ["step"], ms_per_step), 1),
        "effective_frac_of_hbm_peak": round(gbps(occ["step"], ms_per_step) / HBM_PEAK_GBS, 4),
        "compulsory_GBps_step": round(gbps(comp["step"], ms_per_step), 1),
        "compulsory_frac_of_hbm_peak": round(gbps(comp["step"], ms_per_step) / HBM_PEAK_GBS, 4),
        # the committed profile's L2<->fabric bytes of a whole step over this run's step time (null unless the profile
        # was taken on the same workload); memory-side cache hits are inside these bytes, DRAM bytes are not measured
        "profile_fabric_GBps_step": round(gbps(profile_step_bytes, ms_per_step), 1) if profile_step_bytes else None,
        "profile_fabric_frac_of_hbm_peak": (round(gbps(profile_step_bytes, ms_per_step) / HBM_PEAK_GBS, 4)
                                            if profile_step_bytes else None),
        "stage_ms_per_step": {k: round(v, 4) for k, v in per_step_ms.items()},
        "stage_GBps_occurrence": {k: round(gbps(occ[k], per_step_ms[k]), 1) for k in per_step_ms if k in occ},
        "stage_GBps_compulsory": {k: round(gbps(comp[k], per_step_ms[k]), 1) for k in per_step_ms if k in comp},
        "setup_s": round(setup_s, 1),
        "roofline": roofline,
    }
    if cache_report is None and not args.overlap:
        # What this machine delivers to the barest kernel with the same access pattern (emb_probe_random_rows): as many
        # uniformly random whole-row reads as the step has ids, over the benchmark's own table (no key is frequent,
        # so this is the forward without its cache hits) and over its gradient buffer (row = one bag's gradient).
        sink = torch.zeros(4, dtype=torch.int32, device="cuda")
        p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

        def probe_ms(ptr, rows, row_bytes, n):
            binding.emb_probe_random_rows(ptr, rows, row_bytes, n, sink)
            torch.cuda.synchronize()
            p0.record()
            for _ in range(5):
                binding.emb_probe_random_rows(ptr, rows, row_bytes, n, sink)
            p1.record()
            torch.cuda.synchronize()
            return p0.elapsed_time(p1) / 5

        bare = []
        for t in range(T):
            n_t, D_t = int(N_t[t] / prof_steps), cfg.tables[t].dim
            if n_t == 0:
                continue
            w_ptr, _ = ctx.emb_table_ptr(t)
            ms_w = probe_ms(w_ptr, cfg.tables[t].rows, D_t * e_of[t], n_t)
            g_rows = grads[0].numel() // D_t
            ms_g = probe_ms(grads[0].data_ptr(), g_rows, D_t * 4, n_t)
            bare.append({"table": t, "reads": n_t,
                         "table_rows": {"row_bytes": D_t * e_of[t], "ms": round(ms_w, 4), "GBps": round(gbps(n_t * D_t * e_of[t], ms_w), 1)},
                         "gradient_rows": {"row_bytes": D_t * 4, "ms": round(ms_g, 4), "GBps": round(gbps(n_t * D_t * 4, ms_g), 1)}})
        out["bare_random_row_reads"] = bare
    if cache_report is not None:
        out["config"]["tables_in_host_memory"] = cache_report
        # what the host link of this machine delivers to bulk copies (the copy engines, 256 MiB of pinned memory each way):
        # the reference beside the row traffic of the cache, whose rows move as 16-byte accesses of a kernel
        hbuf = torch.empty(1 << 26, dtype=torch.float32, pin_memory=True)
        dbuf = torch.empty(1 << 26, dtype=torch.float32, device="cuda")
        link = {}
        for name, (dst, src) in {"host_to_device": (dbuf, hbuf), "device_to_host": (hbuf, dbuf)}.items():
            dst.copy_(src, non_blocking=True)
            torch.cuda.synchronize()
            c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            c0.record()
            for _ in range(4):
                dst.copy_(src, non_blocking=True)
            c1.record()
            torch.cuda.synchronize()
            link[name + "_GBps"] = round(4 * hbuf.numel() * 4 / (c0.elapsed_time(c1) * 1e-3) / 1e9, 1)
        out["host_link_bulk_copy"] = link

    if not args.no_cpu_baseline:
        from oracle import oracle as O   # the checker, timed as a baseline only
        hb = host_batches[0]
        S = cfg.num_slots
        # a bounded sample: whole batch 0 unless it holds more than ~30 M ids (then as many leading samples as hold that many)
        bs = args.cpu_samples if args.cpu_samples else max(1, min(hb.batch_size, int(3.0e7 * hb.batch_size / max(hb.num_ids, 1))))
        bs = min(bs, hb.batch_size)
        off = hb.offsets[: bs * S + 1]
        ids = hb.ids[: int(off[-1])]
        dp = grads[0][:bs].cpu().numpy()
        table_gb = sum(t.rows * (t.dim + 1) * 4 for t in cfg.tables) / 1e9       # the oracle stores fp32
        # whole (dense) tables when the host has the memory and their initialisation stays short; else the oracle's
        # touched-rows-only mode, whose hash map costs time on every row access
        dense = table_gb * 2.5 < host_mem_available_gb() and table_gb <= args.cpu_dense_gb
        t0 = time.perf_counter()
        orc = O.Oracle.from_config(cfg, dense=dense)
        init_s = time.perf_counter() - t0
        t0 = time.perf_counter()
        orc.lookup_pool(ids, off)
        orc.backward_update(ids, off, dp)
        cpu_s = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(len(ids) / cpu_s, 1), "unit": "IDs/s", "cores": 1, "kind": "oracle",
                               "cpu": cpu_model(), "tables": "dense" if dense else "sparse (touched rows in a hash map)",
                               "sample": f"{bs} of {hb.batch_size} samples of batch 0 ({len(ids)} IDs), one "
                                         f"lookup+bwd+update step, {cpu_s:.1f} s on 1 of {os.cpu_count()} visible cores"
                                         + (f" (+{init_s:.0f} s to initialise the {table_gb:.0f} GB tables, not counted)" if dense else "")}
        orc.close()
    ctx.close()
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
