"""Does bounded staleness of the embedding layer hurt?  (Section 3.2 / section 5 / Table 2's qualitative claim:
the hybrid algorithm -- stale embeddings, synchronous dense network -- trains like the fully synchronous one.)

A synthetic click-through task stands in for the paper's datasets: every (slot, key) has a hidden teacher
vector, a sample's label is Bernoulli(sigmoid(teacher logit)) with the logit linear in the summed teacher
vectors and the non-ID features.  Keys are Zipf-distributed, so hot rows are touched by every batch -- the case
where a lookup that misses the last tau updates differs most from a fresh one.  The student is the library's
embedding layer (row-wise Adagrad) plus its dense step with the paper's FFNN widths, driven by the hyb_* step
loop.  Every batch is fresh data, so the loss mlp_step reports for a batch (computed before that batch updates
anything) is a progressive-validation loss; the study reports its mean over the first and the last batches,
next to the entropy of the teacher's own probabilities (the best reachable loss) and to the loss of always
predicting the base rate.

    python -m paper_2111_05897_amd.staleness_study --taus 0 1 4 16 64 --steps 800

prints one JSON line per tau for the hybrid algorithm and one for the fully asynchronous comparison (the dense
network's gradients applied tau steps late too, mlp_set_update_delay).  Needs the GPU and the built library.
"""
from __future__ import annotations

import argparse
import json
import sys

import numpy as np

FFNN = [4096, 2048, 1024, 512, 256]          # section 6: the network of the paper's experiments


class Task:
    """Seeded generator of the synthetic task (inputs only: no arithmetic of the method)."""

    def __init__(self, seed=0, slots=16, keys_per_slot=2000, zipf_s=1.05, max_len=4, dense=64, teacher_dim=8):
        self.slots, self.keys, self.s, self.max_len, self.dense = slots, keys_per_slot, zipf_s, max_len, dense
        rng = np.random.Generator(np.random.Philox(key=[seed, 0x7EAC]))
        self.teacher = rng.standard_normal((slots, keys_per_slot, teacher_dim)).astype(np.float32)
        self.readout = (rng.standard_normal(teacher_dim) / np.sqrt(teacher_dim)).astype(np.float32)
        self.dense_w = (rng.standard_normal(dense) / np.sqrt(dense)).astype(np.float32)
        self.seed = seed
        self.bias = -1.0                       # base rate around 0.3

    def batch(self, step, batch_size):
        rng = np.random.Generator(np.random.Philox(key=[self.seed, 0xBA7C0000 + step]))
        S = self.slots
        lens = rng.integers(1, self.max_len + 1, size=batch_size * S)
        offsets = np.zeros(batch_size * S + 1, dtype=np.int64)
        np.cumsum(lens, out=offsets[1:])
        n = int(offsets[-1])
        u = rng.random(n)
        a = 1.0 - self.s
        ranks = np.floor((1.0 + u * ((self.keys + 1.0) ** a - 1.0)) ** (1.0 / a)).astype(np.int64)
        keys = np.clip(ranks, 1, self.keys) - 1
        slot_of = np.repeat(np.tile(np.arange(S), batch_size), lens)
        contrib = self.teacher[slot_of, keys] @ self.readout                      # [n]
        per_bag = np.add.reduceat(contrib, offsets[:-1])                          # bags are never empty
        emb_logit = per_bag.reshape(batch_size, S).sum(axis=1) / np.sqrt(S * (self.max_len + 1) / 2.0)
        dense = rng.standard_normal((batch_size, self.dense)).astype(np.float32)
        logit = 2.0 * emb_logit + dense @ self.dense_w + self.bias
        p = 1.0 / (1.0 + np.exp(-logit))
        labels = (rng.random(batch_size) < p).astype(np.float32)
        ids = (slot_of.astype(np.uint64) << np.uint64(32)) | keys.astype(np.uint64)
        bayes = float(np.mean(-(p * np.log(p) + (1 - p) * np.log1p(-p))))
        return ids, offsets.astype(np.int32), dense, labels, bayes, float(labels.mean())


def run(tau, steps, batch_size=4096, seed=0, rows=1 << 20, dim=64, emb_lr=1.0, mlp_lr=0.1, task=None, dense_delay=0):
    """Trains `steps` batches with embedding staleness `tau` and, for the fully asynchronous comparison, a dense
    side whose weights miss the last `dense_delay` gradients; returns the per-batch losses and reference levels."""
    import torch
    from . import binding
    from .workload import default_salt, make_mlp_params

    task = task or Task(seed)
    S = task.slots
    P = S * dim
    widths = [P + task.dense] + FFNN + [1]
    max_ids = batch_size * S * task.max_len
    emb = binding.EmbContext([(rows, dim, 0)], [(0, default_salt(s)) for s in range(S)], hash_kind=1, opt=1, lr=emb_lr,
                             eps=1e-8, acc_init=0.1, init_seed=1234 + seed, init_lo=-0.01, init_hi=0.01,
                             max_batch=batch_size, max_ids=max_ids)
    Ws, bs = make_mlp_params(widths, 99 + seed)
    mlp = binding.MlpContext(widths, P, task.dense, batch_size, mlp_lr, Ws, bs, loss_mean=True)
    if dense_delay:
        mlp.mlp_set_update_delay(dense_delay)
    loop = binding.HybridLoop(emb, mlp, tau)
    bayes, base = [], []
    for t in range(steps):
        ids, offsets, dense, labels, b, rate = task.batch(t, batch_size)
        db = binding.DeviceBatch(batch_size, ids, offsets)
        d, y = torch.from_numpy(dense).cuda(), torch.from_numpy(labels).cuda()
        torch.cuda.synchronize()
        loop.hyb_submit(db, d, y)
        loop.hyb_wait_inputs()                 # the loop has its own copy; db, d, y may go
        bayes.append(b)
        base.append(rate)
    loop.hyb_drain()
    losses = loop.hyb_read_losses(0, steps)
    loop.close()
    mlp.close()
    emb.close()
    rate = float(np.mean(base))
    return losses, float(np.mean(bayes)), float(-(rate * np.log(rate) + (1 - rate) * np.log1p(-rate)))


def summarize(tau, losses, bayes, base_entropy, window, mode="hybrid"):
    w = min(window, len(losses) // 2)
    return {"mode": mode, "tau": tau, "steps": int(len(losses)), "loss_first": round(float(losses[:w].mean()), 5),
            "loss_last": round(float(losses[-w:].mean()), 5), "window": w, "teacher_entropy": round(bayes, 5),
            "base_rate_entropy": round(base_entropy, 5),
            "normalized_entropy_last": round(float(losses[-w:].mean()) / base_entropy, 4)}


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--taus", type=int, nargs="+", default=[0, 1, 4, 16, 64])
    ap.add_argument("--steps", type=int, default=800)
    ap.add_argument("--batch", type=int, default=4096)
    ap.add_argument("--window", type=int, default=100)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-async", action="store_true", help="skip the fully asynchronous comparison runs")
    args = ap.parse_args(argv)
    task = Task(args.seed)
    for tau in args.taus:
        # hybrid: embeddings stale by tau, dense network synchronous (tau = 0: everything synchronous)
        losses, bayes, base = run(tau, args.steps, args.batch, args.seed, task=task)
        print(json.dumps(summarize(tau, losses, bayes, base, args.window, "synchronous" if tau == 0 else "hybrid")),
              flush=True)
        if tau and not args.no_async:
            # fully asynchronous: the dense network's gradients arrive tau steps late as well
            losses, bayes, base = run(tau, args.steps, args.batch, args.seed, task=task, dense_delay=tau)
            print(json.dumps(summarize(tau, losses, bayes, base, args.window, "fully asynchronous")), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
