"""CPU oracle of the hybrid step loop -- TEST INFRASTRUCTURE (plain Python over the two other oracles).

Section 3.2: the embedding layer is trained asynchronously, the dense network synchronously.  Algorithm 1: an
embedding worker's forward task looks the sample's embeddings up (`get`) and sends them on; its backward task,
run when the gradient of those activations comes back, does `put` + the optimizer.  Several samples may be
between the two tasks at once (the worker buffers them, section 4.2.1), so a lookup misses the updates of the
samples still in flight; section 5 assumes that number is bounded by tau.  Algorithm 2: the dense side takes the
batches one after the other, forward + backward + update, and returns F'^emb.

Reading: the staleness is taken as exactly tau, the bound: batch t is trained only once batch t + tau has been
looked up, so the lookup of batch t sees the updates of batches 0 .. t - tau - 1 and no others.  tau = 0 is
fully synchronous training.  Parity status: pinned (tests/test_hybrid_oracle_pins.py: explicit table snapshots,
tau beyond the run length, frozen embeddings, an off-by-one mutant).
"""
from collections import deque

import numpy as np


def run(emb, mlp, batches, tau, record_pooled=False):
    """emb: an embedding oracle with lookup_pool(ids, offsets) and backward_update(ids, offsets, d_pooled);
    mlp: a dense-step oracle with step(pooled, dense, labels) -> (loss, d_pooled, grads);
    batches: iterable of (ids, offsets, dense, labels).  Returns (losses per batch, pooled per batch or None)."""
    in_flight = deque()   # samples between the forward task and the backward task
    losses, pooled_log = [], []

    def train(sample):
        ids, offsets, dense, labels, pooled = sample
        loss, d_pooled, _ = mlp.step(pooled, dense, labels)           # Algorithm 2
        emb.backward_update(ids, offsets, d_pooled)                    # Algorithm 1, backward task
        losses.append(float(loss))

    for ids, offsets, dense, labels in batches:
        pooled = emb.lookup_pool(ids, offsets)                         # Algorithm 1, forward task
        if record_pooled:
            pooled_log.append(np.array(pooled))
        in_flight.append((ids, offsets, dense, labels, pooled))
        if len(in_flight) > tau:
            train(in_flight.popleft())
    while in_flight:
        train(in_flight.popleft())
    return np.array(losses), (pooled_log if record_pooled else None)
