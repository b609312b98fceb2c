"""GPU parity over randomly drawn small configurations (seeded): number of tables, their rows (powers of two and
not), widths, storage types, the slot -> table map, hash kind, optimizer and its constants, batch shape (empty
bags, repeated ids, hot keys, batch sizes that do not fill a tile).  Each draw runs two whole steps through
tests/util.run_steps: hash, pooled, index form, updated rows and accumulators against the oracle."""
import numpy as np
import pytest

from oracle import oracle as O
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


def _draw(seed):
    rng = np.random.default_rng(1000 + seed)
    T = int(rng.integers(1, 5))
    tables = []
    for _ in range(T):
        rows = int(rng.choice([1, 2, 3, 64, 100, 1 << 10, 1500, 1 << 13, 10007]))
        tables.append(W.TableDesc(rows, int(rng.choice([8, 16, 32, 64, 128])), int(rng.integers(0, 2))))
    S = int(rng.integers(T, 3 * T + 2))
    slot_tables = list(range(T)) + [int(x) for x in rng.integers(0, T, size=S - T)]   # every table is read
    rng.shuffle(slot_tables)
    hash_kind = int(rng.integers(0, 2))
    cfg = W.EmbConfig(tables=tables, slots=[W.SlotDesc(t, W.default_salt(s)) for s, t in enumerate(slot_tables)],
                      hash_kind=hash_kind, opt=int(rng.integers(0, 2)), lr=float(rng.choice([0.0, 0.01, 0.3])),
                      eps=float(rng.choice([0.0, 1e-8, 1e-3])), acc_init=float(rng.choice([0.01, 0.1, 1.0])),
                      init_seed=int(rng.integers(0, 1 << 30)), init_lo=-float(rng.choice([0.01, 0.5])),
                      init_hi=float(rng.choice([0.01, 0.5])))
    bsz = int(rng.choice([1, 7, 33, 64, 150]))
    max_len = int(rng.choice([1, 3, 12]))
    id_space = int(rng.choice([5, 200, 100000]))
    batches = [W.random_batch(seed * 10 + s, bsz, S, max_len, id_space, allow_empty=bool(rng.integers(0, 2))) for s in range(2)]
    grads = [rng.standard_normal((bsz, cfg.pooled_width)).astype(np.float32) for _ in range(2)]
    return cfg, bsz, batches, grads


@pytest.mark.parametrize("seed", range(48))
def test_random_configuration(B, seed):
    cfg, bsz, batches, grads = _draw(seed)
    w = W.Workload(f"random{seed}", 0, cfg, bsz, "uniform", 0, 1, "uniform", 1, seed=seed)
    util.run_steps(B, W, O, w, steps=2, batches=batches, grads=grads)
