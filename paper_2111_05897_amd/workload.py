"""Seeded synthetic workloads for the embedding hot path.

This module only *generates inputs*: CSR batches of 64-bit sparse IDs, upstream
gradients, and the static description (tables, slots, optimizer) of the five
benchmark configurations.  It holds none of the method's arithmetic (no hashing
of IDs to rows, no pooling, no dedup, no optimizer) and is the only module that
both the CPU oracle's tests and the HIP path's tests import.

The public recommender datasets the paper trains on (section 6, "Benchmarks")
are not used; batches here are seeded stand-ins with the same structure: a
sample carries several ID-type feature groups ("slots", section 2.1), each a
variable-length list of 64-bit IDs whose frequencies are heavily skewed.

Everything is a pure function of (config, seed, step): the generator is
counter-based, so any slice of any array can be regenerated independently.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np

F32, BF16 = 0, 1
OPT_SGD, OPT_ROWWISE_ADAGRAD = 0, 1
HASH_IDENTITY_MOD, HASH_MIX_MOD = 0, 1

_U64 = np.uint64
_GOLD = _U64(0x9E3779B97F4A7C15)
# odd constant the default per-slot salt is a multiple of (input convention, not method arithmetic)
SALT_STRIDE = 0xA24BAED4963EE407


# --------------------------------------------------------------------------- counter-based RNG
def _scramble(x: np.ndarray) -> np.ndarray:
    """Stateless 64-bit scrambler used only to draw synthetic inputs."""
    x = x.astype(np.uint64, copy=True)
    x ^= x >> _U64(30)
    x *= _U64(0xBF58476D1CE4E5B9)
    x ^= x >> _U64(27)
    x *= _U64(0x94D049BB133111EB)
    x ^= x >> _U64(31)
    return x


def _stream_key(seed: int, tag: int, step: int) -> np.uint64:
    k = np.array([(seed * 0x100000001B3 + tag * 0x9E3779B1 + step * 0x632BE59BD9B4E019 + 0x1234567) % (1 << 64)],
                 dtype=np.uint64)
    return _scramble(_scramble(k))[0]


def counter_u64(seed: int, tag: int, step: int, start: int, count: int) -> np.ndarray:
    """`count` 64-bit draws with counters start..start+count-1 of stream (seed, tag, step)."""
    with np.errstate(over="ignore"):
        ctr = np.arange(start, start + count, dtype=np.uint64)
        return _scramble(ctr * _GOLD + _stream_key(seed, tag, step))


def counter_uniform(seed: int, tag: int, step: int, start: int, count: int) -> np.ndarray:
    """fp64 uniforms in [0, 1) with 53 random bits."""
    return (counter_u64(seed, tag, step, start, count) >> _U64(11)).astype(np.float64) * (1.0 / (1 << 53))


def counter_normal_f32(seed: int, tag: int, step: int, count: int) -> np.ndarray:
    """`count` N(0,1) fp32 draws from numpy's counter-based Philox generator keyed (seed, tag, step)."""
    key = [seed % (1 << 64), ((tag << 32) | step) % (1 << 64)]
    return np.random.Generator(np.random.Philox(key=key)).standard_normal(count, dtype=np.float32)


# --------------------------------------------------------------------------- configuration
@dataclass
class TableDesc:
    rows: int
    dim: int
    dtype: int = F32


@dataclass
class SlotDesc:
    table: int
    salt: int


@dataclass
class EmbConfig:
    """Static description handed to emb_create (and, independently, to the oracle)."""
    tables: List[TableDesc]
    slots: List[SlotDesc]
    hash_kind: int = HASH_MIX_MOD
    opt: int = OPT_ROWWISE_ADAGRAD
    lr: float = 0.05
    eps: float = 1e-8
    acc_init: float = 0.1
    init_seed: int = 0x5EED
    init_lo: float = -0.01
    init_hi: float = 0.01
    max_batch: int = 0
    max_ids: int = 0

    @property
    def num_slots(self) -> int:
        return len(self.slots)

    def slot_dims(self) -> List[int]:
        return [self.tables[s.table].dim for s in self.slots]

    def slot_cols(self) -> List[int]:
        cols, c = [], 0
        for d in self.slot_dims():
            cols.append(c)
            c += d
        return cols

    @property
    def pooled_width(self) -> int:
        return sum(self.slot_dims())


def default_salt(slot: int) -> int:
    """Per-slot salt: (slot+1) times a fixed odd 64-bit constant, so slots are distinct key spaces."""
    return ((slot + 1) * SALT_STRIDE) % (1 << 64)


@dataclass
class Workload:
    """One benchmark configuration: the static config plus the recipe for its batches."""
    name: str
    index: int
    cfg: EmbConfig
    batch: int
    len_kind: str                 # "const" | "uniform" | "poisson"
    len_a: int                    # const: length; uniform: lo; poisson: mean
    len_b: int                    # uniform: hi; poisson: clip hi
    id_kind: str                  # "uniform" | "zipf"
    id_space: int                 # uniform: ids in [0, id_space); zipf: number of keys K
    zipf_s: float = 0.0
    steps: int = 1
    seed: int = 0
    notes: str = ""

    @property
    def bags(self) -> int:
        return self.batch * self.cfg.num_slots


def _single_table(rows, dim, dtype, slots, **kw) -> EmbConfig:
    return EmbConfig(tables=[TableDesc(rows, dim, dtype)],
                     slots=[SlotDesc(0, default_salt(s)) for s in range(slots)], **kw)


def make_workload(index: int, scale: float = 1.0) -> Workload:
    """The five benchmark configurations (0: one-hot unit test ... 4: 64 GiB bf16 table).  `scale` < 1 shrinks
    batch and table rows (power-of-two rows kept) for quick tests; scale == 1 is the full size."""
    seed = 0x5EED0000 + index

    def rows(r):
        if scale >= 1.0:
            return r
        k = max(10, int(np.floor(np.log2(r * scale))))
        return 1 << k

    def bsz(b):
        return b if scale >= 1.0 else max(8, int(b * scale))

    if index == 0:
        cfg = _single_table(65536, 16, F32, 8, hash_kind=HASH_IDENTITY_MOD, opt=OPT_SGD, lr=0.01,
                            init_seed=seed)
        return Workload("cfg0_tiny_onehot", 0, cfg, bsz(512), "const", 1, 1, "uniform", 65536, 0.0, 1, seed)
    if index == 1:
        cfg = _single_table(rows(1 << 22), 32, F32, 26, init_seed=seed)
        return Workload("cfg1_criteo_like", 1, cfg, bsz(8192), "uniform", 1, 20, "zipf", 10 ** 8, 1.05, 1, seed)
    if index == 2:
        cfg = _single_table(rows(1 << 26), 64, F32, 100, init_seed=seed)
        return Workload("cfg2_100slot_fp32_d64", 2, cfg, bsz(16384), "poisson", 8, 64, "zipf", 10 ** 9, 1.2, 10, seed)
    if index == 3:
        dims = [8, 16, 32, 64, 128]
        trows = [rows(1 << 26), rows(1 << 25), rows(1 << 24), rows(1 << 23), rows(1 << 23)]
        tables = [TableDesc(r, d, BF16) for r, d in zip(trows, dims)]
        slots = [SlotDesc(s % 5, default_salt(s)) for s in range(200)]
        cfg = EmbConfig(tables=tables, slots=slots, init_seed=seed)
        return Workload("cfg3_hybrid_mixed_dims_bf16", 3, cfg, bsz(32768), "uniform", 1, 32, "zipf", 10 ** 9, 1.1, 1,
                        seed)
    if index == 4:
        cfg = _single_table(rows(1 << 29), 64, BF16, 50, init_seed=seed)
        return Workload("cfg4_capacity_contention", 4, cfg, bsz(65536), "uniform", 1, 16, "zipf", 10 ** 10, 1.4, 3,
                        seed)
    raise ValueError(f"no such config {index}")


# --------------------------------------------------------------------------- batch generation
_TAG_LEN, _TAG_ID, _TAG_GRAD = 1, 2, 3
_CHUNK = 1 << 20


def _poisson_cdf(mean: float, kmax: int) -> np.ndarray:
    k = np.arange(0, kmax + 1, dtype=np.float64)
    logp = -mean + k * np.log(mean) - np.cumsum(np.concatenate([[0.0], np.log(np.arange(1, kmax + 1))]))
    return np.cumsum(np.exp(logp))


def bag_lengths(w: Workload, step: int) -> np.ndarray:
    n = w.bags
    if w.len_kind == "const":
        return np.full(n, w.len_a, dtype=np.int64)
    if w.len_kind not in ("uniform", "poisson"):
        raise ValueError(w.len_kind)
    out = np.empty(n, dtype=np.int64)
    cdf = _poisson_cdf(float(w.len_a), 4 * w.len_b) if w.len_kind == "poisson" else None
    for i0 in range(0, n, _CHUNK):          # chunked so temporaries stay small and get reused
        i1 = min(n, i0 + _CHUNK)
        u = counter_uniform(w.seed, _TAG_LEN, step, i0, i1 - i0)
        if cdf is None:
            out[i0:i1] = w.len_a + np.floor(u * (w.len_b - w.len_a + 1))
        else:
            out[i0:i1] = np.clip(np.searchsorted(cdf, u, side="right"), 1, w.len_b)
    return out


def zipf_ranks(u: np.ndarray, num_keys: int, s: float) -> np.ndarray:
    """Rank k in [1, K] with P(k) ~ k^-s via the continuous inverse CDF
    k = floor((1 + u*((K+1)^(1-s) - 1))^(1/(1-s))), O(1) memory in K."""
    e = 1.0 - s
    t = 1.0 + u * ((num_keys + 1.0) ** e - 1.0)
    k = np.floor(t ** (1.0 / e))
    return np.clip(k, 1, num_keys).astype(np.uint64)


def make_ids(w: Workload, step: int, n: int) -> np.ndarray:
    if w.id_kind == "uniform":
        u = counter_uniform(w.seed, _TAG_ID, step, 0, n)
        return np.floor(u * w.id_space).astype(np.uint64)
    out = np.empty(n, dtype=np.uint64)
    for i0 in range(0, n, _CHUNK):
        i1 = min(n, i0 + _CHUNK)
        u = counter_uniform(w.seed, _TAG_ID, step, i0, i1 - i0)
        k = zipf_ranks(u, w.id_space, w.zipf_s)
        with np.errstate(over="ignore"):
            out[i0:i1] = _scramble(k * _U64(0xD6E8FEB86659FD93) + _U64(0x2545F4914F6CDD1D))  # rank -> 64-bit ID
    return out


@dataclass
class Batch:
    batch_size: int
    ids: np.ndarray        # [N] uint64
    offsets: np.ndarray    # [B*S+1] int32, offsets[0] = 0, offsets[-1] = N

    @property
    def num_ids(self) -> int:
        return int(self.offsets[-1])


def make_batch(w: Workload, step: int = 0) -> Batch:
    lens = bag_lengths(w, step)
    offsets = np.zeros(w.bags + 1, dtype=np.int64)
    np.cumsum(lens, out=offsets[1:])
    n = int(offsets[-1])
    assert n < (1 << 31)
    return Batch(w.batch, make_ids(w, step, n), offsets.astype(np.int32))


def make_d_pooled(w: Workload, step: int = 0) -> np.ndarray:
    """Upstream gradient of the pooled activations, N(0,1), shape [B, sum of slot dims] fp32."""
    width = w.cfg.pooled_width
    return counter_normal_f32(w.seed, _TAG_GRAD, step, w.batch * width).reshape(w.batch, width)


def random_batch(seed: int, batch: int, num_slots: int, max_len: int, id_space: int,
                 allow_empty: bool = True) -> Batch:
    """Small irregular batch for unit tests: lengths uniform in [0 or 1, max_len], ids uniform in [0, id_space)."""
    lo = 0 if allow_empty else 1
    u = counter_uniform(seed, _TAG_LEN, 0, 0, batch * num_slots)
    lens = (lo + np.floor(u * (max_len - lo + 1))).astype(np.int64)
    offsets = np.zeros(batch * num_slots + 1, dtype=np.int64)
    np.cumsum(lens, out=offsets[1:])
    n = int(offsets[-1])
    ids = np.floor(counter_uniform(seed, _TAG_ID, 0, 0, n) * id_space).astype(np.uint64)
    return Batch(batch, ids, offsets.astype(np.int32))


# --------------------------------------------------------------------------- dense side (config 3)
MLP_HIDDEN = [4096, 2048, 1024]
DENSE_FEATURES = 512


def make_mlp_params(widths, seed):
    """Initial weights N(0, 2/fan_in) and zero biases for a ReLU net with layer widths `widths` (inputs to the
    dense step, drawn here so that the GPU library and the oracle receive the same arrays)."""
    rng = np.random.Generator(np.random.Philox(key=[seed % (1 << 64), 0xD15E]))
    Ws = [(rng.standard_normal((i, o), dtype=np.float32) * np.float32(np.sqrt(2.0 / i))) for i, o in
          zip(widths[:-1], widths[1:])]
    bs = [np.zeros(o, dtype=np.float32) for o in widths[1:]]
    return Ws, bs


def make_dense_and_labels(seed, step, batch, dense_width=DENSE_FEATURES, positive_rate=0.05):
    """Non-ID features N(0,1) fp32 [B, dense_width] and labels Bernoulli(positive_rate) fp32 [B]."""
    rng = np.random.Generator(np.random.Philox(key=[seed % (1 << 64), 0xDE45E000 + step]))
    dense = rng.standard_normal((batch, dense_width), dtype=np.float32)
    labels = (rng.random(batch) < positive_rate).astype(np.float32)
    return dense, labels
