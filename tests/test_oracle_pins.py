"""Pins for the CPU oracle: every function is checked against something other than itself --
library routines (torch embedding_bag / autograd / SGD / Adagrad / bf16 cast, numpy unique),
brute force on tiny inputs (dense count-matrix products, python dicts), an explicit inverse of
the hash mixer, and invariants.  CPU only."""
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_2111_05897_amd import workload as W

M64 = (1 << 64) - 1


# ----------------------------------------------------------------------------- helpers
def make_oracle(tables, slot_tables, hash_kind=W.HASH_IDENTITY_MOD, opt=W.OPT_SGD, lr=0.01, eps=1e-8, acc_init=0.1,
                seed=7, lo=-0.01, hi=0.01, dense=True):
    slots = [(t, W.default_salt(s)) for s, t in enumerate(slot_tables)]
    return O.Oracle(tables, slots, hash_kind, opt, lr, eps, acc_init, seed, lo, hi, dense=dense)


def table_values(orc, t):
    rows = np.arange(orc.tables[t][0], dtype=np.uint64)
    return orc.read_rows(t, rows)


def count_matrix(rows, offsets, R):
    """C[bag, r] = multiplicity of row r in the bag."""
    nb = len(offsets) - 1
    Cm = np.zeros((nb, R), dtype=np.float64)
    for bag in range(nb):
        for i in range(offsets[bag], offsets[bag + 1]):
            Cm[bag, rows[i]] += 1.0
    return Cm


# ----------------------------------------------------------------------------- hash (a1)
def _unxorshift(z, s):
    x = z
    for _ in range(64 // s + 1):
        x = z ^ (x >> s)
    return x & M64


def mix64_inverse(z):
    """Inverse of: z^=z>>31; z*=C1; z^=z>>29; z*=C2; z^=z>>32 -- derived, not retyped:
    undo each step in reverse with the modular inverse of the odd multiplier."""
    c1, c2 = 0x9FB21C651E98DF25, 0xC2B2AE3D27D4EB4F
    z = _unxorshift(z, 32)
    z = (z * pow(c2, -1, 1 << 64)) & M64
    z = _unxorshift(z, 29)
    z = (z * pow(c1, -1, 1 << 64)) & M64
    z = _unxorshift(z, 31)
    return z


def test_mix64_is_the_documented_bijection():
    rng = np.random.default_rng(1)
    xs = [0, 1, M64, 1 << 63] + [int(v) for v in rng.integers(0, 1 << 63, size=20000, dtype=np.uint64)]
    ys = [O.mix64(x) for x in xs]
    assert all(mix64_inverse(y) == x for x, y in zip(xs, ys))
    assert len(set(ys)) == len(set(xs))
    # avalanche sanity: flipping one input bit flips about half the output bits
    flips = [bin(O.mix64(x) ^ O.mix64(x ^ (1 << b))).count("1") for x in xs[4:300] for b in (0, 17, 40, 63)]
    assert 28 < np.mean(flips) < 36


def test_hash_identity_is_mod_and_mix_is_salted_mod():
    R = 1000  # not a power of two on purpose
    orc = make_oracle([(R, 8, W.F32)], [0, 0, 0], hash_kind=W.HASH_IDENTITY_MOD)
    b = W.random_batch(3, 16, 3, 5, 1 << 40)
    np.testing.assert_array_equal(orc.hash_rows(b.ids, b.offsets), (b.ids % np.uint64(R)).astype(np.uint32))
    orc2 = make_oracle([(R, 8, W.F32)], [0, 0, 0], hash_kind=W.HASH_MIX_MOD)
    rows = orc2.hash_rows(b.ids, b.offsets)
    assert rows.max() < R
    S = 3
    for bag in range(16 * S):
        for i in range(b.offsets[bag], b.offsets[bag + 1]):
            z = (int(b.ids[i]) + W.default_salt(bag % S)) & M64
            assert mix64_inverse((O.mix64(z))) == z
            assert rows[i] == O.mix64(z) % R
    # same id in two slots lands on different rows (distinct key spaces), mostly
    ids = np.arange(1000, dtype=np.uint64).repeat(3)
    off = np.arange(0, 3001, dtype=np.int32)
    r3 = make_oracle([(1 << 20, 8, W.F32)], [0, 0, 0], hash_kind=W.HASH_MIX_MOD).hash_rows(ids, off).reshape(1000, 3)
    assert (r3[:, 0] != r3[:, 1]).mean() > 0.99 and (r3[:, 1] != r3[:, 2]).mean() > 0.99


def test_hash_rows_uniform_over_table():
    R = 1 << 10
    orc = make_oracle([(R, 8, W.F32)], [0], hash_kind=W.HASH_MIX_MOD)
    ids = np.arange(1 << 16, dtype=np.uint64)  # sequential ids: worst case for a weak mixer
    off = np.arange(0, (1 << 16) + 1, dtype=np.int32)
    cnt = np.bincount(orc.hash_rows(ids, off), minlength=R)
    chi2 = ((cnt - 64.0) ** 2 / 64.0).sum()
    assert chi2 < R + 6 * math.sqrt(2 * R)


# ----------------------------------------------------------------------------- bf16 (storage rounding)
def test_bf16_round_matches_torch_cast():
    rng = np.random.default_rng(2)
    bits = rng.integers(0, 1 << 32, size=200000, dtype=np.uint64).astype(np.uint32)
    special = np.array([0x00000000, 0x80000000, 0x3F808000, 0x3F818000, 0x3F80FFFF, 0x3F807FFF, 0x7F7FFFFF, 0x7F800000,
                        0xFF800000, 0x00000001, 0x00008000, 0x00018000, 0x007FFFFF, 0x7F7F8000, 0x3F800001],
                       dtype=np.uint32)
    bits = np.concatenate([bits, special])
    x = bits.view(np.float32)
    want = torch.from_numpy(x.copy()).to(torch.bfloat16).to(torch.float32).numpy()
    got = O.round_bf16(x)
    fin = ~np.isnan(want)
    np.testing.assert_array_equal(got[fin].view(np.uint32), want[fin].view(np.uint32))
    assert np.isnan(got[~fin]).all()


def test_bf16_round_is_identity_on_all_bf16_patterns():
    hi = np.arange(1 << 16, dtype=np.uint32) << 16
    x = hi.view(np.float32)
    got = O.round_bf16(x)
    fin = ~np.isnan(x)
    np.testing.assert_array_equal(got[fin].view(np.uint32), hi[fin])


# Exact binary rounding with integers and fractions only: the nearest value m * 2^q with |m| < 2^p (p significant
# bits), exponent of the spacing no lower than q_min (where subnormals begin), ties to the even m.
def round_to_format(x: Fraction, p: int, q_min: int) -> Fraction:
    if x == 0:
        return Fraction(0)
    sign = -1 if x < 0 else 1
    a = abs(x)
    e = a.numerator.bit_length() - a.denominator.bit_length()      # 2^(e-1) <= a < 2^(e+1)
    if Fraction(2) ** e > a:
        e -= 1                                                      # now 2^e <= a < 2^(e+1)
    q = max(e - (p - 1), q_min)
    scaled = a / Fraction(2) ** q
    m = scaled.numerator // scaled.denominator
    rest = scaled - m
    if rest > Fraction(1, 2) or (rest == Fraction(1, 2) and m % 2 == 1):
        m += 1
    return sign * m * Fraction(2) ** q


def to_f32_exact(x: Fraction) -> Fraction:
    return round_to_format(x, 24, -149)


def to_bf16_exact(x: Fraction) -> Fraction:
    return round_to_format(x, 8, -133)


def test_exact_rounding_helper_agrees_with_numpy_on_fp32():
    # the helper itself, against the machine's own fp64 -> fp32 conversion
    rng = np.random.default_rng(12)
    xs = np.concatenate([rng.standard_normal(2000) * 10.0 ** rng.integers(-40, 38, 2000),
                         [1.0 + 2.0 ** -24, 1.0 + 3 * 2.0 ** -24, 2.0 ** -149 * 0.5, 2.0 ** -149 * 1.5, 2.0 ** -127]])
    for x in xs:
        assert float(to_f32_exact(Fraction(float(x)))) == float(np.float32(x)), x


def test_store_rounds_fp64_to_bf16_once():
    rng = np.random.default_rng(13)
    xs = list(rng.standard_normal(3000) * 10.0 ** rng.integers(-42, 38, 3000))
    # exact bf16 ties, and fp64 values a hair off a tie: fp64 -> fp32 lands ON the tie, so a second rounding
    # (ties to even) goes the other way than the single rounding
    for m in (128, 129, 200, 255):
        for e in (-130, -20, 0, 5, 100):
            tie = (m + 0.5) * 2.0 ** (e - 7)
            xs += [tie, -tie, tie * (1 + 2.0 ** -40), tie * (1 - 2.0 ** -40), -tie * (1 + 2.0 ** -40)]
    xs += [0.0, -0.0, 2.0 ** -134, 2.0 ** -134 * 1.0001, 3 * 2.0 ** -134, 2.0 ** -126, 3.3895e38, 3.4e38, -3.4e38, 1e-300]
    twice_differs = 0
    for x in xs:
        got = O.round_bf16_once(float(x))
        want = to_bf16_exact(Fraction(float(x)))
        if abs(want) > Fraction(255) * Fraction(2) ** 120:
            assert math.isinf(got) and (got > 0) == (x > 0), x
            continue
        assert Fraction(got) == want, (x, got, float(want))
        with np.errstate(over="ignore"):
            twice = float(O.round_bf16(np.array([np.float32(x)]))[0])
        twice_differs += twice != got
    assert twice_differs >= 10          # the cases above do tell one rounding from two
    assert math.isnan(O.round_bf16_once(float("nan"))) and O.round_bf16_once(float("inf")) == float("inf")


def test_init_value_is_exactly_the_two_rounding_definition():
    """value = fl32(fl32(k * scale) + mid), k = (top 24 bits of the element's hash) - 2^23, scale = fl32(hi - lo) * 2^-24,
    mid = fl32(hi + lo) / 2 -- every rounding done here in exact rational arithmetic.  The hash comes from the
    oracle's mix64, which the bijection pin above covers."""
    fused_differs = 0
    for seed, lo, hi, dim in [(3, -0.5, 0.25, 8), (2021, -0.01, 0.03, 16), (9, 0.125, 1.0, 32), (11, -0.01, 0.01, 64)]:
        lo32, hi32 = Fraction(float(np.float32(lo))), Fraction(float(np.float32(hi)))
        scale = to_f32_exact(hi32 - lo32) * Fraction(1, 1 << 24)
        mid = to_f32_exact(hi32 + lo32) / 2
        for t in (0, 3):
            table_key = O.mix64(seed + (t + 1) * 0x9E3779B97F4A7C15)
            for r in (0, 1, 77, 123456789):
                for d in range(dim):
                    k = (O.mix64(table_key + r * dim + d) >> 40) - (1 << 23)
                    want = to_f32_exact(to_f32_exact(k * scale) + mid)
                    got = O.init_value(seed, t, r, dim, d, lo, hi)
                    assert Fraction(got) == want, (seed, t, r, d)
                    fused_differs += to_f32_exact(k * scale + mid) != want
    assert fused_differs > 50           # a fused multiply-add would have been noticed


# ----------------------------------------------------------------------------- init
def test_init_range_uniformity_and_determinism():
    lo, hi = -0.01, 0.01
    orc = make_oracle([(4096, 16, W.F32), (4096, 16, W.F32)], [0, 1], lo=lo, hi=hi, seed=11)
    w0, a0 = table_values(orc, 0)
    w1, _ = table_values(orc, 1)
    assert (a0 == np.float32(0.1)).all()
    assert w0.min() >= np.float32(lo) and w0.max() < np.float32(hi)
    # uniform: mean 0, variance (hi-lo)^2/12, flat histogram, tables and columns decorrelated
    n = w0.size
    assert abs(w0.mean()) < 5 * (hi - lo) / math.sqrt(12 * n)
    assert abs(w0.var() / ((hi - lo) ** 2 / 12) - 1) < 0.02
    hist = np.histogram(w0, bins=64, range=(lo, hi))[0]
    assert ((hist - n / 64) ** 2 / (n / 64)).sum() < 64 + 6 * math.sqrt(128)
    assert abs(np.corrcoef(w0.ravel(), w1.ravel())[0, 1]) < 0.02
    assert abs(np.corrcoef(w0[:, 0], w0[:, 1])[0, 1]) < 0.06
    assert abs(np.corrcoef(w0[:-1].ravel(), w0[1:].ravel())[0, 1]) < 0.02
    # values sit on the documented grid lo + (hi-lo)*k/2^24 to within one fp32 rounding
    k = (w0.astype(np.float64) - lo) / (hi - lo) * (1 << 24)
    assert np.abs(k - np.round(k)).max() < 0.01 * (1 << 24) * 2 ** -23 / (hi - lo) * 2
    # same seed -> same table, other seed -> another; sparse mode regenerates the same rows
    again = make_oracle([(4096, 16, W.F32), (4096, 16, W.F32)], [0, 1], lo=lo, hi=hi, seed=11)
    np.testing.assert_array_equal(table_values(again, 0)[0], w0)
    other = make_oracle([(4096, 16, W.F32)], [0], lo=lo, hi=hi, seed=12)
    assert (table_values(other, 0)[0] != w0).mean() > 0.99
    sparse = make_oracle([(4096, 16, W.F32), (4096, 16, W.F32)], [0, 1], lo=lo, hi=hi, seed=11, dense=False)
    pick = np.array([4095, 0, 17, 17, 2000], dtype=np.uint64)
    np.testing.assert_array_equal(sparse.read_rows(1, pick)[0], w1[pick.astype(np.int64)])
    assert sparse.rows_stored(1) == 4 and sparse.rows_stored(0) == 0


def test_init_bf16_tables_hold_bf16_values():
    orc = make_oracle([(1024, 8, W.BF16)], [0], seed=5)
    w, _ = table_values(orc, 0)
    assert ((w.view(np.uint32) & 0xFFFF) == 0).all()
    ref = make_oracle([(1024, 8, W.F32)], [0], seed=5)
    w32, _ = table_values(ref, 0)
    np.testing.assert_array_equal(w, torch.from_numpy(w32).to(torch.bfloat16).float().numpy())


# ----------------------------------------------------------------------------- lookup + pool (a2)
def _torch_pool(Wt, rows, offsets):
    """Library routine: sum-mode embedding_bag in fp64."""
    return torch.nn.functional.embedding_bag(torch.from_numpy(rows.astype(np.int64)), Wt,
                                             torch.from_numpy(offsets[:-1].astype(np.int64)), mode="sum")


@pytest.mark.parametrize("hash_kind", [W.HASH_IDENTITY_MOD, W.HASH_MIX_MOD])
def test_lookup_pool_matches_embedding_bag_and_count_matrix(hash_kind):
    R, D, S, B = 64, 8, 3, 20
    orc = make_oracle([(R, D, W.F32)], [0] * S, hash_kind=hash_kind)
    b = W.random_batch(5, B, S, 6, 1 << 30)         # includes empty bags and duplicates inside bags
    rows = orc.hash_rows(b.ids, b.offsets)
    w, _ = table_values(orc, 0)
    pooled = orc.lookup_pool(b.ids, b.offsets)
    assert pooled.shape == (B, S * D)
    want = _torch_pool(torch.from_numpy(w.astype(np.float64)), rows, b.offsets).numpy().reshape(B, S * D)
    np.testing.assert_allclose(pooled, want, rtol=1e-7, atol=1e-10)
    brute = (count_matrix(rows, b.offsets, R) @ w.astype(np.float64)).reshape(B, S * D)
    np.testing.assert_allclose(pooled, brute, rtol=1e-7, atol=1e-10)
    lens = np.diff(b.offsets).reshape(B, S)
    assert (lens == 0).any()
    for bb, s in zip(*np.nonzero(lens == 0)):
        assert (pooled[bb, s * D:(s + 1) * D] == 0).all()


def test_lookup_pool_single_id_bags_return_rows_bit_exact():
    w = W.make_workload(0)
    orc = O.Oracle.from_config(w.cfg, dense=True)
    b = W.make_batch(w)
    pooled = orc.lookup_pool(b.ids, b.offsets)
    rows, _ = orc.read_rows(0, b.ids % np.uint64(65536))
    np.testing.assert_array_equal(pooled.reshape(-1, 16), rows)


def test_lookup_pool_integer_table_duplicates_and_order():
    R, D = 50, 8
    orc = make_oracle([(R, D, W.F32)], [0, 0])
    allr = np.arange(R, dtype=np.uint64)
    orc.write_rows(0, allr, np.repeat(np.arange(R, dtype=np.float32)[:, None], D, 1) + np.arange(D, dtype=np.float32))
    ids = np.array([3, 3, 7, 49, 0, 1, 2, 2, 2], dtype=np.uint64)
    off = np.array([0, 3, 4, 4, 9], dtype=np.int32)     # B=2, S=2; bag 2 empty
    p = orc.lookup_pool(ids, off).reshape(4, D)
    for bag, members in enumerate([[3, 3, 7], [49], [], [0, 1, 2, 2, 2]]):
        np.testing.assert_array_equal(p[bag], sum(members) + len(members) * np.arange(D, dtype=np.float32))
    perm = np.array([7, 3, 3, 49, 2, 2, 1, 0, 2], dtype=np.uint64)
    np.testing.assert_array_equal(orc.lookup_pool(perm, off), p.reshape(2, 2 * D))


def test_lookup_pool_mixed_tables_column_layout():
    tables = [(32, 8, W.F32), (16, 16, W.BF16), (64, 32, W.F32)]
    slot_tables = [2, 0, 1, 0, 2]
    orc = make_oracle(tables, slot_tables, hash_kind=W.HASH_MIX_MOD)
    B, S = 6, len(slot_tables)
    b = W.random_batch(9, B, S, 4, 1 << 20)
    rows = orc.hash_rows(b.ids, b.offsets)
    pooled = orc.lookup_pool(b.ids, b.offsets)
    assert pooled.shape == (B, 32 + 8 + 16 + 8 + 32)
    col = 0
    for s, t in enumerate(slot_tables):
        D = tables[t][1]
        wt = torch.from_numpy(table_values(orc, t)[0].astype(np.float64))
        for bb in range(B):
            bag = bb * S + s
            r = rows[b.offsets[bag]:b.offsets[bag + 1]].astype(np.int64)
            assert (r < tables[t][0]).all()
            want = wt[r].sum(0).numpy() if len(r) else np.zeros(D)
            np.testing.assert_allclose(pooled[bb, col:col + D], want, rtol=1e-7, atol=1e-12)
        col += D


# ----------------------------------------------------------------------------- dedup (a3, a4)
def _dict_dedup(keys, bags):
    d = {}
    for k, bag in zip(keys, bags):
        d.setdefault(int(k), []).append(int(bag))
    return d


def _bag_of_occurrence(offsets):
    return np.repeat(np.arange(len(offsets) - 1, dtype=np.uint32), np.diff(offsets))


@pytest.mark.parametrize("seed,R", [(1, 8), (2, 100), (3, 1 << 16)])
def test_dedup_against_dict_and_numpy_unique(seed, R):
    tables = [(R, 8, W.F32), (max(2, R // 2), 16, W.F32)]
    slot_tables = [0, 1, 0]
    orc = make_oracle(tables, slot_tables, hash_kind=W.HASH_MIX_MOD)
    b = W.random_batch(seed, 40, 3, 7, 500)
    rows = orc.hash_rows(b.ids, b.offsets)
    bags = _bag_of_occurrence(b.offsets)
    keys_occ = (np.array(slot_tables, dtype=np.uint64)[bags % 3] << np.uint64(32)) | rows.astype(np.uint64)
    keys, seg_off, seg_bags = orc.dedup(b.ids, b.offsets)
    N = len(b.ids)
    # the index form of a batch: unique key -> positions holding it, nothing lost
    d = _dict_dedup(keys_occ, bags)
    assert len(keys) == len(d) == len(set(keys_occ.tolist()))
    np.testing.assert_array_equal(keys, np.unique(keys_occ))
    assert (np.diff(keys.astype(np.int64)) > 0).all()
    assert seg_off[0] == 0 and seg_off[-1] == N and len(seg_off) == len(keys) + 1
    for u, k in enumerate(keys):
        seg = seg_bags[seg_off[u]:seg_off[u + 1]]
        assert seg.tolist() == d[int(k)]               # batch order kept inside a segment
        assert (np.diff(seg.astype(np.int64)) >= 0).all()
    np.testing.assert_array_equal(np.sort(seg_bags), np.sort(bags))
    order = np.argsort(keys_occ, kind="stable")
    np.testing.assert_array_equal(seg_bags, bags[order])


def test_dedup_degenerate_cases():
    orc = make_oracle([(16, 8, W.F32)], [0])
    keys, seg_off, seg_bags = orc.dedup(np.zeros(0, np.uint64), np.zeros(5, np.int32))       # N = 0
    assert len(keys) == 0 and seg_off.tolist() == [0] and len(seg_bags) == 0
    keys, seg_off, seg_bags = orc.dedup(np.array([5], np.uint64), np.array([0, 1], np.int32))  # N = 1
    assert keys.tolist() == [5] and seg_off.tolist() == [0, 1] and seg_bags.tolist() == [0]
    ids = np.full(9, 21, np.uint64)                                                        # all equal
    keys, seg_off, seg_bags = orc.dedup(ids, np.array([0, 2, 2, 9], np.int32))
    assert keys.tolist() == [5] and seg_off.tolist() == [0, 9] and seg_bags.tolist() == [0, 0, 2, 2, 2, 2, 2, 2, 2]
    ids = np.arange(15, -1, -1, dtype=np.uint64)                                           # all distinct
    keys, seg_off, seg_bags = orc.dedup(ids, np.arange(17, dtype=np.int32))
    assert keys.tolist() == list(range(16)) and seg_off.tolist() == list(range(17))
    assert seg_bags.tolist() == list(range(15, -1, -1))


def test_sample_indices_fit_uint16_for_paper_batch_bound():
    # section 4.2.3: with batch <= 65535 (here even 65536) the sample index bag // S fits 16 bits
    S, B = 3, 65536
    assert (B * S - 1) // S == 65535 < (1 << 16)


# ----------------------------------------------------------------------------- gradient (a5)
def _setup_grad_case(seed=4, R=40, D=8, S=3, B=25, hash_kind=W.HASH_MIX_MOD):
    orc = make_oracle([(R, D, W.F32)], [0] * S, hash_kind=hash_kind)
    b = W.random_batch(seed, B, S, 6, 1 << 20)
    dp = np.random.default_rng(seed).standard_normal((B, S * D)).astype(np.float32)
    return orc, b, dp


def test_gradient_matches_autograd_and_count_matrix_transpose():
    orc, b, dp = _setup_grad_case()
    R, D = 40, 8
    rows = orc.hash_rows(b.ids, b.offsets)
    G = orc.gradient(b.ids, b.offsets, dp).reshape(-1, D)
    keys, seg_off, _ = orc._dedup_out()
    Wt = torch.from_numpy(table_values(orc, 0)[0].astype(np.float64)).requires_grad_(True)
    out = _torch_pool(Wt, rows, b.offsets)                      # [Bags, D]
    out.backward(torch.from_numpy(dp.astype(np.float64)).reshape(-1, D))
    dense = Wt.grad.numpy()
    touched = (keys & np.uint64(0xFFFFFFFF)).astype(np.int64)
    np.testing.assert_allclose(G, dense[touched], rtol=1e-12, atol=1e-12)
    mask = np.ones(R, bool)
    mask[touched] = False
    assert (dense[mask] == 0).all()
    brute = count_matrix(rows, b.offsets, R).T @ dp.astype(np.float64).reshape(-1, D)
    np.testing.assert_allclose(G, brute[touched], rtol=1e-12, atol=1e-12)
    # mass conservation: sum_u G[u] = sum_bags len(bag) * d_pooled[bag]
    lens = np.diff(b.offsets).astype(np.float64)
    np.testing.assert_allclose(G.sum(0), (lens[:, None] * dp.astype(np.float64).reshape(-1, D)).sum(0), rtol=1e-11)


def test_gradient_is_the_derivative_of_the_linear_map():
    # W -> <pooled(W), Gamma> is linear, so a finite difference is exact up to fp32 rounding of pooled
    orc, b, dp = _setup_grad_case(seed=6, R=16, D=8, S=2, B=10, hash_kind=W.HASH_IDENTITY_MOD)
    G = orc.gradient(b.ids, b.offsets, dp).reshape(-1, 8)
    keys, _, _ = orc._dedup_out()
    allr = np.arange(16, dtype=np.uint64)
    orc.write_rows(0, allr, np.zeros((16, 8), np.float32))
    for u in (0, len(keys) // 2, len(keys) - 1):
        r = int(keys[u] & np.uint64(0xFFFFFFFF))
        for d in (0, 5):
            e = np.zeros((1, 8), np.float32)
            e[0, d] = 1.0
            orc.write_rows(0, np.array([r], np.uint64), e)
            f = (orc.lookup_pool(b.ids, b.offsets).astype(np.float64) * dp).sum()
            orc.write_rows(0, np.array([r], np.uint64), np.zeros((1, 8), np.float32))
            assert abs(f - G[u, d]) < 1e-9


# ----------------------------------------------------------------------------- optimizer (a6)
def _dense_grad(orc, b, dp, R, D):
    rows = orc.hash_rows(b.ids, b.offsets)
    return count_matrix(rows, b.offsets, R).T @ dp.astype(np.float64).reshape(-1, D)


def test_sgd_matches_torch_sgd_and_leaves_other_rows_alone():
    R, D, S, B = 64, 8, 2, 12
    orc = make_oracle([(R, D, W.F32)], [0] * S, hash_kind=W.HASH_MIX_MOD, opt=W.OPT_SGD, lr=0.01)
    w0, a0 = table_values(orc, 0)
    p = torch.nn.Parameter(torch.from_numpy(w0.astype(np.float64)))
    sgd = torch.optim.SGD([p], lr=float(np.float32(0.01)))
    for step in range(3):
        b = W.random_batch(20 + step, B, S, 4, 1 << 20)
        dp = np.random.default_rng(step).standard_normal((B, S * D)).astype(np.float32)
        before, _ = table_values(orc, 0)
        p.grad = torch.from_numpy(_dense_grad(orc, b, dp, R, D))
        keys, _, _ = orc.backward_update(b.ids, b.offsets, dp)
        sgd.step()
        after, acc = table_values(orc, 0)
        np.testing.assert_allclose(after, p.detach().numpy(), rtol=3e-7, atol=1e-9)
        untouched = np.ones(R, bool)
        untouched[(keys & np.uint64(0xFFFFFFFF)).astype(np.int64)] = False
        assert untouched.any()
        np.testing.assert_array_equal(after[untouched], before[untouched])
        np.testing.assert_array_equal(acc, a0)
        p.data = torch.from_numpy(after.astype(np.float64))     # follow the fp32-rounded trajectory


def test_rowwise_adagrad_dim1_is_textbook_adagrad():
    R, S, B = 32, 2, 10
    lr, eps, acc0 = 0.05, 1e-8, 0.1
    orc = make_oracle([(R, 1, W.F32)], [0] * S, hash_kind=W.HASH_MIX_MOD, opt=W.OPT_ROWWISE_ADAGRAD, lr=lr, eps=eps,
                      acc_init=acc0)
    w0, _ = table_values(orc, 0)
    p = torch.nn.Parameter(torch.from_numpy(w0.astype(np.float64)))
    ada = torch.optim.Adagrad([p], lr=float(np.float32(lr)), eps=float(np.float32(eps)),
                              initial_accumulator_value=float(np.float32(acc0)))
    for step in range(4):
        b = W.random_batch(40 + step, B, S, 4, 1 << 20)
        dp = np.random.default_rng(100 + step).standard_normal((B, S)).astype(np.float32)
        p.grad = torch.from_numpy(_dense_grad(orc, b, dp, R, 1))
        orc.backward_update(b.ids, b.offsets, dp)
        ada.step()
        after, acc = table_values(orc, 0)
        np.testing.assert_allclose(after, p.detach().numpy(), rtol=1e-6, atol=4e-9)
        np.testing.assert_allclose(acc, ada.state[p]["sum"].numpy().ravel(), rtol=1e-6)
        p.data = torch.from_numpy(after.astype(np.float64))
        ada.state[p]["sum"] = torch.from_numpy(acc.astype(np.float64)[:, None].copy())


def test_rowwise_adagrad_equal_magnitude_rows_reduce_to_elementwise_adagrad():
    # if |G_d| is the same for every d of a row, mean_d G_d^2 = G_d^2 and row-wise == element-wise
    R, D, S, B = 32, 8, 1, 16
    lr, eps, acc0 = 0.05, 1e-8, 0.1
    orc = make_oracle([(R, D, W.F32)], [0], hash_kind=W.HASH_IDENTITY_MOD, opt=W.OPT_ROWWISE_ADAGRAD, lr=lr, eps=eps,
                      acc_init=acc0)
    w0, _ = table_values(orc, 0)
    p = torch.nn.Parameter(torch.from_numpy(w0.astype(np.float64)))
    ada = torch.optim.Adagrad([p], lr=float(np.float32(lr)), eps=float(np.float32(eps)),
                              initial_accumulator_value=float(np.float32(acc0)))
    rng = np.random.default_rng(3)
    for step in range(3):
        ids = rng.permutation(R)[:B].astype(np.uint64)          # distinct rows, one per bag
        off = np.arange(B + 1, dtype=np.int32)
        mag = rng.uniform(0.5, 2.0, size=(B, 1)).astype(np.float32)
        dp = (mag * rng.choice([-1.0, 1.0], size=(B, D))).astype(np.float32)
        g = np.zeros((R, D))
        g[ids.astype(np.int64)] = dp
        p.grad = torch.from_numpy(g)
        orc.backward_update(ids, off, dp)
        ada.step()
        after, acc = table_values(orc, 0)
        np.testing.assert_allclose(after, p.detach().numpy(), rtol=1e-6, atol=4e-9)   # one fp32 rounding at |w|<0.06
        np.testing.assert_allclose(acc, ada.state[p]["sum"].numpy()[:, 0], rtol=1e-6)
        p.data = torch.from_numpy(after.astype(np.float64))     # follow the fp32-rounded trajectory
        ada.state[p]["sum"] = torch.from_numpy(np.repeat(acc.astype(np.float64)[:, None], D, 1))


def test_rowwise_adagrad_uses_mean_not_sum_and_eps_outside_sqrt():
    # one row hit once: closed form with numbers a sum / eps-inside reading would miss
    lr, eps, acc0 = 0.5, 0.25, 1.0
    orc = make_oracle([(4, 4, W.F32)], [0], opt=W.OPT_ROWWISE_ADAGRAD, lr=lr, eps=eps, acc_init=acc0)
    orc.write_rows(0, np.arange(4, dtype=np.uint64), np.ones((4, 4), np.float32))
    dp = np.array([[2.0, -2.0, 4.0, 0.0]], np.float32)          # mean g^2 = 6 -> acc 7
    orc.backward_update(np.array([2], np.uint64), np.array([0, 1], np.int32), dp)
    w, acc = table_values(orc, 0)
    assert acc.tolist() == [1.0, 1.0, 7.0, 1.0]
    denom = math.sqrt(7.0) + 0.25
    np.testing.assert_allclose(w[2], 1.0 - 0.5 * dp[0] / denom, rtol=1e-7)
    assert (w[[0, 1, 3]] == 1.0).all()


def test_adagrad_accumulator_monotone_and_duplicates_updated_once():
    R, D = 16, 8
    orc = make_oracle([(R, D, W.F32)], [0, 0], hash_kind=W.HASH_IDENTITY_MOD, opt=W.OPT_ROWWISE_ADAGRAD, lr=0.05)
    prev = table_values(orc, 0)[1]
    for step in range(3):
        b = W.random_batch(60 + step, 8, 2, 5, R)
        dp = np.random.default_rng(step).standard_normal((8, 2 * D)).astype(np.float32)
        w_before = table_values(orc, 0)[0].astype(np.float64)
        G = _dense_grad(orc, b, dp, R, D)
        orc.backward_update(b.ids, b.offsets, dp)
        w, acc = table_values(orc, 0)
        assert (acc >= prev).all()
        # one update per unique row with the batch-summed gradient, however often the row occurs
        a_new = prev.astype(np.float64) + (G ** 2).mean(1)
        want = w_before - float(np.float32(0.05)) * G / (np.sqrt(a_new) + float(np.float32(1e-8)))[:, None]
        np.testing.assert_allclose(w, want, rtol=2e-7, atol=1e-10)
        prev = acc


def test_bf16_table_update_rounds_once_to_nearest_even():
    R, D = 8, 8
    orc = make_oracle([(R, D, W.BF16)], [0], hash_kind=W.HASH_IDENTITY_MOD, opt=W.OPT_SGD, lr=0.01)
    w0, _ = table_values(orc, 0)
    dp = np.random.default_rng(1).standard_normal((3, D)).astype(np.float32)
    ids = np.array([1, 1, 6], np.uint64)
    orc.backward_update(ids, np.array([0, 1, 2, 3], np.int32), dp)
    w, _ = table_values(orc, 0)
    lr = Fraction(float(np.float32(0.01)))
    for d in range(D):     # exact arithmetic, one rounding to the bf16 grid
        want = to_bf16_exact(Fraction(float(w0[1, d])) - lr * (Fraction(float(dp[0, d])) + Fraction(float(dp[1, d]))))
        assert Fraction(float(w[1, d])) == want
    np.testing.assert_array_equal(w[[0, 2, 3, 4, 5, 7]], w0[[0, 2, 3, 4, 5, 7]])


def test_bf16_table_update_does_not_round_through_fp32():
    # w = 1, lr * G chosen so that w - lr G sits a hair above the tie between the bf16 neighbours 1 and 1 + 2^-7:
    # fp64 -> fp32 lands exactly on the tie and a second rounding would then go to the even neighbour 1.0
    orc = make_oracle([(4, 8, W.BF16)], [0], hash_kind=W.HASH_IDENTITY_MOD, opt=W.OPT_SGD, lr=1.0)
    orc.write_rows(0, np.arange(4, dtype=np.uint64), np.ones((4, 8), np.float32))
    g = np.float32(-(2.0 ** -8 + 2.0 ** -30))                  # exact in fp32; 1 - g = 1 + 2^-8 + 2^-30
    dp = np.full((1, 8), g, np.float32)
    orc.backward_update(np.array([2], np.uint64), np.array([0, 1], np.int32), dp)
    w, _ = table_values(orc, 0)
    assert (w[2] == np.float32(1.0 + 2.0 ** -7)).all()
    assert float(np.float32(1.0 - float(g))) == 1.0 + 2.0 ** -8   # what fp32 would have kept: the exact tie


def test_sparse_and_dense_oracle_agree_over_steps():
    w = W.make_workload(1, scale=1 / 64)
    dense = O.Oracle.from_config(w.cfg, dense=True)
    sparse = O.Oracle.from_config(w.cfg, dense=False)
    for step in range(2):
        b = W.make_batch(w, step)
        dp = W.make_d_pooled(w, step)
        np.testing.assert_array_equal(dense.lookup_pool(b.ids, b.offsets), sparse.lookup_pool(b.ids, b.offsets))
        k1, o1, g1 = dense.backward_update(b.ids, b.offsets, dp)
        k2, o2, g2 = sparse.backward_update(b.ids, b.offsets, dp)
        np.testing.assert_array_equal(k1, k2)
        np.testing.assert_array_equal(o1, o2)
        np.testing.assert_array_equal(g1, g2)
    rows = (k1 & np.uint64(0xFFFFFFFF))
    for a, c in zip(dense.read_rows(0, rows), sparse.read_rows(0, rows)):
        np.testing.assert_array_equal(a, c)
