"""Pins of the value-codec oracle (section 4.2.3, lossy compression): error bound that follows from fp16's
11 significant bits, exact cases, scale behaviour, and an independent bit-level fp32->fp16 conversion."""
import numpy as np

from oracle import codec_oracle as C

KAPPA = 2.0 ** 15


def _blocks(seed, n_blocks, block_len, scale=1.0):
    return (np.random.default_rng(seed).standard_normal((n_blocks, block_len)) * scale).astype(np.float32)


def test_roundtrip_error_is_bounded_by_the_block_norm():
    for seed, scale in [(1, 1.0), (2, 1e-6), (3, 1e6), (4, 3e-30)]:
        v = _blocks(seed, 64, 200, scale)
        q, norm = C.compress(v, 200, KAPPA)
        out = C.decompress(q, norm, KAPPA)
        # |x*f| <= kappa = 2^15, fp16 keeps 11 significant bits, so the absolute error in the scaled domain is at most
        # half a unit in the last place of the largest binade: 2^15 * 2^-11 / 2 ... mapped back: ||v||_inf * 2^-11;
        # values below fp16's normal range after scaling (|x*f| < 2^-14) lose at most 2^-25 there, i.e. far less
        bound = norm[:, None].astype(np.float64) * 2.0 ** -11 * (1 + 1e-6)
        assert (np.abs(out.astype(np.float64) - v) <= bound).all()
        # and the error is relative to each element for elements within 2^11 of the norm
        big = np.abs(v) >= norm[:, None] * 2.0 ** -4
        assert (np.abs(out - v)[big] <= np.abs(v)[big] * 2.0 ** -10).all()


def test_uniform_fp16_cast_would_be_worse_for_small_blocks():
    # the reason the paper scales: a block of tiny values survives, a plain cast flushes it to zero
    v = _blocks(5, 4, 64, 1e-9)
    q, norm = C.compress(v, 64, KAPPA)
    out = C.decompress(q, norm, KAPPA)
    assert (v.astype(np.float16) == 0).all()
    assert np.abs(out - v).max() <= norm.max() * 2.0 ** -11


def test_exact_cases():
    # powers of two times small integers are exact in fp16 after scaling by a power of two
    v = np.array([[1.0, -0.5, 0.25, 0.0, 0.75, -1.0, 0.125, 0.5]], np.float32)
    q, norm = C.compress(v, 8, KAPPA)
    assert norm.tolist() == [1.0]
    np.testing.assert_array_equal(q.astype(np.float64), v * KAPPA)
    np.testing.assert_array_equal(C.decompress(q, norm, KAPPA), v)
    # a block of zeros
    q, norm = C.compress(np.zeros((3, 8), np.float32), 8, KAPPA)
    assert (q == 0).all() and (norm == 0).all()
    assert (C.decompress(q, norm, KAPPA) == 0).all()
    # the largest element maps to +-kappa up to one rounding of the factor
    v = _blocks(6, 32, 16)
    q, norm = C.compress(v, 16, KAPPA)
    assert np.abs(np.abs(q.astype(np.float64)).max(axis=1) - KAPPA).max() <= KAPPA * 2.0 ** -10


def test_power_of_two_scaling_of_the_input_leaves_the_codes_unchanged():
    v = _blocks(7, 16, 128)
    q1, n1 = C.compress(v, 128, KAPPA)
    q2, n2 = C.compress(v * np.float32(2.0 ** 20), 128, KAPPA)
    np.testing.assert_array_equal(q1.view(np.uint16), q2.view(np.uint16))
    np.testing.assert_array_equal(n2, n1 * np.float32(2.0 ** 20))
    np.testing.assert_array_equal(C.decompress(q2, n2, KAPPA), C.decompress(q1, n1, KAPPA) * np.float32(2.0 ** 20))


def _fp16_bits_rne(x):
    """Bit-level fp32 -> fp16 (round to nearest even) for finite |x| <= 65504, written from the formats."""
    out = np.zeros(x.shape, np.uint16)
    for i, f in enumerate(x.ravel()):
        u = int(np.float32(f).view(np.uint32))
        sign, e, m = (u >> 31) << 15, ((u >> 23) & 0xFF) - 127, u & 0x7FFFFF
        if (u & 0x7FFFFFFF) == 0:
            out.ravel()[i] = sign
            continue
        if e >= -14:                                  # normal in fp16
            val = ((e + 15) << 10) | (m >> 13)
            rem = m & 0x1FFF
            if rem > 0x1000 or (rem == 0x1000 and (val & 1)):
                val += 1                              # may carry into the exponent: still the right encoding
        else:                                         # subnormal in fp16: value = frac * 2^-24
            full = (m | 0x800000)                     # 24-bit significand, exponent e
            shift = -e - 14 + 13                      # bits dropped
            if shift > 25:
                val = 0
            else:
                val = full >> shift
                rem = full & ((1 << shift) - 1)
                half = 1 << (shift - 1)
                if rem > half or (rem == half and (val & 1)):
                    val += 1
        out.ravel()[i] = sign | val
    return out


def test_fp16_conversion_is_round_to_nearest_even():
    rng = np.random.default_rng(8)
    x = np.concatenate([rng.standard_normal(3000) * 1000, rng.standard_normal(2000) * 1e-5,
                        [2049.0, 2051.0, 1025.5, 2.0 ** -24, 2.0 ** -25, 3 * 2.0 ** -25, 65504.0, 0.0, -0.0]]).astype(np.float32)
    np.testing.assert_array_equal(x.astype(np.float16).view(np.uint16), _fp16_bits_rne(x))
