"""CPU checks of the test helper that restates the library's block-scaled 16-bit storage of the
down projection's output (tests/y_block16.py): values by hand, the error bound, exactness."""
import numpy as np

import y_block16 as yb


def test_block16_storage_codec():
    """The library's own storage format of the down projection's output (blocks of 16 columns,
    int16 codes, shared power-of-two scale): values by hand, the error bound, exactness."""
    # one block by hand: amax = 3.0 -> exponent 128, k = 128, scale 2^-13; 3.0 -> 24576, 1.0 -> 8192
    y = np.zeros((1, 16), dtype=np.float32)
    y[0, :4] = [3.0, -1.0, 2.0 ** -13, 2.0 ** -14]
    c, k = yb.quantize_blocks_i16(y)
    assert k[0, 0] == 128 and c[0, :4].tolist() == [24576, -8192, 1, 0]      # 0.5 rounds to even (0)
    assert np.array_equal(yb.dequantize_blocks_i16(c, k)[0, :3], y[0, :3])
    # the largest code would round to 32768: the exponent moves up by one
    y[0, 0] = np.float32(4.0) - np.float32(2.0 ** -14)       # 4 - 2^-14 = 2^1 * (2 - 2^-15): top 15 mantissa bits set
    c, k = yb.quantize_blocks_i16(y)
    assert k[0, 0] == 129 and c[0, 0] == 16384
    y[0, 0] = np.float32(4.0) - np.float32(2.0 ** -13)       # just below: stays, code 32767
    c, k = yb.quantize_blocks_i16(y)
    assert k[0, 0] == 128 and c[0, 0] == 32767
    # zero block and tiny values: k is held at 15, codes are exact multiples of 2^-126
    z = np.zeros((2, 32), dtype=np.float32)
    z[1, 16] = np.float32(2.0 ** -126)
    c, k = yb.quantize_blocks_i16(z)
    assert k.tolist() == [[15, 15], [15, 15]] and c[1, 16] == 1 and np.count_nonzero(c) == 1
    # random rows: error at most half a code step = 2^(k-142) <= amax/32768; codes use the range
    rng = np.random.default_rng(0)
    r = (rng.standard_normal((64, 256)) * np.exp(rng.standard_normal((64, 1)) * 3)).astype(np.float32)
    c, k = yb.quantize_blocks_i16(r)
    d = yb.dequantize_blocks_i16(c, k)
    half = np.repeat(np.ldexp(1.0, k.astype(np.int64) - 142), 16, axis=1)
    amax = np.repeat(np.abs(r).reshape(64, 16, 16).max(-1), 16, axis=1)
    assert np.all(np.abs(d.astype(np.float64) - r) <= half) and np.all(half <= amax / 32768.0 * (1 + 1e-12))
    assert np.abs(c).reshape(64, 16, 16).max(-1).min() >= 16384
    # values that are already multiples of the block's step come back exactly
    e = (rng.integers(-32767, 32768, size=(8, 16)) * 2.0 ** -20).astype(np.float32)
    e[:, 0] = np.float32(32767 * 2.0 ** -20)
    c, k = yb.quantize_blocks_i16(e)
    assert np.array_equal(yb.dequantize_blocks_i16(c, k), e)


def test_block16_non_finite_values():
    """An overflowed accumulator stays visible: a block with +-Inf reads back as NaN in all of its
    16 elements and leaves its neighbours alone; a NaN element alone reads back as 0."""
    y = np.ones((1, 48), dtype=np.float32)
    y[0, 20] = -np.inf
    y[0, 40] = np.nan
    c, k = yb.quantize_blocks_i16(y)
    assert k[0].tolist() == [127, 255, 127]
    d = yb.dequantize_blocks_i16(c, k)
    assert np.array_equal(d[0, :16], y[0, :16]) and np.all(np.isnan(d[0, 16:32]))
    assert d[0, 40] == 0.0 and np.array_equal(np.delete(d[0, 32:], 8), np.ones(15, dtype=np.float32))
