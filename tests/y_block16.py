"""Test helper, not part of the method's oracle: the library's own storage format of the down
projection's output between its down-projection and combine kernels (declared with
MOE_FLAG_Y_F32 in include/moe_prefill.h), restated in numpy so that GPU tests can apply it to
float32 values bit for bit.  Blocks of 16 adjacent columns share a power-of-two scale."""
import numpy as np

Y_BLOCK = 16


def quantize_blocks_i16(y32):
    """y32: float32 [rows, H], H a multiple of 16.  Returns (codes int16 [rows, H], k uint8
    [rows, H/16]): per block amax = max|v|; k = biased float32 exponent of amax, one higher when
    amax * 2^(141-k) >= 32767.5 (the top 15 mantissa bits of amax all set), at least 15;
    code = rint(v * 2^(141-k)) (round half to even); value = 2^(k-141) * code.  A block that holds
    +-Inf gets k = 255 and reads back as NaN throughout; a NaN element gets code 0."""
    y32 = np.ascontiguousarray(y32, dtype=np.float32)
    rows, H = y32.shape
    b = y32.reshape(rows, H // Y_BLOCK, Y_BLOCK)
    amax = np.fmax.reduce(np.abs(b), axis=-1)                   # the kernel's maximum skips NaN operands
    bits = amax.view(np.uint32).astype(np.int64)
    k = np.maximum((bits + 0x100) >> 23, 15)
    with np.errstate(invalid="ignore"):
        codes = np.rint(np.ldexp(b.astype(np.float64), (141 - k)[..., None].astype(np.int64)))
    codes = np.where(np.isfinite(codes), codes, 0.0)          # the low 16 bits of Inf + 1.5 * 2^23 and of NaN are 0
    assert np.all(np.abs(codes) <= 32767)
    return codes.astype(np.int16).reshape(rows, H), k.astype(np.uint8)


def dequantize_blocks_i16(codes, k):
    rows, H = codes.shape
    c = codes.reshape(rows, H // Y_BLOCK, Y_BLOCK).astype(np.float64)
    v = np.ldexp(c, (k.astype(np.int64) - 141)[..., None])
    v = np.where((k == 255)[..., None], np.nan, v)
    return v.astype(np.float32).reshape(rows, H)
