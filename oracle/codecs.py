"""Software bf16 and OCP e4m3 codecs for the oracle (test infrastructure only).

bf16: 1 sign, 8 exponent, 7 mantissa bits = the upper half of an IEEE binary32.
e4m3 (OCP "FN" flavour, the FP8 precision named in Sec. 8.1 of the paper as it
exists on gfx950): 1 sign, 4 exponent bits with bias 7, 3 mantissa bits, no
infinities, 0x7f/0xff are NaN, largest finite value 448 = 1.75 * 2^8, smallest
subnormal 2^-9.  All conversions round to nearest, ties to even, and the e4m3
encoder saturates at +-448.
"""
import numpy as np

E4M3_MAX = 448.0


# --------------------------------------------------------------------------- bf16
def f32_to_bf16_bits(a):
    """binary32 array -> uint16 bf16 bit patterns, round-to-nearest-even."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    nan = np.isnan(a)
    if nan.any():
        r = np.where(nan, (u >> np.uint32(16)) | np.uint32(0x40), r)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b):
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(a):
    """Value of `a` (any float array) after one rounding to bf16, as float64.

    The input is first taken to binary32 (exact for values that already are
    binary32; one extra rounding otherwise, used only where the method itself
    holds the value in binary32)."""
    return bf16_bits_to_f32(f32_to_bf16_bits(np.asarray(a, dtype=np.float32))).astype(np.float64)


def f64_to_bf16_value(a):
    """float64 -> nearest bf16 value (ties to even) without passing through
    binary32, so there is no double rounding.  Returns float64."""
    a = np.asarray(a, dtype=np.float64)
    out = np.zeros_like(a)
    nz = (a != 0) & np.isfinite(a)
    m, e = np.frexp(a[nz])              # a = m * 2^e, 0.5 <= |m| < 1
    e = np.maximum(e, -125)             # bf16 subnormal grid: 2^-133 = 2^(-125-8)
    q = np.rint(np.ldexp(a[nz], 8 - e))  # 8 significant bits
    out[nz] = np.ldexp(q, e - 8)
    out[~np.isfinite(a)] = a[~np.isfinite(a)]
    return out


# --------------------------------------------------------------------------- e4m3
def e4m3_decode_table():
    """All 256 codes -> float64 value, straight from the bit fields."""
    t = np.empty(256, dtype=np.float64)
    for c in range(256):
        s = -1.0 if c & 0x80 else 1.0
        ex = (c >> 3) & 0xF
        mn = c & 0x7
        if ex == 0xF and mn == 0x7:
            t[c] = np.nan
        elif ex == 0:
            t[c] = s * (mn / 8.0) * 2.0 ** -6
        else:
            t[c] = s * (1.0 + mn / 8.0) * 2.0 ** (ex - 7)
    return t


_DEC = e4m3_decode_table()


def e4m3_decode(codes):
    return _DEC[np.asarray(codes, dtype=np.uint8)]


def e4m3_encode(a):
    """Float array -> uint8 e4m3 codes: nearest representable value, ties to the
    even mantissa, magnitudes above 448 saturate to 448, NaN -> 0x7f."""
    a = np.asarray(a, dtype=np.float64)
    mag = np.minimum(np.abs(a), E4M3_MAX)
    mag = np.where(np.isnan(a), 0.0, mag)
    # exponent of the grid the value falls in; subnormals share exponent -6
    _, e = np.frexp(mag)                 # mag = m * 2^e with m in [0.5,1) -> floor(log2) = e-1
    fl = np.maximum(e - 1, -6)
    step = np.ldexp(1.0, fl - 3)         # spacing of representable values there
    q = np.rint(mag / step)              # ties to even; may reach 16 = next binade
    val = q * step
    # value -> code through the bit fields
    _, e2 = np.frexp(val)
    ex = np.maximum(e2 - 1, -6)
    is_sub = val < 2.0 ** -6
    mant = np.where(is_sub, np.rint(val * 2.0 ** 9), np.rint((val / np.ldexp(1.0, ex) - 1.0) * 8.0))
    expf = np.where(is_sub, 0, ex + 7)
    code = (expf.astype(np.int64) << 3) | mant.astype(np.int64)
    code = np.where(val == 0, 0, code)
    code = code | np.where(np.signbit(a), 0x80, 0)
    code = np.where(np.isnan(a), 0x7F, code)
    return code.astype(np.uint8)


def quantize_rows_e4m3(v):
    """Per-row dynamic quantisation used for fp8 activations and, with rows =
    output channels, for fp8 weights.  Every step is IEEE binary32:
        s = amax(|row|) / 448      (s = 1 for an all-zero row)
        q = e4m3(row / s)          (true division, then one rounding)
    Returns (codes uint8 [R,C], scales float32 [R])."""
    v = np.ascontiguousarray(v, dtype=np.float32)
    amax = np.max(np.abs(v), axis=1).astype(np.float32)
    s = (amax / np.float32(E4M3_MAX)).astype(np.float32)
    s = np.where(amax == 0, np.float32(1.0), s).astype(np.float32)
    scaled = (v / s[:, None]).astype(np.float32)
    return e4m3_encode(scaled), s


def dequantize_rows_e4m3(codes, s):
    """codes [R,C], s [R] -> float64 values code*scale (exact in float64)."""
    return e4m3_decode(codes) * np.asarray(s, dtype=np.float64)[:, None]
