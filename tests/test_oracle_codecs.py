"""Pins for the oracle's bf16 / e4m3 codecs: the format's own definition
(enumerated table), round-trip, tie and saturation cases, and torch's CPU casts
as an independent implementation."""
import numpy as np
import torch

from oracle import codecs


def test_e4m3_table_facts():
    t = codecs.e4m3_decode_table()
    assert np.isnan(t[0x7F]) and np.isnan(t[0xFF])
    assert np.isfinite(t).sum() == 254
    assert t[0x7E] == 448.0 and t[0xFE] == -448.0
    assert t[0x01] == 2.0 ** -9 and t[0x08] == 2.0 ** -6 and t[0x38] == 1.0
    pos = t[:0x7F]
    assert np.all(np.diff(pos) > 0)
    assert np.array_equal(t[0x80:0xFF], -pos)


def test_e4m3_table_matches_torch():
    t = codecs.e4m3_decode_table()
    ref = torch.arange(256, dtype=torch.int16).to(torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(np.isnan(t), np.isnan(ref))
    m = ~np.isnan(t)
    assert np.array_equal(t[m], ref[m])


def test_e4m3_roundtrip_all_codes():
    t = codecs.e4m3_decode_table()
    codes = np.array([c for c in range(256) if c not in (0x7F, 0xFF)], dtype=np.uint8)
    assert np.array_equal(codecs.e4m3_encode(t[codes]), codes)


def test_e4m3_ties_to_even_and_saturation():
    t = codecs.e4m3_decode_table()
    for c in range(0, 0x7E):
        mid = 0.5 * (t[c] + t[c + 1])
        want = c if c % 2 == 0 else c + 1
        assert codecs.e4m3_encode(np.array([mid]))[0] == want, c
        assert codecs.e4m3_encode(np.array([-mid]))[0] == (want | 0x80), c
        assert codecs.e4m3_encode(np.array([np.nextafter(mid, np.inf)]))[0] == c + 1
        assert codecs.e4m3_encode(np.array([np.nextafter(mid, -np.inf)]))[0] == c
    sat = codecs.e4m3_encode(np.array([448.0, 449.0, 463.9, 464.0, 480.0, 1e30, np.inf, -1e30, -np.inf]))
    assert list(sat) == [0x7E] * 7 + [0xFE] * 2
    assert codecs.e4m3_encode(np.array([np.nan]))[0] == 0x7F
    assert codecs.e4m3_encode(np.array([2.0 ** -10]))[0] == 0      # tie between 0 and 2^-9 -> even (0)
    assert codecs.e4m3_encode(np.array([2.0 ** -10 * 1.01]))[0] == 1


def test_e4m3_encode_matches_torch_in_range():
    rng = np.random.default_rng(5)
    v = np.concatenate([rng.standard_normal(200000) * s for s in (1e-3, 0.05, 1.0, 30.0, 150.0)]).astype(np.float32)
    v = v[np.abs(v) <= 448.0]
    ref = torch.from_numpy(v).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = codecs.e4m3_encode(v)
    # torch keeps the sign of values that round to zero; so does the encoder
    assert np.array_equal(got, ref)


def test_bf16_matches_torch_exhaustive_upper_bits():
    rng = np.random.default_rng(7)
    hi = np.arange(65536, dtype=np.uint32) << np.uint32(16)
    for lo in (0, 1, 0x7FFF, 0x8000, 0x8001, 0xFFFF):
        u = hi | np.uint32(lo)
        f = u.view(np.float32)
        ok = ~np.isnan(f)
        ref = torch.from_numpy(f.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        got = codecs.f32_to_bf16_bits(f)
        assert np.array_equal(got[ok], ref[ok])
    lo = rng.integers(0, 65536, size=65536, dtype=np.uint32)
    f = (hi | lo).view(np.float32)
    ok = ~np.isnan(f)
    ref = torch.from_numpy(f.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(codecs.f32_to_bf16_bits(f)[ok], ref[ok])
    assert np.array_equal(codecs.bf16_bits_to_f32(ref[ok]),
                          torch.from_numpy(ref[ok].view(np.int16)).view(torch.bfloat16).float().numpy())


def test_f64_to_bf16_value():
    rng = np.random.default_rng(11)
    f = (rng.standard_normal(100000) * np.exp(rng.uniform(-30, 30, 100000))).astype(np.float32)
    assert np.array_equal(codecs.f64_to_bf16_value(f.astype(np.float64)), codecs.round_to_bf16(f))
    # a float64 just above a bf16 midpoint that binary32 would first round down onto the midpoint
    x = 1.0 + 2.0 ** -8 + 2.0 ** -40
    assert codecs.f64_to_bf16_value(np.array([x]))[0] == 1.0 + 2.0 ** -7
    assert codecs.f64_to_bf16_value(np.array([1.0 + 2.0 ** -8]))[0] == 1.0          # tie -> even
    assert codecs.f64_to_bf16_value(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    assert codecs.f64_to_bf16_value(np.array([0.0, -0.0, 2.0 ** -133, 2.0 ** -134]))[2] == 2.0 ** -133


def test_quantize_rows():
    rng = np.random.default_rng(3)
    v = (rng.standard_normal((64, 96)) * np.exp(rng.uniform(-6, 6, (64, 1)))).astype(np.float32)
    v[5] = 0.0
    q, s = codecs.quantize_rows_e4m3(v)
    assert s.dtype == np.float32 and q.dtype == np.uint8
    assert s[5] == 1.0 and np.all(q[5] == 0)
    amax = np.abs(v).max(axis=1)
    assert np.array_equal(s[amax > 0], (amax / np.float32(448.0))[amax > 0])
    # the row's largest magnitude lands on +-448
    r = np.arange(64)
    j = np.abs(v).argmax(axis=1)
    assert np.all((q[r, j] & 0x7F)[amax > 0] == 0x7E)
    # independent quantiser: torch float32 division + torch's e4m3 cast
    tv = torch.from_numpy(v)
    ts = torch.from_numpy(s)
    ref = (tv / ts[:, None]).clamp(-448, 448).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(q, ref)
    d = codecs.dequantize_rows_e4m3(q, s)
    assert np.max(np.abs(d - v) / np.maximum(amax[:, None], 1e-30)) <= 2.0 ** -4 / 1.75 + 1e-7
