"""Pins for oracle/formats.py: format definitions, exhaustive tables, and PyTorch's CPU casts as an
independent implementation of the same conversions."""
import numpy as np
import torch

from oracle import formats as F


def test_bf16_decode_is_top_half_of_float32():
    assert F.bf16_to_f32(np.array([0x3F80, 0xC000, 0x0000, 0x8000, 0x3DCD], dtype=np.uint16)).tolist()[:2] == [1.0, -2.0]
    x = F.bf16_to_f32(np.array([0x3DCD], dtype=np.uint16))[0]
    assert abs(float(x) - 0.1) < 0.1 * 2 ** -8


def test_bf16_roundtrip_all_finite_patterns():
    allb = np.arange(65536, dtype=np.uint16)
    f = F.bf16_to_f32(allb)
    fin = np.isfinite(f)
    assert np.array_equal(F.f32_to_bf16_rne(f[fin]), allb[fin])


def test_bf16_rne_ties_by_hand():
    # 1 + 2^-8 lies exactly between 1.0 (even mantissa) and 1 + 2^-7: ties to even -> 1.0
    assert F.f32_to_bf16_rne(np.array([1.0 + 2.0 ** -8], dtype=np.float32))[0] == 0x3F80
    # 1 + 3*2^-8 lies between 1+2^-7 (odd) and 1+2^-6 (even) -> 1+2^-6
    assert F.f32_to_bf16_rne(np.array([1.0 + 3 * 2.0 ** -8], dtype=np.float32))[0] == 0x3F82
    # just above the tie rounds up
    assert F.f32_to_bf16_rne(np.array([np.nextafter(np.float32(1.0 + 2.0 ** -8), np.float32(2))], dtype=np.float32))[0] == 0x3F81


def test_bf16_rne_matches_torch_cast():
    rng = np.random.default_rng(1)
    y = (rng.standard_normal(500000) * np.exp(rng.uniform(-20, 20, 500000))).astype(np.float32)
    ref = torch.from_numpy(y).to(torch.bfloat16).view(torch.uint16).numpy()
    assert np.array_equal(ref, F.f32_to_bf16_rne(y))


def test_e4m3_decode_table_by_definition():
    assert F.e4m3_to_f32(np.array([0x38], dtype=np.uint8))[0] == 1.0          # e=7,m=0
    assert F.e4m3_to_f32(np.array([0x7E], dtype=np.uint8))[0] == 448.0        # e=15,m=6
    assert F.e4m3_to_f32(np.array([0x01], dtype=np.uint8))[0] == 2.0 ** -9    # smallest subnormal
    assert F.e4m3_to_f32(np.array([0x08], dtype=np.uint8))[0] == 2.0 ** -6    # smallest normal
    assert F.e4m3_to_f32(np.array([0xC4], dtype=np.uint8))[0] == -3.0
    assert np.isnan(F.e4m3_to_f32(np.array([0x7F], dtype=np.uint8))[0])
    allc = np.arange(256, dtype=np.uint8)
    ref = torch.from_numpy(allc.copy()).view(torch.float8_e4m3fn).float().numpy()
    got = F.e4m3_to_f32(allc)
    assert np.array_equal(np.isnan(ref), np.isnan(got))
    ok = ~np.isnan(ref)
    assert np.array_equal(ref[ok], got[ok])


def test_e4m3_encode_roundtrip_and_ties():
    allc = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    assert np.array_equal(F.f32_to_e4m3_rne_sat(F.e4m3_to_f32(allc)), allc)
    # 1.0625 is halfway between 1.0 (m=0, even) and 1.125 (m=1): ties to even -> 1.0
    assert F.f32_to_e4m3_rne_sat(np.array([1.0625], dtype=np.float32))[0] == 0x38
    # 1.1875 halfway between 1.125 (odd) and 1.25 (even) -> 1.25
    assert F.f32_to_e4m3_rne_sat(np.array([1.1875], dtype=np.float32))[0] == 0x3A
    # saturation and subnormal rounding: 2^-10 is half the smallest subnormal -> ties to even -> 0
    assert F.f32_to_e4m3_rne_sat(np.array([1e6, -1e6, 2.0 ** -10, 3 * 2.0 ** -10], dtype=np.float32)).tolist() == [0x7E, 0xFE, 0x00, 0x02]
    # 15.5 * 2^-6 * ... carry into the next binade: 1.96875 -> 2.0
    assert F.f32_to_e4m3_rne_sat(np.array([1.96875], dtype=np.float32))[0] == 0x40


def test_e4m3_encode_matches_torch_cast_in_range():
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(300000) * np.exp(rng.uniform(-12, 5, 300000))).astype(np.float32)
    x = np.clip(x, -448, 448)
    ref = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(ref, F.f32_to_e4m3_rne_sat(x))


def test_e5m2_decode_table_by_definition():
    assert F.e5m2_to_f32(np.array([0x3C], dtype=np.uint8))[0] == 1.0          # e=15,m=0
    assert F.e5m2_to_f32(np.array([0x7B], dtype=np.uint8))[0] == 57344.0      # e=30,m=3
    assert F.e5m2_to_f32(np.array([0x01], dtype=np.uint8))[0] == 2.0 ** -16   # smallest subnormal
    assert F.e5m2_to_f32(np.array([0x04], dtype=np.uint8))[0] == 2.0 ** -14   # smallest normal
    assert F.e5m2_to_f32(np.array([0xC2], dtype=np.uint8))[0] == -3.0
    assert np.isinf(F.e5m2_to_f32(np.array([0x7C], dtype=np.uint8))[0])
    assert np.isnan(F.e5m2_to_f32(np.array([0x7D], dtype=np.uint8))[0])
    allc = np.arange(256, dtype=np.uint8)
    # e5m2 is the top byte of an IEEE half: decode through numpy's float16 and through PyTorch's type
    half = (allc.astype(np.uint16) << 8).view(np.float16).astype(np.float32)
    ref = torch.from_numpy(allc.copy()).view(torch.float8_e5m2).float().numpy()
    got = F.e5m2_to_f32(allc)
    for r in (half, ref):
        assert np.array_equal(np.isnan(r), np.isnan(got))
        ok = ~np.isnan(r)
        assert np.array_equal(r[ok], got[ok])


def test_e5m2_encode_roundtrip_and_ties():
    allc = np.array([c for c in range(256) if (c & 0x7C) != 0x7C], dtype=np.uint8)
    assert np.array_equal(F.f32_to_e5m2_rne_sat(F.e5m2_to_f32(allc)), allc)
    # 1.125 is halfway between 1.0 (m=0, even) and 1.25 (m=1): ties to even -> 1.0
    assert F.f32_to_e5m2_rne_sat(np.array([1.125], dtype=np.float32))[0] == 0x3C
    # 1.375 halfway between 1.25 (odd) and 1.5 (even) -> 1.5
    assert F.f32_to_e5m2_rne_sat(np.array([1.375], dtype=np.float32))[0] == 0x3E
    # saturation (never infinity), and subnormal rounding: 2^-17 is half the smallest subnormal -> 0
    assert F.f32_to_e5m2_rne_sat(np.array([1e9, -1e9, 2.0 ** -17, 3 * 2.0 ** -17], dtype=np.float32)).tolist() == [0x7B, 0xFB, 0x00, 0x02]
    # carry into the next binade: 1.9375 -> 2.0
    assert F.f32_to_e5m2_rne_sat(np.array([1.9375], dtype=np.float32))[0] == 0x40


def test_e5m2_encode_matches_torch_cast_in_range():
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(300000) * np.exp(rng.uniform(-14, 9, 300000))).astype(np.float32)
    x = np.clip(x, -57344, 57344)
    ref = torch.from_numpy(x).to(torch.float8_e5m2).view(torch.uint8).numpy()
    assert np.array_equal(ref, F.f32_to_e5m2_rne_sat(x))


def test_cast_fp8_against_torch_and_by_hand():
    """Scale-then-cast: hand values, saturation at the format maximum, and PyTorch's float32 division +
    float8 casts as an independent implementation."""
    rng = np.random.default_rng(3)
    x = F.f32_to_bf16_rne(rng.standard_normal((64, 48)).astype(np.float32) * np.exp(rng.uniform(-6, 3, (64, 48))).astype(np.float32))
    x = x.reshape(64, 48)
    xf = torch.from_numpy(F.bf16_to_f32(x))
    for fmt, tdt, mx in (("e4m3", torch.float8_e4m3fn, 448.0), ("e5m2", torch.float8_e5m2, 57344.0)):
        amax_ref = float(xf.abs().max())
        scale = np.float32(amax_ref / mx)
        codes, amax = F.cast_fp8(x, scale, fmt)
        assert float(amax) == amax_ref
        ref = (xf / float(scale)).clamp(-mx, mx).to(tdt).view(torch.uint8).numpy()
        assert np.array_equal(codes, ref)
        # a scale that is too small saturates instead of overflowing
        codes, _ = F.cast_fp8(x, np.float32(scale / 64), fmt)
        dec = F.e4m3_to_f32(codes) if fmt == "e4m3" else F.e5m2_to_f32(codes)
        assert np.all(np.isfinite(dec)) and np.max(np.abs(dec)) == mx
    one = np.array([[0x3F80, 0xC000, 0x0000, 0x8000]], dtype=np.uint16)            # 1, -2, +0, -0
    codes, amax = F.cast_fp8(one, 0.5, "e4m3")
    assert codes.tolist() == [[0x40, 0xC8, 0x00, 0x80]] and amax == 2.0            # 2, -4, +0, -0
    codes, _ = F.cast_fp8(one, 0.5, "e5m2")
    assert codes.tolist() == [[0x40, 0xC4, 0x00, 0x80]]
