"""The oracle's plain C routines (oracle/native) against their numpy reference forms, element for element.

The numpy forms carry the pins to the paper; these tests make the C forms interchangeable with them, so
that the parity tests at the full workload sizes can afford to compare every element."""
import numpy as np
import pytest

from oracle import formats as F
from oracle import mvue as M
from oracle import native as N
from oracle import projection as P


def _bf16_patterns(rs, shape, std):
    return F.f32_to_bf16_rne((rs.standard_normal(shape) * std).astype(np.float32)).reshape(shape)


@pytest.mark.parametrize("fmt", ["e4m3", "e5m2"])
def test_cast_equals_numpy_on_every_finite_bf16_pattern_and_on_gaussians(fmt):
    every = np.arange(1 << 16, dtype=np.uint16)
    every = every[(every & 0x7F80) != 0x7F80]                      # finite patterns, both signs, subnormals, zeros
    for scale in (1.0, 0.37, 2.0 ** -20, 3.1e4, 1.0e-30, 7.0e33):
        a, amax_a = N.cast_fp8(every, scale, fmt)
        b, amax_b = F.cast_fp8(every, np.float32(scale), fmt)
        assert np.array_equal(a, b), scale
        assert amax_a == amax_b
    rs = np.random.default_rng(1)
    x = _bf16_patterns(rs, (257, 96), 1.0)
    amax = np.float32(np.max(np.abs(F.bf16_to_f32(x))))
    scale = np.float32(float(amax) / (448.0 if fmt == "e4m3" else 57344.0))
    a, amax_a = N.cast_fp8(x, scale, fmt)
    b, amax_b = F.cast_fp8(x, scale, fmt)
    assert a.shape == x.shape and np.array_equal(a, b) and amax_a == amax_b == amax
    e, amax_e = N.cast_fp8(np.zeros((0, 8), dtype=np.uint16), 1.0, fmt)
    assert e.shape == (0, 8) and amax_e == 0.0


def _edge_groups():
    g = np.array([[1, 1, 1, 1], [10, 1, 1, 1], [3, 1, 1, 1], [0, 0, 0, 0], [0, 0, 7, 0], [7, 0, 0, 0], [0, 0, 0, -7],
                  [2, 0, 2, 0], [-1, 2, -3, 4], [1, -8, 2, 1], [1, 2.0 ** -30, 0, 0], [-0.0, 0, -5, 0],
                  [1e-3, -1e-3, 1e-3, -1e-3], [448, 448, 448, 448], [448, -1, 0.5, 0.25], [3, -3, 1, 0]], dtype=np.float32)
    cols = np.concatenate([g.T, g.T[::-1]], axis=0)               # (8 tokens, 16 channels): each column holds two groups
    return np.tile(cols, (4, 1))                                    # 32 tokens


@pytest.mark.parametrize("dtype", ["bf16", "e4m3", "e5m2"])
def test_mvue_pack_equals_numpy(dtype):
    rs = np.random.default_rng(2)
    enc = {"bf16": F.f32_to_bf16_rne, "e4m3": F.f32_to_e4m3_rne_sat, "e5m2": F.f32_to_e5m2_rne_sat}[dtype]
    cases = [enc(_edge_groups()).reshape(32, 16)]
    g = (rs.standard_normal((264, 40)) * np.exp(rs.uniform(-4, 4, (264, 40)))).astype(np.float32)
    g[rs.random(g.shape) < 0.15] = 0.0
    cases.append(enc(g).reshape(g.shape))
    if dtype != "bf16":                                             # every pair of codes meets somewhere
        codes = rs.integers(0, 256, (512, 24)).astype(np.uint8)
        bad = (codes & 0x7F) == 0x7F if dtype == "e4m3" else (codes & 0x7C) == 0x7C
        codes[bad] = 0
        cases.append(codes)
    for codes in cases:
        for seed, offset, first_token in [(0, 0, 0), (12345678901234567, 99, 0), (3, 1, 4 * ((1 << 32) // 8 - 3)), (7, 7, 1 << 40)]:
            av, am = N.mvue_pack(codes, seed, offset, dtype, first_group=first_token // 4)
            bv, bm = M.mvue_pack(codes, seed, offset, dtype, first_token=first_token)
            assert np.array_equal(am, bm), (dtype, seed)
            assert np.array_equal(av, bv), (dtype, seed)


@pytest.mark.parametrize("dtype", ["bf16", "e4m3", "e5m2"])
def test_decode_packed_equals_numpy(dtype):
    rs = np.random.default_rng(3)
    R, K = 37, 96
    if dtype == "bf16":
        vals = _bf16_patterns(rs, (R, K // 2), 3.0)
    else:
        vals = np.arange(R * (K // 2), dtype=np.int64).reshape(R, K // 2).astype(np.uint8)      # every code appears
        bad = (vals & 0x7F) == 0x7F if dtype == "e4m3" else (vals & 0x7C) == 0x7C
        vals[bad] = 1
    meta = rs.integers(0, 256, (R, K // 8)).astype(np.uint8)       # includes malformed nibbles (equal positions)
    assert np.array_equal(N.decode_packed(vals, meta, dtype), P.decode_packed(vals, meta, dtype))
