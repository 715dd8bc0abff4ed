"""Storage formats used by the bit-spec layer: bfloat16, OCP FP8 e4m3fn and OCP FP8 e5m2 (Sec. 5.2
of the paper uses per-tensor scaled FP8, e5m2 in the backward pass; the workload fixes e4m3 for
weights, activations, gradients -- e5m2 output gradients are the paper's own recipe).

Test infrastructure only (see the package header).  Pinned: every function here is checked in
``tests/test_oracle_formats.py`` against the format definitions (exhaustive decode tables,
round-trips, hand-computed ties) and against PyTorch's CPU casts, which are an independent
implementation of the same IEEE-style round-to-nearest-even conversions.
"""
import numpy as np

E4M3_MAX = 448.0  # largest finite e4m3fn magnitude: 2^8 * 1.75
E5M2_MAX = 57344.0  # largest finite e5m2 magnitude: 2^15 * 1.75


def bf16_to_f32(bits):
    """uint16 bfloat16 patterns -> float32 values (exact: bf16 is the top half of a float32)."""
    bits = np.asarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_bf16_rne(x):
    """float32 -> bfloat16 patterns (uint16), round to nearest, ties to even.  NaN not handled."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    r = (u + np.uint64(0x7FFF) + lsb) >> np.uint64(16)
    return r.astype(np.uint16)


def e4m3_to_f32(codes):
    """uint8 e4m3fn codes -> float32.  1 sign, 4 exponent (bias 7), 3 mantissa bits; exponent 0 is
    subnormal (m * 2^-9); there is no infinity; S.1111.111 is NaN.  The definition is evaluated on the
    256 codes once and then indexed (same values, far fewer transcendental calls on large tensors)."""
    global _E4M3_TABLE
    if _E4M3_TABLE is None:
        _E4M3_TABLE = _e4m3_decode_definition(np.arange(256, dtype=np.uint8))
    return _E4M3_TABLE[np.asarray(codes, dtype=np.uint8)]


_E4M3_TABLE = None
_E5M2_TABLE = None


def _e4m3_decode_definition(codes):
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    s = (c >> 7) & 1
    e = (c >> 3) & 15
    m = c & 7
    mag = np.where(e == 0, m * 2.0 ** -9, (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64)))
    mag = np.where((e == 15) & (m == 7), np.nan, mag)
    return np.where(s == 1, -mag, mag).astype(np.float32)


def f32_to_e4m3_rne_sat(x):
    """float32 -> e4m3fn codes (uint8): clamp to +-448, then round to nearest, ties to even;
    subnormals are kept (no flush); the sign of zero is kept."""
    x = np.asarray(x, dtype=np.float32)
    neg = np.signbit(x)
    a = np.minimum(np.abs(x).astype(np.float64), E4M3_MAX)
    # exponent of the binade that holds a (clamped below at the subnormal binade 2^-6), from frexp (exact)
    mant, ex = np.frexp(a)            # a = mant * 2^ex, mant in [0.5, 1)
    e = np.clip(np.where(a > 0, ex - 1, -6), -6, 8).astype(np.int64)
    step = np.ldexp(1.0, e - 3)                      # spacing of representable values in that binade
    q = np.rint(a / step)                            # half-to-even, exact scaling by a power of two
    # q is in [0, 16]; q == 16 carries into the next binade
    carry = q >= 16
    e = np.where(carry, e + 1, e)
    q = np.where(carry, 8, q).astype(np.int64)
    sub = q < 8                                      # below the smallest normal of binade -6
    code = np.where(sub, q, ((e + 7) << 3) | (q - 8))
    code = code | (neg.astype(np.int64) << 7)
    return code.astype(np.uint8)


def e5m2_to_f32(codes):
    """uint8 e5m2 codes -> float32.  1 sign, 5 exponent (bias 15), 2 mantissa bits: the top byte of an
    IEEE half.  Exponent 0 is subnormal (m * 2^-16); exponent 31 is infinity (m = 0) or NaN.  Evaluated
    on the 256 codes once, then indexed."""
    global _E5M2_TABLE
    if _E5M2_TABLE is None:
        _E5M2_TABLE = _e5m2_decode_definition(np.arange(256, dtype=np.uint8))
    return _E5M2_TABLE[np.asarray(codes, dtype=np.uint8)]


def _e5m2_decode_definition(codes):
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    s = (c >> 7) & 1
    e = (c >> 2) & 31
    m = c & 3
    mag = np.where(e == 0, m * 2.0 ** -16, (1.0 + m / 4.0) * np.exp2((e - 15).astype(np.float64)))
    mag = np.where(e == 31, np.where(m == 0, np.inf, np.nan), mag)
    return np.where(s == 1, -mag, mag).astype(np.float32)


def f32_to_e5m2_rne_sat(x):
    """float32 -> e5m2 codes (uint8): clamp to +-57344, then round to nearest, ties to even;
    subnormals are kept; the sign of zero is kept.  Never produces infinity or NaN."""
    x = np.asarray(x, dtype=np.float32)
    neg = np.signbit(x)
    a = np.minimum(np.abs(x).astype(np.float64), E5M2_MAX)
    mant, ex = np.frexp(a)                           # a = mant * 2^ex, mant in [0.5, 1)
    e = np.clip(np.where(a > 0, ex - 1, -14), -14, 15).astype(np.int64)
    step = np.ldexp(1.0, e - 2)                      # spacing of representable values in that binade
    q = np.rint(a / step)                            # half-to-even; q in [0, 8]
    carry = q >= 8
    e = np.where(carry, e + 1, e)
    q = np.where(carry, 4, q).astype(np.int64)
    sub = q < 4                                      # below the smallest normal 2^-14
    code = np.where(sub, q, ((e + 15) << 2) | (q - 4))
    code = code | (neg.astype(np.int64) << 7)
    return code.astype(np.uint8)


def cast_fp8(x_bits, scale, fmt="e4m3"):
    """Per-tensor rescaling and cast of a bf16 tensor to an 8-bit format (Sec. 5.2: the operands are
    rescaled per tensor before they are cast).  q = x / scale as ONE float32 division, clamped to the
    format's largest finite value, rounded to nearest even.  Returns (codes uint8, amax float32) with
    amax = max |x| over the tensor (exact: the inputs are bf16), from which a caller derives the next
    scale (amax / format maximum)."""
    x = bf16_to_f32(x_bits)
    with np.errstate(over="ignore"):                 # a scale far too small: infinity, then the clamp
        q = (x / np.float32(scale)).astype(np.float32)
    codes = f32_to_e4m3_rne_sat(q) if fmt == "e4m3" else f32_to_e5m2_rne_sat(q)
    amax = np.float32(np.max(np.abs(x))) if x.size else np.float32(0.0)
    return codes.reshape(x.shape), amax


def delayed_scale(amax_window, fmt="e4m3"):
    """Delayed scaling (the per-tensor recipe Sec. 5.2 refers to): the scale of an 8-bit tensor from the
    largest magnitudes of earlier iterations -- max(window) / format maximum in float32, 1 while the
    window holds only zeros."""
    fmax = np.float32(E4M3_MAX if fmt == "e4m3" else E5M2_MAX)
    m = np.float32(max([np.float32(a) for a in amax_window], default=np.float32(0.0)))
    return np.float32(m / fmax) if m > 0 else np.float32(1.0)
