"""Counter-based random numbers for the MVUE sparsifier.

Test infrastructure only (see the package header).

The paper does not say how the estimator of Sec. 5.1 draws its randomness; the only requirement
that follows from using it inside a tiled GEMM is that the draw for a group must be a pure
function of (seed, offset, group id), so that every tile that re-derives a group sees the same
number.  The function specified for this build is:

  key   : (k0, k1) = the low / high 32 bits of mix64(seed xor mix64(offset + GOLDEN64)), where
          mix64 is the 64-bit finalizer z ^= z>>30; z *= 0xBF58476D1CE4E5B9; z ^= z>>27;
          z *= 0x94D049BB133111EB; z ^= z>>31 (SplitMix64's output function);
  draw  : x = (gid mod 2^32) xor k0;  x += (gid >> 32) * 0x9E3779B9;
          x ^= x>>17; x *= 0xED5AD4BB; x += k1; x ^= x>>11; x *= 0xAC4C1B51; x ^= x>>15;
          x *= 0x31848BAB; x ^= x>>14
          (a three-round 32-bit multiply-xorshift integer hash with the second key word injected
          after the first multiply; all arithmetic modulo 2^32.  The three shift / multiplier
          pairs are those of the public-domain "triple32" hash published by C. Wellons' hash-
          prospector search for low-bias 32-bit mixers; the keying around them is this build's.  A two-round hash of this family
          was tried first and rejected: on consecutive counters its top bits failed the
          chi-square test below by ten standard deviations);
  u     : (x >> 8) * 2^-24, an exact float32 in [0, 1).

Pinned (tests/test_oracle_rng.py): frozen key words, draws and uniforms in
tests/golden/rng_known_answers.txt, the published SplitMix64 outputs for seed 1234567 (key
mixer), step-by-step inversion of the draw with the modular inverses of its multipliers,
chi-square uniformity, lag-1 correlation across consecutive group ids, across consecutive seeds
and across consecutive offsets, and bijectivity on a 2^16 window.
"""
import numpy as np

_M64 = (1 << 64) - 1
GOLDEN64 = 0x9E3779B97F4A7C15


def mix64(z):
    z &= _M64
    z ^= z >> 30
    z = (z * 0xBF58476D1CE4E5B9) & _M64
    z ^= z >> 27
    z = (z * 0x94D049BB133111EB) & _M64
    z ^= z >> 31
    return z


def derive_key(seed, offset):
    """(seed, offset) -> (k0, k1), two 32-bit key words (Python ints)."""
    k = mix64((int(seed) & _M64) ^ mix64((int(offset) + GOLDEN64) & _M64))
    return k & 0xFFFFFFFF, k >> 32


def draw_u32(k0, k1, gid):
    """32-bit draw for each group id (array of non-negative integers < 2^64)."""
    gid = np.asarray(gid, dtype=np.uint64)
    m32 = np.uint64(0xFFFFFFFF)
    x = (gid & m32) ^ np.uint64(k0)
    x = (x + (gid >> np.uint64(32)) * np.uint64(0x9E3779B9)) & m32
    x ^= x >> np.uint64(17)
    x = (x * np.uint64(0xED5AD4BB)) & m32
    x = (x + np.uint64(k1)) & m32
    x ^= x >> np.uint64(11)
    x = (x * np.uint64(0xAC4C1B51)) & m32
    x ^= x >> np.uint64(15)
    x = (x * np.uint64(0x31848BAB)) & m32
    x ^= x >> np.uint64(14)
    return x.astype(np.uint32)


def uniform24(seed, offset, gid):
    """float32 uniforms in [0,1) with 24 random bits, one per group id."""
    k0, k1 = derive_key(seed, offset)
    x = draw_u32(k0, k1, gid)
    return (x >> np.uint32(8)).astype(np.float32) * np.float32(2.0 ** -24)
