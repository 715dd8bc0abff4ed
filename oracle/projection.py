"""2:4 soft-threshold projection S_soft, MSE-optimal scale beta, and the packed 2:4 format.

Test infrastructure only (see the package header).

Math layer (float64) -- the paper's definitions written out:
  * ``soft_threshold``   Sec. 4.1, the displayed definition of S_soft (t = |t_2| of the
                         ascending magnitude order = third-largest magnitude of the group);
  * ``soft_threshold_sorted_form``  the same function as the appendix proof of Theorem 1 writes
                         it for a magnitude-sorted group (used as a cross-check);
  * ``hard_threshold`` / ``hard_threshold_mask``  Sec. 2, Eq. (hard-thresholding);
  * ``beta_mse``         Sec. 4.2, beta = w^T S_soft(w) / ||S_soft(w)||^2;
  * ``beta_l1``          Sec. 4.2, the L1-preserving variant the paper compares with;
  * ``flip_rate``        Sec. 3.3, r_k = ||m(w_k) xor m(w_{k-1})||_1 / d.

Bit-spec layer (float32 + integers) -- the rounding sequence a bf16 / e4m3 packed operand forces:
  * ``project_pack``     S(w) = beta * S_soft(w) on bf16 inputs -> (values, 2-bit metadata, amax);
  * ``decode_packed``    packed (values, metadata) -> dense-with-zeros matrix;
  * ``sgd_step``         Sec. 2, Eq. (7): the dense weight moves by -alpha * gradient of the sparse
                         weight; ``sgd_project_pack`` is that step followed by ``project_pack``;
  * ``kept_positions``   metadata -> the two recorded positions per group.

Readings taken where the paper is silent (all restated in the design notes of the repository):
  * ties: the VALUES of S_soft do not depend on how ties are broken (every element whose
    magnitude equals t maps to 0); only the two RECORDED positions do.  Rule: rank by magnitude
    descending, then index ascending; ranks 0 and 1 are recorded, in ascending index order.
    Magnitude order is the unsigned order of the bf16 pattern with the sign bit cleared.
  * sign of a kept-but-zero value: the literal forms a - t and a + t give +0 at a tie.
  * rounding: sd = a -/+ t in float32, p = sd * beta in float32 (beta a float32 input),
    bf16 path: value = RNE_bf16(p); e4m3 path: q = p / val_scale (float32 division), clamp to
    +-448, value = RNE_e4m3(q).  amax = max |p| over recorded values (float32).

  * the step of Eq. (7): step = alpha * g in float32, w' = w - step in float32 (two roundings, no
    fused multiply-add); a bf16 dense weight stores RNE_bf16(w') and is projected from that; a
    float32 dense weight stores w' and is projected from RNE_bf16(w').

Pinned (tests/test_oracle_projection.py): worked groups, the appendix's sorted form, the 2:4
invariant, idempotence (projection), homogeneity, the 2-delta continuity bound of the Theorem 1
proof, agreement of supports with the hard threshold, optimality of beta,
decode(pack(w)) against the float64 definition, and the blocked device layout
(``to_fragment_major`` / ``from_fragment_major`` / ``k_step``) against an index-by-index
construction from its description, with round trips on ragged row counts.
"""
import numpy as np

from . import formats


# --------------------------------------------------------------------------- math layer

def _groups(a):
    a = np.asarray(a, dtype=np.float64)
    if a.shape[-1] % 4 != 0:
        raise ValueError("last dimension must be a multiple of 4 (the method is defined on whole groups)")
    return a.reshape(-1, 4)


def soft_threshold(a, gamma=0.0):
    """S_soft of Sec. 4.1 applied block-wise along the last axis (float64).

    gamma: the threshold ablation of Sec. 4.1 "Choosing optimal threshold".  Any t in [|t2|, |t3|] is
    feasible; the paper writes the interpolation as gamma |t2| + (1 - gamma) |t3| but describes it the
    other way round (larger gamma -> t closer to |t3|, gamma = 0 -> t = |t2|, which is the method).
    Reading taken: t = (1 - gamma) |t2| + gamma |t3|, the one consistent with the text, the definition
    above it and the table's best row gamma = 0."""
    a = np.asarray(a, dtype=np.float64)
    g = _groups(a)
    mags = np.sort(np.abs(g), axis=1)                # ascending magnitudes |t1|<=|t2|<=..: t = |t2| for gamma = 0
    t = (1.0 - gamma) * mags[:, 1:2] + gamma * mags[:, 2:3]
    out = np.where(g >= t, g - t, np.where(g <= -t, g + t, 0.0))
    # the middle case (-t, t) -> 0 takes precedence only where the intervals do not overlap; for
    # t == 0 the first and third intervals both contain 0 and both give 0, so no ambiguity.
    return out.reshape(a.shape)


def soft_threshold_sorted_form(a):
    """The appendix's way of writing S_soft: after sorting a group by magnitude the result is
    [0, 0, sign(a3)(|a3|-|a2|), sign(a4)(|a4|-|a2|)] put back in place (float64)."""
    a = np.asarray(a, dtype=np.float64)
    g = _groups(a)
    order = np.argsort(np.abs(g), axis=1, kind="stable")
    srt = np.take_along_axis(g, order, axis=1)
    t = np.abs(srt[:, 1])
    res_sorted = np.zeros_like(srt)
    res_sorted[:, 2] = np.sign(srt[:, 2]) * (np.abs(srt[:, 2]) - t)
    res_sorted[:, 3] = np.sign(srt[:, 3]) * (np.abs(srt[:, 3]) - t)
    out = np.zeros_like(g)
    np.put_along_axis(out, order, res_sorted, axis=1)
    return out.reshape(a.shape)


def hard_threshold(a):
    """S_h of Sec. 2: keep a_i where |a_i| >= t, t the 2nd-largest magnitude of the group."""
    a = np.asarray(a, dtype=np.float64)
    g = _groups(a)
    t = np.sort(np.abs(g), axis=1)[:, 2:3]
    return np.where(np.abs(g) >= t, g, 0.0).reshape(a.shape)


def hard_threshold_mask(a):
    """0/1 mask of S_h (support of the kept elements), same shape as ``a``."""
    a = np.asarray(a, dtype=np.float64)
    g = _groups(a)
    t = np.sort(np.abs(g), axis=1)[:, 2:3]
    return (np.abs(g) >= t).reshape(a.shape)


def beta_mse(w, gamma=0.0):
    """Sec. 4.2: argmin_beta ||w - beta S_soft(w)||^2 = <w, S_soft(w)> / ||S_soft(w)||^2 (float64)."""
    w = np.asarray(w, dtype=np.float64)
    s = soft_threshold(w, gamma)
    den = float(np.sum(s * s))
    if den == 0.0:
        raise ValueError("S_soft(w) is identically zero: beta is undefined")
    return float(np.sum(w * s)) / den


def beta_l1(w, gamma=0.0):
    """Sec. 4.2: the L1-norm preserving scale ||w||_1 / ||S_soft(w)||_1 (comparison variant)."""
    w = np.asarray(w, dtype=np.float64)
    s = soft_threshold(w, gamma)
    return float(np.sum(np.abs(w))) / float(np.sum(np.abs(s)))


def flip_rate(mask_now, mask_before):
    """Sec. 3.3: fraction of positions whose 0/1 mask changed between two iterations."""
    a = np.asarray(mask_now, dtype=bool)
    b = np.asarray(mask_before, dtype=bool)
    return float(np.count_nonzero(a ^ b)) / a.size


# --------------------------------------------------------------------------- bit-spec layer

def rank_positions(w_bits):
    """bf16 patterns (..., I) -> (idx0, idx1, third_mag_bits) per group of 4 along the last axis.

    Ranking key: magnitude field (pattern & 0x7FFF) descending, then index ascending.
    idx0 < idx1 are the positions of ranks 0 and 1; third_mag_bits is the magnitude field of rank 2.
    """
    bits = np.asarray(w_bits, dtype=np.uint16)
    mag = (bits & np.uint16(0x7FFF)).astype(np.int64).reshape(-1, 4)
    n = mag.shape[0]
    rank = np.zeros((n, 4), dtype=np.int64)
    for i in range(4):
        for j in range(4):
            if i == j:
                continue
            beats = (mag[:, j] > mag[:, i]) | ((mag[:, j] == mag[:, i]) & (j < i))
            rank[:, i] += beats
    kept = rank < 2
    pos = np.tile(np.arange(4), (n, 1))
    idx0 = np.where(kept, pos, 9).min(axis=1)
    idx1 = np.where(kept, pos, -1).max(axis=1)
    third = np.take_along_axis(mag, np.argmax(rank == 2, axis=1)[:, None], axis=1)[:, 0]
    return idx0, idx1, third.astype(np.uint16)


def second_magnitude_bits(w_bits):
    """Magnitude field of the second-ranked element of each group (same order as ``rank_positions``)."""
    bits = np.asarray(w_bits, dtype=np.uint16)
    mag = (bits & np.uint16(0x7FFF)).reshape(-1, 4)
    return np.sort(mag, axis=1)[:, 2].astype(np.uint16)


def project_pack(w_bits, beta, val_dtype="bf16", val_scale=1.0, gamma=0.0):
    """beta * S_soft(W) on a bf16 matrix, packed 2:4.

    gamma (threshold ablation, see ``soft_threshold``): t = m3 + gamma * (m2 - m3) as three float32
    operations on the third- and second-largest magnitudes; gamma = 0 leaves t = m3 untouched.

    w_bits : uint16 (O, I) bf16 patterns, groups of 4 along I.
    Returns (vals, meta, amax):
      vals : (O, I/2) uint16 bf16 patterns, or uint8 e4m3 codes -- the two recorded values of each
             group in ascending position order;
      meta : (O, I/8) uint8 -- per group a nibble idx0 | idx1 << 2; the even group of a pair sits in
             the low nibble;
      amax : float32 max |p| over the recorded values before the storage rounding.
    """
    w_bits = np.asarray(w_bits, dtype=np.uint16)
    O, I = w_bits.shape
    if I % 8 != 0:
        raise ValueError("I must be a multiple of 8 (two groups per metadata byte)")
    beta32 = np.float32(beta)
    idx0, idx1, third = rank_positions(w_bits)
    a = formats.bf16_to_f32(w_bits).reshape(-1, 4)
    t = formats.bf16_to_f32(third)                                    # >= 0
    if float(gamma) != 0.0:
        m2 = formats.bf16_to_f32(second_magnitude_bits(w_bits))
        span = (m2 - t).astype(np.float32)
        part = (np.float32(gamma) * span).astype(np.float32)
        t = (t + part).astype(np.float32)
    rows = np.arange(a.shape[0])
    out_vals = []
    amax = np.float32(0.0)
    for idx in (idx0, idx1):
        ai = a[rows, idx]
        sd = (ai - np.copysign(t, ai)).astype(np.float32)             # a - t  or  a + t, one float32 op
        with np.errstate(over="ignore"):                              # weights near the bf16 maximum: p = inf, as in float32
            p = (sd * beta32).astype(np.float32)
        if p.size:
            amax = max(amax, np.float32(np.max(np.abs(p))))
        if val_dtype == "bf16":
            if float(val_scale) != 1.0:
                raise ValueError("val_scale must be 1 for bf16 values")
            out_vals.append(formats.f32_to_bf16_rne(p))
        elif val_dtype == "e4m3":
            with np.errstate(over="ignore"):
                q = (p / np.float32(val_scale)).astype(np.float32)
            out_vals.append(formats.f32_to_e4m3_rne_sat(q))
        else:
            raise ValueError("val_dtype must be 'bf16' or 'e4m3'")
    vals = np.stack(out_vals, axis=1).reshape(O, I // 2)
    nib = (idx0 | (idx1 << 2)).astype(np.uint8).reshape(O, I // 8, 2)
    meta = (nib[:, :, 0] | (nib[:, :, 1] << 4)).astype(np.uint8)
    return vals, meta, np.float32(amax)


def sgd_step(w, g, alpha, master="bf16"):
    """Eq. (7): w_{k+1} = w_k - alpha_k * g, with g the gradient taken at the sparse weight.

    w : (O, I) uint16 bf16 patterns (master="bf16") or float32 values (master="f32");
    g : (O, I) float32.  Returns (w_next in the storage of w, bf16 patterns the projection reads).
    """
    g32 = np.asarray(g, dtype=np.float32)
    a32 = np.float32(alpha)
    if master == "bf16":
        w32 = formats.bf16_to_f32(np.asarray(w, dtype=np.uint16))
    elif master == "f32":
        w32 = np.asarray(w, dtype=np.float32)
    else:
        raise ValueError("master must be 'bf16' or 'f32'")
    step = (a32 * g32).astype(np.float32)
    nxt = (w32 - step).astype(np.float32)
    bits = formats.f32_to_bf16_rne(nxt).reshape(nxt.shape)
    return (bits if master == "bf16" else nxt), bits


def sgd_project_pack(w, g, alpha, beta, master="bf16", val_dtype="bf16", val_scale=1.0):
    """One iteration's weight side (Sec. 2, steps 3 then 1): update the dense weight with Eq. (7),
    then S(w) = beta * S_soft(w) of the new weight, packed.  Returns (w_next, vals, meta)."""
    w_next, bits = sgd_step(w, g, alpha, master)
    vals, meta, _ = project_pack(bits, beta, val_dtype, val_scale)
    return w_next, vals, meta


def kept_positions(meta):
    """(O, I/8) metadata bytes -> (idx0, idx1) arrays of shape (O, I/4)."""
    meta = np.asarray(meta, dtype=np.uint8)
    O = meta.shape[0]
    nib = np.stack([meta & 0xF, meta >> 4], axis=2).reshape(O, -1)
    return (nib & 3).astype(np.int64), ((nib >> 2) & 3).astype(np.int64)


def decode_packed(vals, meta, val_dtype="bf16"):
    """Packed (vals, meta) -> dense-with-zeros float64 (O, I) holding the exact stored values."""
    idx0, idx1 = kept_positions(meta)
    O, G = idx0.shape
    v = {"bf16": formats.bf16_to_f32, "e4m3": formats.e4m3_to_f32, "e5m2": formats.e5m2_to_f32}[val_dtype](vals)
    v = v.astype(np.float64).reshape(O, G, 2)
    dense = np.zeros((O, G, 4), dtype=np.float64)
    r, g = np.meshgrid(np.arange(O), np.arange(G), indexing="ij")
    dense[r, g, idx0] = v[:, :, 0]
    # a well-formed group has idx0 != idx1; if they coincide the later write wins, as documented
    dense[r, g, idx1] = v[:, :, 1]
    return dense.reshape(O, G * 4)


# --------------------------------------------------------------------------- device layout

def k_step(val_dtype):
    """Dense columns covered by one sparse matrix instruction step: 64 (bf16) / 128 (e4m3, e5m2)."""
    return 64 if val_dtype == "bf16" else 128


def to_fragment_major(vals, meta, val_dtype="bf16"):
    """Row-major packed (vals (R, K/2), meta (R, K/8)) -> the blocked layout the GPU library stores.

    Pure data movement (no arithmetic).  Rows are padded to a multiple of 16 with the packing of
    all-zero rows (values 0, nibble 0 | 1 << 2: an all-zero group records positions 0 and 1).  With
    KS = k_step(val_dtype), RB = ceil(R/16) row blocks and S = K / KS column steps:
      vals_fm[rb, s, q, j, :]  = the 16 bytes (8 bf16 / 16 e4m3 values) of row 16*rb + j that cover dense
                                 columns [KS*s + KS/4*q, KS*s + KS/4*(q+1));
      meta_fm[rb, s, q, j, :]  = the 2 (bf16) / 4 (e4m3) metadata bytes of the same row and columns.
    Both are returned flattened to 1-D byte-compatible arrays in (rb, s, q, j) order."""
    vals = np.asarray(vals)
    meta = np.asarray(meta, dtype=np.uint8)
    R = vals.shape[0]
    KS = k_step(val_dtype)
    K = vals.shape[1] * 2
    if K % KS != 0:
        raise ValueError("K must be a multiple of the column step")
    S = K // KS
    RB = (R + 15) // 16
    per = KS // 8                       # values per (row, q): 8 or 16
    mper = KS // 32                     # metadata bytes per (row, q): 2 or 4
    vp = np.zeros((RB * 16, K // 2), dtype=vals.dtype)
    vp[:R] = vals
    mp = np.full((RB * 16, K // 8), 0x44, dtype=np.uint8)
    mp[:R] = meta
    v = vp.reshape(RB, 16, S, 4, per).transpose(0, 2, 3, 1, 4)
    m = mp.reshape(RB, 16, S, 4, mper).transpose(0, 2, 3, 1, 4)
    return np.ascontiguousarray(v).reshape(-1), np.ascontiguousarray(m).reshape(-1)


def from_fragment_major(vals_fm, meta_fm, R, K, val_dtype="bf16"):
    """Inverse of ``to_fragment_major``: blocked layout -> row-major (vals (R, K/2), meta (R, K/8))."""
    KS = k_step(val_dtype)
    S = K // KS
    RB = (R + 15) // 16
    per = KS // 8
    mper = KS // 32
    v = np.asarray(vals_fm).reshape(RB, S, 4, 16, per).transpose(0, 3, 1, 2, 4).reshape(RB * 16, K // 2)
    m = np.asarray(meta_fm, dtype=np.uint8).reshape(RB, S, 4, 16, mper).transpose(0, 3, 1, 2, 4).reshape(RB * 16, K // 8)
    return np.ascontiguousarray(v[:R]), np.ascontiguousarray(m[:R])


def structural_mask(meta):
    """(O, I/8) metadata -> boolean (O, I) mask of the recorded positions."""
    idx0, idx1 = kept_positions(meta)
    O, G = idx0.shape
    m = np.zeros((O, G, 4), dtype=bool)
    r, g = np.meshgrid(np.arange(O), np.arange(G), indexing="ij")
    m[r, g, idx0] = True
    m[r, g, idx1] = True
    return m.reshape(O, G * 4)
