"""Pins for oracle/projection.py (Sec. 4.1 soft threshold, Sec. 4.2 beta, packed 2:4 format)."""
import os

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle import formats as F
from oracle import projection as P

GOLD = os.path.join(os.path.dirname(__file__), "golden", "soft_threshold_groups.txt")


def _golden():
    rows = []
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        a, s, p = [np.array(part.split(), dtype=np.float64) for part in line.split("|")]
        rows.append((a, s, p.astype(int)))
    return rows


def test_golden_groups_math_layer():
    for a, s, _ in _golden():
        assert np.array_equal(P.soft_threshold(a), s), (a, s)
        assert np.array_equal(P.soft_threshold_sorted_form(a), s), (a, s)


def test_golden_groups_bitspec_positions_and_values():
    for a, s, pos in _golden():
        # all golden numbers are exactly representable in bf16
        wb = F.f32_to_bf16_rne(np.concatenate([a, a]).astype(np.float32)).reshape(1, 8)
        vals, meta, amax = P.project_pack(wb, 1.0)
        nib = int(meta[0, 0]) & 0xF
        assert (nib & 3, nib >> 2) == (pos[0], pos[1]), (a, nib)
        assert int(meta[0, 0]) >> 4 == nib
        got = F.bf16_to_f32(vals[0, :2])
        assert got[0] == s[pos[0]] and got[1] == s[pos[1]]
        assert np.array_equal(P.decode_packed(vals, meta)[0, :4], s)
        assert amax == np.float32(np.max(np.abs(s)))


def test_north_star_example_and_its_beta():
    a = np.array([1, -3, 0.5, 2.0])
    assert P.soft_threshold(a).tolist() == [0, -2, 0, 1]
    # beta = <w, S> / |S|^2 = (6 + 2) / (4 + 1)
    assert P.beta_mse(a) == pytest.approx(1.6, rel=0, abs=1e-15)
    # L1 variant: (1+3+.5+2)/(2+1)
    assert P.beta_l1(a) == pytest.approx(6.5 / 3)


def test_kept_but_zero_value_is_plus_zero_and_negative_zero_inputs():
    wb = F.f32_to_bf16_rne(np.array([[-3, -1, -1, 0, -0.0, 0, -0.0, 0]], dtype=np.float32))
    vals, meta, _ = P.project_pack(wb, 1.5)
    assert vals[0].tolist() == [F.f32_to_bf16_rne(np.array([-3.0], dtype=np.float32))[0], 0x0000, 0x0000, 0x0000]
    assert meta[0, 0] == (0 | (1 << 2)) | ((0 | (1 << 2)) << 4)


@settings(max_examples=300, deadline=None)
@given(st.lists(st.floats(-8, 8, allow_nan=False, width=32), min_size=4, max_size=4))
def test_invariants_on_single_groups(vals):
    a = np.array(vals, dtype=np.float64)
    s = P.soft_threshold(a)
    assert np.count_nonzero(s) <= 2                                   # result lies in the 2:4 set
    assert np.all(np.abs(s) <= np.abs(a) + 0.0)                       # shrinkage
    assert np.all((s == 0) | (np.sign(s) == np.sign(a)))              # sign preserved
    assert np.allclose(P.soft_threshold(s), s, rtol=0, atol=0)        # projection: idempotent
    assert np.allclose(P.soft_threshold_sorted_form(a), s, rtol=0, atol=0)
    c = 1.75
    assert np.allclose(P.soft_threshold(c * a), c * s, rtol=1e-15, atol=0)   # positive homogeneity
    assert np.allclose(P.soft_threshold(-a), -s, rtol=0, atol=0)             # odd
    # permutation equivariance
    perm = np.array([2, 0, 3, 1])
    assert np.array_equal(P.soft_threshold(a[perm]), s[perm])


@settings(max_examples=300, deadline=None)
@given(st.lists(st.floats(-4, 4, allow_nan=False, width=32), min_size=4, max_size=4),
       st.lists(st.floats(-1, 1, allow_nan=False, width=32), min_size=4, max_size=4),
       st.floats(1e-6, 0.5))
def test_continuity_bound_of_theorem_1(vals, direction, delta):
    """The proof of Theorem 1 bounds each output coordinate's change by 2*delta when every input
    coordinate moves by at most delta."""
    a = np.array(vals, dtype=np.float64)
    e = np.array(direction, dtype=np.float64) * delta
    d = np.abs(P.soft_threshold(a + e) - P.soft_threshold(a)).max()
    assert d <= 2 * np.abs(e).max() + 1e-12


def test_continuity_across_the_flip_boundary():
    """At |a2| = |a3| (the flip boundary in the proof's case 2) three outputs are zero and the
    function has no jump, unlike the hard threshold."""
    base = np.array([0.1, 1.0, -1.0, 3.0])
    for eps in (1e-3, 1e-6, 1e-9):
        lo = P.soft_threshold(base + np.array([0, eps, 0, 0]))
        hi = P.soft_threshold(base + np.array([0, 0, -eps, 0]))
        mid = P.soft_threshold(base)
        assert np.count_nonzero(mid) == 1
        assert np.abs(lo - mid).max() <= 2 * eps and np.abs(hi - mid).max() <= 2 * eps
        # the hard threshold jumps by ~1 between the two sides
        assert np.abs(P.hard_threshold(base + np.array([0, eps, 0, 0])) - P.hard_threshold(base + np.array([0, 0, -eps, 0]))).max() > 0.9


def test_support_matches_hard_threshold_without_ties():
    rng = np.random.default_rng(3)
    w = rng.standard_normal((64, 256))
    assert np.array_equal(P.soft_threshold(w) != 0, P.hard_threshold_mask(w))
    # with ties the soft support is a subset
    w2 = np.round(rng.standard_normal((64, 256)) * 2)
    assert np.all((P.soft_threshold(w2) != 0) <= P.hard_threshold_mask(w2))


def test_beta_minimises_the_mse_and_gaussian_value():
    rng = np.random.default_rng(4)
    w = rng.standard_normal((256, 1024)) * 0.02
    b = P.beta_mse(w)
    s = P.soft_threshold(w)
    mse = lambda beta: np.sum((w - beta * s) ** 2)
    assert mse(b) < mse(b * 1.001) and mse(b) < mse(b * 0.999)
    # derivative of the quadratic vanishes at b
    assert abs(np.sum((w - b * s) * s)) < 1e-9 * np.sum(s * s)
    # for i.i.d. Gaussian groups the optimum is scale invariant; Monte-Carlo value ~1.48
    assert 1.45 < b < 1.52
    assert P.beta_mse(3.0 * w) == pytest.approx(b, rel=1e-12)
    with pytest.raises(ValueError):
        P.beta_mse(np.ones((2, 8)))


def test_flip_rate_definition():
    a = np.array([1, 1, 0, 0, 1, 0, 1, 0], dtype=bool)
    b = np.array([1, 0, 1, 0, 1, 0, 1, 0], dtype=bool)
    assert P.flip_rate(a, b) == 2 / 8


def _random_bf16(rng, shape, std=0.02):
    return F.f32_to_bf16_rne((rng.standard_normal(shape) * std).astype(np.float32))


@pytest.mark.parametrize("beta", [1.0, 1.4830322265625, 0.73])
def test_pack_decode_equals_rounded_definition_bf16(beta):
    rng = np.random.default_rng(5)
    wb = _random_bf16(rng, (48, 512))
    vals, meta, amax = P.project_pack(wb, beta)
    dense = P.decode_packed(vals, meta)
    w = F.bf16_to_f32(wb).astype(np.float64)
    exact = np.float64(np.float32(beta)) * P.soft_threshold(w)
    # the stored value is the bf16 rounding of the float64 definition up to one double rounding:
    # relative error <= 2^-8 (half an ulp of the 8-bit significand, relative to the binade base) + 2^-23
    err = np.abs(dense - exact)
    assert np.all(err <= np.abs(exact) * (2.0 ** -8 + 2.0 ** -23) + 1e-45)
    # and on almost all elements it IS the RNE rounding of the exact value
    rne = F.bf16_to_f32(F.f32_to_bf16_rne(exact.astype(np.float32))).astype(np.float64)
    assert np.mean(rne == dense) > 0.999
    # structure
    idx0, idx1 = P.kept_positions(meta)
    assert np.all(idx0 < idx1)
    assert np.array_equal(P.structural_mask(meta).reshape(48, -1, 4).sum(axis=2), np.full((48, 128), 2))
    assert np.all((dense != 0) <= P.structural_mask(meta))
    assert amax == np.float32(np.abs(exact).max()) or abs(float(amax) - np.abs(exact).max()) <= 2.0 ** -23 * np.abs(exact).max()


def test_pack_e4m3_against_definition():
    rng = np.random.default_rng(6)
    wb = _random_bf16(rng, (32, 256))
    w = F.bf16_to_f32(wb).astype(np.float64)
    beta = 1.48
    exact = np.float64(np.float32(beta)) * P.soft_threshold(w)
    scale = np.float32(np.abs(exact).max() / 448.0)
    vals, meta, amax = P.project_pack(wb, beta, "e4m3", scale)
    assert vals.dtype == np.uint8 and vals.shape == (32, 128)
    dense = P.decode_packed(vals, meta, "e4m3") * np.float64(scale)
    # e4m3 half-ulp is 2^-4 relative for normals; absolute 2^-10 * scale for subnormals
    tol = np.maximum(np.abs(exact) * (2.0 ** -4 + 2.0 ** -20), np.float64(scale) * 2.0 ** -10 * 1.001)
    assert np.all(np.abs(dense - exact) <= tol)
    assert np.max(np.abs(P.decode_packed(vals, meta, "e4m3"))) <= 448.0
    # same positions as the bf16 packing: the selection does not depend on the value type
    _, meta16, _ = P.project_pack(wb, beta)
    assert np.array_equal(meta, meta16)
    with pytest.raises(ValueError):
        P.project_pack(wb, beta, "bf16", 2.0)


def test_tie_break_rule_exhaustive_small_alphabet():
    """All 3^4 groups over magnitudes {0,1,2} with mixed signs: recorded positions follow
    (magnitude desc, index asc) computed here by an explicit sort."""
    import itertools
    for combo in itertools.product([0.0, 1.0, -1.0, 2.0, -2.0], repeat=4):
        a = np.array(combo, dtype=np.float32)
        order = sorted(range(4), key=lambda i: (-abs(a[i]), i))
        want = sorted(order[:2])
        wb = F.f32_to_bf16_rne(np.concatenate([a, a])).reshape(1, 8)
        _, meta, _ = P.project_pack(wb, 1.0)
        nib = int(meta[0, 0]) & 0xF
        assert [nib & 3, nib >> 2] == want, (combo, nib)


def test_sgd_step_hand_values_and_library_cast():
    """Eq. (7) with the stated rounding sequence: hand-worked bf16 ties, alpha = 0, and PyTorch's
    CPU float32 arithmetic + bfloat16 cast as an independent implementation."""
    import torch
    one = np.array([[0x3F80]], dtype=np.uint16)                       # 1.0
    # 1 - 2^-9 lies midway between the bf16 neighbours 1 - 2^-8 and 1: ties-to-even gives 1.0
    nxt, bits = P.sgd_step(one, np.array([[1.0]], np.float32), 2.0 ** -9)
    assert nxt[0, 0] == 0x3F80 and bits[0, 0] == 0x3F80
    # 1 - 2^-8 is a bf16 number (0x3F7F)
    nxt, _ = P.sgd_step(one, np.array([[1.0]], np.float32), 2.0 ** -8)
    assert nxt[0, 0] == 0x3F7F
    # sign: a positive gradient lowers the weight, a negative one raises it (1 + 2^-7 = 0x3F81)
    nxt, _ = P.sgd_step(one, np.array([[-1.0]], np.float32), 2.0 ** -7)
    assert nxt[0, 0] == 0x3F81
    # a float32 dense weight keeps the unrounded step; the projection sees the rounded one
    nxt, bits = P.sgd_step(np.array([[1.0]], np.float32), np.array([[1.0]], np.float32), 2.0 ** -9, master="f32")
    assert nxt.dtype == np.float32 and nxt[0, 0] == np.float32(1.0 - 2.0 ** -9) and bits[0, 0] == 0x3F80
    rng = np.random.default_rng(5)
    w = rng.normal(0, 0.02, (16, 64)).astype(np.float32)
    wb = F.f32_to_bf16_rne(w).reshape(w.shape)
    g = rng.normal(0, 1e-3, (16, 64)).astype(np.float32)
    same, _ = P.sgd_step(wb, g, 0.0)
    assert np.array_equal(same, wb)
    for alpha in (1e-2, 0.37, 3.0):
        nxt, bits = P.sgd_step(wb, g, alpha)
        tw = torch.from_numpy(wb.view(np.int16)).view(torch.bfloat16)
        ref = (tw.float() - torch.tensor(alpha, dtype=torch.float32) * torch.from_numpy(g)).to(torch.bfloat16)
        assert np.array_equal(nxt, ref.view(torch.int16).numpy().view(np.uint16))
        nf, bf = P.sgd_step(w, g, alpha, master="f32")
        reff = torch.from_numpy(w) - torch.tensor(alpha, dtype=torch.float32) * torch.from_numpy(g)
        assert np.array_equal(nf, reff.numpy())
        assert np.array_equal(bf, reff.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))


def test_sgd_project_pack_is_step_then_projection_of_the_definition():
    """The fused call equals the float64 definition applied to the stepped weight: decode(pack) is
    RNE_bf16(beta * S_soft(w')) with w' the stored next weight."""
    rng = np.random.default_rng(6)
    w = F.f32_to_bf16_rne(rng.normal(0, 0.02, (8, 64)).astype(np.float32)).reshape(8, 64)
    g = rng.normal(0, 1e-2, (8, 64)).astype(np.float32)
    w_next, vals, meta = P.sgd_project_pack(w, g, 0.5, 1.25)
    assert not np.array_equal(w_next, w)
    dense = P.decode_packed(vals, meta)
    want = 1.25 * P.soft_threshold(F.bf16_to_f32(w_next).astype(np.float64))
    got = dense.astype(np.float64)
    assert np.all(np.abs(got - want) <= np.abs(want) * 2.0 ** -8 + 1e-30)
    assert np.array_equal(got != 0, want != 0)


# ------------------------------------------------------------------ the blocked device layout (pure data movement)

def _fragment_major_by_hand(vals, meta, KS):
    """The blocked layout written with explicit indices from its description: block (rb, s) of 16 rows x
    one column step; in a block, slot 16 q + j holds row 16 rb + j, dense columns [KS s + KS/4 q, KS s +
    KS/4 (q + 1)): KS/8 recorded values and KS/32 metadata bytes (two groups per byte); blocks follow each
    other in (rb, s) order; rows past R are all-zero rows (values 0, nibbles 0 | 1 << 2)."""
    R, half = vals.shape
    K = 2 * half
    S, RB = K // KS, (R + 15) // 16
    per, mper = KS // 8, KS // 32
    out_v = np.zeros(RB * S * 64 * per, dtype=vals.dtype)
    out_m = np.zeros(RB * S * 64 * mper, dtype=np.uint8)
    for rb in range(RB):
        for s in range(S):
            for q in range(4):
                for j in range(16):
                    slot = (rb * S + s) * 64 + 16 * q + j
                    row = 16 * rb + j
                    col0 = KS * s + KS // 4 * q                     # first dense column of the slot
                    for e in range(per):
                        out_v[slot * per + e] = vals[row, col0 // 2 + e] if row < R else 0
                    for e in range(mper):
                        out_m[slot * mper + e] = meta[row, col0 // 8 + e] if row < R else 0x44
    return out_v, out_m


@pytest.mark.parametrize("val_dtype,R,K", [("bf16", 37, 192), ("bf16", 16, 64), ("e4m3", 20, 256), ("e5m2", 3, 128)])
def test_fragment_major_layout_by_hand_and_round_trip(val_dtype, R, K):
    rs = np.random.default_rng(R * 1000 + K)
    KS = P.k_step(val_dtype)
    assert KS == (64 if val_dtype == "bf16" else 128)
    if val_dtype == "bf16":
        vals = rs.integers(0, 1 << 16, (R, K // 2)).astype(np.uint16)
    else:
        vals = rs.integers(0, 256, (R, K // 2)).astype(np.uint8)
    meta = rs.integers(0, 256, (R, K // 8)).astype(np.uint8)
    fv, fm = P.to_fragment_major(vals, meta, val_dtype)
    hv, hm = _fragment_major_by_hand(vals, meta, KS)
    assert fv.dtype == vals.dtype and np.array_equal(fv, hv)
    assert np.array_equal(fm, hm)
    rv, rm = P.from_fragment_major(fv, fm, R, K, val_dtype)
    assert np.array_equal(rv, vals) and np.array_equal(rm, meta)
    # one slot spelled out: block (rb = 0, s = last), q = 2, j = 5 holds row 5, dense columns KS (S - 1) + KS / 2 ...
    if R > 5:
        S = K // KS
        per = KS // 8
        slot = (0 * S + (S - 1)) * 64 + 16 * 2 + 5
        first_col = KS * (S - 1) + KS // 2
        assert np.array_equal(fv[slot * per:(slot + 1) * per], vals[5, first_col // 2:first_col // 2 + per])


# ------------------------------------------------------------------ threshold interpolation and the L1 scale (ablations)

def test_threshold_interpolation_hand_values_and_monotone_norm():
    """Sec. 4.1 'Choosing optimal threshold': gamma = 0 is the method (t = third-largest magnitude), gamma = 1
    puts t on the second-largest magnitude (one survivor per group), and the norm of S_soft shrinks as gamma
    grows -- the statement that fixes which way the paper's interpolation runs."""
    g = np.array([1.0, -3.0, 0.5, 2.0])
    assert P.soft_threshold(g, 0.0).tolist() == [0.0, -2.0, 0.0, 1.0]
    assert P.soft_threshold(g, 0.5).tolist() == [0.0, -1.5, 0.0, 0.5]
    assert P.soft_threshold(g, 1.0).tolist() == [0.0, -1.0, 0.0, 0.0]
    w = np.random.default_rng(4).standard_normal((64, 32))
    norms = [np.linalg.norm(P.soft_threshold(w, gm)) for gm in (0.0, 0.33, 0.67, 1.0)]
    assert all(a > b for a, b in zip(norms, norms[1:]))
    for gm in (0.33, 1.0):                              # still 2:4, still continuous (Theorem 1's bound holds for any feasible t)
        s = P.soft_threshold(w, gm)
        assert np.count_nonzero(s.reshape(-1, 4), axis=1).max() <= 2
        e = np.random.default_rng(5).uniform(-1e-3, 1e-3, w.shape)
        assert np.abs(P.soft_threshold(w + e, gm) - s).max() <= 2 * np.abs(e).max() * (1 + 1e-9)


@pytest.mark.parametrize("gamma", [0.33, 0.67, 1.0])
def test_pack_with_threshold_interpolation_equals_rounded_definition(gamma):
    rs = np.random.default_rng(6)
    w = F.f32_to_bf16_rne((rs.standard_normal((32, 64)) * 0.02).astype(np.float32)).reshape(32, 64)
    beta = np.float32(1.3)
    vals, meta, _ = P.project_pack(w, beta, gamma=gamma)
    v0, m0, _ = P.project_pack(w, beta)
    assert np.array_equal(meta, m0)                     # the recorded positions do not depend on gamma
    dense = P.decode_packed(vals, meta)
    want = float(beta) * P.soft_threshold(F.bf16_to_f32(w).astype(np.float64), float(np.float32(gamma)))
    assert np.all(np.abs(dense - want) <= np.abs(want) * 2.0 ** -8 + 1e-9)          # float32 steps, then one bf16 rounding
    assert np.array_equal(P.project_pack(w, beta, gamma=0.0)[0], v0)


def test_l1_scale_hand_value_and_definition():
    g = np.array([[1.0, -3.0, 0.5, 2.0]])
    assert abs(P.beta_l1(g) - 6.5 / 3.0) < 1e-15        # ||w||_1 = 6.5, ||S_soft(w)||_1 = 3
    assert abs(P.beta_l1(g, 1.0) - 6.5 / 1.0) < 1e-15
    w = np.random.default_rng(7).standard_normal((128, 64))
    b = P.beta_l1(w)
    assert abs(np.abs(b * P.soft_threshold(w)).sum() - np.abs(w).sum()) < 1e-9 * np.abs(w).sum()
    assert 2.3 < b < 2.7 and b > P.beta_mse(w)          # i.i.d. Gaussian weights: about 2.5 against 1.48
