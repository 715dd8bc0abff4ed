"""Pins for oracle/mvue.py (the 2:4 minimum-variance unbiased estimator of Sec. 5.1)."""
import os

import numpy as np
import pytest

from oracle import formats as F
from oracle import mvue as M
from oracle import rng as R

GOLD = os.path.join(os.path.dirname(__file__), "golden", "mvue_groups.txt")


def _golden():
    rows = []
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        g, u, th, pos = [np.array(p.split(), dtype=np.float64) for p in line.split("|")]
        rows.append((g, float(u[0]), th, pos.astype(int)))
    return rows


def test_golden_groups_math_and_bitspec():
    for g, u, th, pos in _golden():
        theta, p = M.mvue_sample(g[None, :], np.array([u]))
        assert np.array_equal(theta[0], th), (g, u, theta)
        assert p[0].tolist() == pos.tolist(), (g, u, p)
        # every golden number is exact in bf16, so the bit-spec layer must agree exactly
        codes = F.f32_to_bf16_rne(g.astype(np.float32))[None, :]
        vals, nib = M.mvue_groups_bits(codes, np.array([u], dtype=np.float32))
        assert (int(nib[0]) & 3, int(nib[0]) >> 2) == (pos[0], pos[1])
        got = F.bf16_to_f32(vals[0]).astype(np.float64)
        assert got[0] == th[pos[0]] and got[1] == th[pos[1]]


def test_probabilities_closed_form_cases():
    pi = M.inclusion_probabilities(np.array([[1, 1, 1, 1], [10, 1, 1, 1], [0, 0, 7, 0], [4, 3, 2, 1.0]]))
    assert np.allclose(pi[0], 0.5)
    assert np.allclose(pi[1], [1, 1 / 3, 1 / 3, 1 / 3])
    assert pi[2].tolist() == [0, 0, 1, 0]
    assert np.allclose(pi[3], [0.8, 0.6, 0.4, 0.2])
    g = np.random.default_rng(0).standard_normal((1000, 4))
    pi = M.inclusion_probabilities(g)
    assert np.allclose(pi.sum(axis=1), 2.0) and pi.max() <= 1.0 + 1e-15 and pi.min() >= 0


def test_probabilities_minimise_the_variance():
    """No feasible pi' (sum 2, 0 < pi' <= 1) has lower sum g_i^2 (1/pi'_i - 1)."""
    rng = np.random.default_rng(1)
    g = rng.standard_normal((200, 4)) * np.exp(rng.uniform(-2, 2, (200, 4)))
    best = M.total_variance(g)
    for _ in range(200):
        alt = rng.dirichlet(np.ones(4) * rng.uniform(0.3, 5), size=200) * 2
        ok = alt.max(axis=1) <= 1.0
        var = (g * g * (1.0 / alt - 1.0)).sum(axis=1)
        assert np.all(var[ok] >= best[ok] * (1 - 1e-12))
    # and a local perturbation of the optimum does not improve it
    pi = M.inclusion_probabilities(g)
    for i in range(4):
        for j in range(4):
            if i == j:
                continue
            alt = pi.copy()
            alt[:, i] += 1e-4
            alt[:, j] -= 1e-4
            ok = (alt.max(axis=1) <= 1.0) & (alt.min(axis=1) > 0)
            var = (g * g * (1.0 / alt - 1.0)).sum(axis=1)
            assert np.all(var[ok] >= best[ok] * (1 - 1e-12))


def test_exactly_two_positions_and_at_most_two_nonzeros():
    rng = np.random.default_rng(2)
    g = rng.standard_normal((5000, 4)) * np.exp(rng.uniform(-3, 3, (5000, 4)))
    g[rng.random((5000, 4)) < 0.2] = 0
    u = rng.random(5000)
    theta, pos = M.mvue_sample(g, u)
    assert np.all(pos[:, 0] < pos[:, 1]) and pos.min() >= 0 and pos.max() <= 3
    assert np.all(np.count_nonzero(theta, axis=1) <= 2)
    rows = np.arange(5000)
    off = np.ones_like(theta, dtype=bool)
    off[rows, pos[:, 0]] = False
    off[rows, pos[:, 1]] = False
    assert np.all(theta[off] == 0)
    assert np.all((theta == 0) | (np.sign(theta) == np.sign(g)))


def test_inclusion_frequencies_and_unbiasedness_with_closed_form_variance():
    """Mean over 10^4 draws converges to g with the standard error the closed-form variance predicts."""
    rng = np.random.default_rng(3)
    groups = np.concatenate([rng.standard_normal((20, 4)), rng.standard_normal((20, 4)) * np.array([8, 1, 1, 1]),
                             np.array([[1, 1, 1, 1], [3, 1, 1, 1], [0, 2, 0, -5], [1e-3, 2e-3, -1e-3, 5e-4]])])
    n = 10000
    u = R.uniform24(11, 0, np.arange(n)).astype(np.float64)
    pi = M.inclusion_probabilities(groups)
    var = M.total_variance(groups)
    for k, g in enumerate(groups):
        theta, pos = M.mvue_sample(np.tile(g, (n, 1)), u)
        freq = np.zeros(4)
        for i in range(4):
            freq[i] = np.mean((pos[:, 0] == i) | (pos[:, 1] == i))
        sel = g != 0
        assert np.all(np.abs(freq[sel] - pi[k][sel]) <= 5 * np.sqrt(pi[k][sel] * (1 - pi[k][sel]) / n) + 2e-7), (g, freq, pi[k])
        mean = theta.mean(axis=0)
        per_elem_var = np.where(sel, g * g * (1 / np.where(sel, pi[k], 1) - 1), 0)
        assert np.all(np.abs(mean - g) <= 5 * np.sqrt(per_elem_var / n) + 1e-9 * np.abs(g).max()), (g, mean)
        emp = theta.var(axis=0).sum()
        assert abs(emp - var[k]) <= 0.1 * var[k] + 1e-12


def test_branches_agree_at_the_cap_boundary():
    """At mx == r both formulas give pi_c = 1 and the same values (continuity of the estimator's law)."""
    u = (np.arange(97) + 0.37) / 97         # off the interval edges, where a 1e-9 shift flips the pick
    for g in ([3.0, 1, 1, 1], [1, 4.0, 2, 1], [0.5, 0.25, 0.25, 1.0]):
        g = np.array(g)
        lo = g.copy()
        hi = g.copy()
        c = np.argmax(np.abs(g))
        lo[c] -= 1e-9
        hi[c] += 1e-9
        tl, _ = M.mvue_sample(np.tile(lo, (97, 1)), u)
        th, _ = M.mvue_sample(np.tile(hi, (97, 1)), u)
        assert np.abs(tl - th).max() < 1e-8


def test_already_sparse_equal_magnitude_groups_are_fixed_points():
    u = np.linspace(0, 1, 50, endpoint=False)
    for g in ([2.0, 0, 2, 0], [0, -1.5, 0, 1.5], [7.0, 7, 0, 0], [0, 0, -3.0, -3.0]):
        theta, _ = M.mvue_sample(np.tile(np.array(g), (50, 1)), u)
        assert np.array_equal(theta, np.tile(np.array(g), (50, 1)))
    # a group with a single nonzero is returned unchanged as well
    theta, _ = M.mvue_sample(np.tile(np.array([0, 0, 0, -9.0]), (50, 1)), u)
    assert np.array_equal(theta, np.tile(np.array([0, 0, 0, -9.0]), (50, 1)))


def test_tiny_elements_next_to_a_large_one_keep_the_large_one():
    """float32 sums can absorb tiny magnitudes entirely (r rounds to 0); element c must still be kept."""
    g = np.array([[1.0, 2.0 ** -30, 0, 0], [0, 0, 2.0 ** -40, 1.0]], dtype=np.float32)
    codes = F.f32_to_bf16_rne(g)
    for u in (0.0, 0.5, 0.999):
        vals, nib = M.mvue_groups_bits(codes, np.full(2, u, dtype=np.float32))
        dense = np.zeros((2, 4))
        for k in range(2):
            p0, p1 = int(nib[k]) & 3, int(nib[k]) >> 2
            assert p0 < p1
            dense[k, p0], dense[k, p1] = F.bf16_to_f32(vals[k])
        assert dense[0, 0] == 1.0 and dense[1, 3] == 1.0


def test_bitspec_layer_tracks_math_layer_on_bf16_inputs():
    rng = np.random.default_rng(4)
    codes = F.f32_to_bf16_rne((rng.standard_normal((20000, 4)) * 1e-3).astype(np.float32))
    u = R.uniform24(5, 6, np.arange(20000))
    vals, nib = M.mvue_groups_bits(codes, u)
    g = F.bf16_to_f32(codes).astype(np.float64)
    theta, pos = M.mvue_sample(g, u.astype(np.float64))
    # float32 vs float64 selection can differ only when tau lands within rounding of a boundary
    same = ((nib & 3) == pos[:, 0]) & ((nib >> 2) == pos[:, 1])
    assert same.mean() > 0.9999
    rows = np.arange(20000)[same]
    got0 = F.bf16_to_f32(vals[same, 0]).astype(np.float64)
    want0 = theta[rows, pos[same, 0]]
    assert np.all(np.abs(got0 - want0) <= np.abs(want0) * 2.0 ** -8)


def test_e4m3_bitspec_stores_half_theta():
    rng = np.random.default_rng(5)
    x = (rng.standard_normal((4000, 4)) * 100).astype(np.float32)
    codes = F.f32_to_e4m3_rne_sat(np.clip(x, -448, 448))
    u = R.uniform24(1, 1, np.arange(4000))
    vals, nib = M.mvue_groups_bits(codes, u, "e4m3")
    g = F.e4m3_to_f32(codes).astype(np.float64)
    theta, pos = M.mvue_sample(g, u.astype(np.float64))
    same = ((nib & 3) == pos[:, 0]) & ((nib >> 2) == pos[:, 1])
    assert same.mean() > 0.999
    rows = np.arange(4000)[same]
    for k in range(2):
        got = 2.0 * F.e4m3_to_f32(vals[same, k]).astype(np.float64)
        want = theta[rows, pos[same, k]]
        assert np.all(np.abs(got - want) <= np.maximum(np.abs(want) * 2.0 ** -4, 2.0 ** -9))
    assert np.all(np.abs(F.e4m3_to_f32(vals)) <= 448)


def test_e5m2_bitspec_stores_half_theta_and_is_unbiased():
    """The e5m2 storage (two mantissa bits) follows the float64 estimator to within its own rounding,
    stays finite at the top of the range, and its mean over many draws converges to the stored gradient
    (rounding of h to e5m2 is the only source of bias: below 2^-3 relative)."""
    rng = np.random.default_rng(15)
    x = (rng.standard_normal((4000, 4)) * 12000).astype(np.float32)
    codes = F.f32_to_e5m2_rne_sat(np.clip(x, -57344, 57344))
    codes[0] = [0x7B, 0xFB, 0x7B, 0x7B]                                # four elements at the largest magnitude
    u = R.uniform24(2, 1, np.arange(4000))
    vals, nib = M.mvue_groups_bits(codes, u, "e5m2")
    g = F.e5m2_to_f32(codes).astype(np.float64)
    theta, pos = M.mvue_sample(g, u.astype(np.float64))
    same = ((nib & 3) == pos[:, 0]) & ((nib >> 2) == pos[:, 1])
    assert same.mean() > 0.999
    rows = np.arange(4000)[same]
    for k in range(2):
        got = 2.0 * F.e5m2_to_f32(vals[same, k]).astype(np.float64)
        want = theta[rows, pos[same, k]]
        assert np.all(np.abs(got - want) <= np.maximum(np.abs(want) * 2.0 ** -3, 2.0 ** -16))
    assert np.all(np.isfinite(F.e5m2_to_f32(vals))) and np.all(np.abs(F.e5m2_to_f32(vals)) <= 57344)
    # unbiasedness on one group whose h = (1.5 + 1 + 0.75 + 0.5) / 2 = 1.875 rounds to 2 in e5m2 after halving
    # (0.9375 -> 1.0), and on one whose h is exactly representable
    for grp, tol in (([1.5, -1.0, 0.75, 0.5], 0.08), ([2.0, -1.0, 0.5, 0.5], 0.02)):
        c = F.f32_to_e5m2_rne_sat(np.array([grp], dtype=np.float32))
        n = 40000
        uu = R.uniform24(9, 9, np.arange(n))
        v, nb = M.mvue_groups_bits(np.repeat(c, n, axis=0), uu, "e5m2")
        dense = np.zeros((n, 4))
        r = np.arange(n)
        dense[r, nb & 3] = 2.0 * F.e5m2_to_f32(v[:, 0])
        dense[r, nb >> 2] = 2.0 * F.e5m2_to_f32(v[:, 1])
        assert np.all(np.abs(dense.mean(axis=0) - np.array(grp)) <= tol * np.abs(np.array(grp)) + 0.02)


def test_pack_layout_and_group_ids():
    rng = np.random.default_rng(6)
    T, O = 32, 8
    dy = F.f32_to_bf16_rne((rng.standard_normal((T, O)) * 1e-3).astype(np.float32))
    vals, meta = M.mvue_pack(dy, 3, 9)
    assert vals.shape == (O, T // 2) and meta.shape == (O, T // 8)
    # recompute one group by hand: tokens 8..11 of channel 5 -> gid = 2 * O + 5
    k, o = 2, 5
    u = R.uniform24(3, 9, np.array([k * O + o], dtype=np.uint64))
    v1, n1 = M.mvue_groups_bits(dy[4 * k:4 * k + 4, o][None, :], u)
    assert vals[o, 2 * k:2 * k + 2].tolist() == v1[0].tolist()
    assert (int(meta[o, k // 2]) >> (4 * (k % 2))) & 0xF == int(n1[0])
    with pytest.raises(ValueError):
        M.mvue_pack(dy[:12], 0, 0)


# ------------------------------------------------------------------ the plain definition, draw by draw

def _definition_groups(rs, n):
    """Random groups of every kind the estimator distinguishes: generic, capped, on the cap boundary,
    with zeros, with ties, one huge element beside tiny ones."""
    g = rs.standard_normal((n, 4)) * np.exp(rs.uniform(-3, 3, (n, 1)))
    kind = rs.integers(0, 8, n)
    big = kind == 1                                     # clearly capped
    g[big, rs.integers(0, 4, big.sum())] *= 50.0
    for k, zeros in ((2, 1), (3, 2), (4, 3)):           # one, two, three zeros
        rows = np.flatnonzero(kind == k)
        for z in range(zeros):
            g[rows, (rs.integers(0, 4, rows.size) + z) % 4 if z == 0 else rs.integers(0, 4, rows.size)] = 0.0
    ties = np.flatnonzero(kind == 5)                    # equal magnitudes, mixed signs
    g[ties] = np.sign(g[ties]) * np.abs(g[ties, :1]) * rs.choice([1.0, 1.0, 2.0, 0.5], (ties.size, 4))
    edge = np.flatnonzero(kind == 6)                    # largest == sum of the others, exactly (small integers)
    small = rs.integers(0, 6, (edge.size, 3)).astype(np.float64)
    col = rs.integers(0, 4, edge.size)
    ge = np.zeros((edge.size, 4))
    for n_, (row, c) in enumerate(zip(small, col)):
        others = [i for i in range(4) if i != c]
        ge[n_, others] = row * rs.choice([-1.0, 1.0], 3)
        ge[n_, c] = row.sum()
    g[edge] = ge
    tiny = np.flatnonzero(kind == 7)                    # a huge element next to tiny ones
    g[tiny] *= 1e-12
    g[tiny, rs.integers(0, 4, tiny.size)] = rs.choice([-1.0, 1.0], tiny.size) * 1e6
    return g


def test_branch_free_sequence_equals_the_plain_definition_draw_by_draw():
    """mvue_sample (the branch-free sequence in float64) records the same positions and values as the
    estimator written out from its definition, on >= 1e5 groups of every kind, for draws that do not
    sit on an interval end (there two roundings of the same rule may differ; such draws are rare and
    counted)."""
    rs = np.random.default_rng(20240911)
    n = 120000
    g = _definition_groups(rs, n)
    u = rs.integers(0, 1 << 24, n).astype(np.float64) * 2.0 ** -24        # the 24-bit uniforms the draw produces
    theta_d, pos_d = M.mvue_definition(g, u)
    theta_s, pos_s = M.mvue_sample(g, u)
    clear = M.definition_edge_distance(g, u) > 1e-9
    assert clear.mean() > 0.97
    assert np.array_equal(pos_d[clear], pos_s[clear])
    scale = np.abs(g).sum(axis=1, keepdims=True) + 1e-300
    assert np.max(np.abs(theta_d[clear] - theta_s[clear]) / scale[clear]) < 1e-12
    # on an interval end the two may pick either neighbour, nothing else
    off = ~clear & np.any(pos_d != pos_s, axis=1)
    assert np.all(np.abs(pos_d[off] - pos_s[off]).max(axis=1) <= 1)


def test_plain_definition_on_exact_inputs_including_interval_ends():
    """Small-integer groups and dyadic u: every quantity is exact in both forms, so they must agree
    everywhere, also when u sits exactly on an interval end; the worked groups of the golden file too."""
    vals = np.array([0.0, 1.0, -1.0, 2.0, -2.0, 4.0])
    grid = np.stack(np.meshgrid(vals, vals, vals, vals, indexing="ij"), axis=-1).reshape(-1, 4)
    # keep groups whose probabilities are dyadic: sum of magnitudes (uncapped) or of the three others (capped) a power of two
    m = np.abs(grid)
    s = m.sum(axis=1)
    r = s - m.max(axis=1)
    capped = m.max(axis=1) > r
    denom = np.where(capped, r, s)
    dyadic = (denom > 0) & (np.log2(np.where(denom > 0, denom, 1.0)) % 1 == 0)
    grid = grid[dyadic]
    assert grid.shape[0] > 150
    for u in (0.0, 0.125, 0.25, 0.5, 0.75, 0.875, 1.0 - 2.0 ** -24):
        uu = np.full(grid.shape[0], u)
        theta_d, pos_d = M.mvue_definition(grid, uu)
        theta_s, pos_s = M.mvue_sample(grid, uu)
        assert np.array_equal(pos_d, pos_s), u
        assert np.array_equal(theta_d, theta_s), u
    for g, u, th, pos in _golden():
        theta, p = M.mvue_definition(g[None, :], np.array([u]))
        assert np.array_equal(theta[0], th) and p[0].tolist() == pos.tolist(), (g, u)


def test_bitspec_positions_equal_the_plain_definition_on_stored_patterns():
    """The float32 rounding sequence on bf16 / e4m3 patterns records the positions of the definition
    (evaluated in float64 on the decoded values) wherever the draw is clear of an interval end by more
    than float32 rounding, and its values are the definition's rounded to the storage format."""
    rs = np.random.default_rng(7)
    n = 60000
    g = _definition_groups(rs, n).astype(np.float32)
    codes = F.f32_to_bf16_rne(g)
    gq = F.bf16_to_f32(codes).astype(np.float64)
    u32 = (rs.integers(0, 1 << 24, n).astype(np.float32) * np.float32(2.0 ** -24))
    vals, nib = M.mvue_groups_bits(codes, u32, "bf16")
    theta_d, pos_d = M.mvue_definition(gq, u32.astype(np.float64))
    clear = M.definition_edge_distance(gq, u32.astype(np.float64)) > 1e-5
    assert clear.mean() > 0.95
    assert np.array_equal((nib & 3)[clear], pos_d[clear, 0]) and np.array_equal((nib >> 2)[clear], pos_d[clear, 1])
    rows = np.flatnonzero(clear)
    got = F.bf16_to_f32(vals[rows]).astype(np.float64)
    want = np.stack([theta_d[rows, pos_d[rows, 0]], theta_d[rows, pos_d[rows, 1]]], axis=1)
    assert np.all(np.abs(got - want) <= 2.0 ** -8 * np.abs(want) + 1e-45)          # one bf16 rounding of h


def test_token_shards_draw_what_the_whole_tensor_draws():
    """first_token places a shard of the token axis in the whole batch: its packed operand is the
    corresponding column range of the whole tensor's, and group ids follow (first_token / 4 + k) * O + o."""
    rs = np.random.default_rng(11)
    codes = F.f32_to_bf16_rne(rs.standard_normal((64, 24)).astype(np.float32)).reshape(64, 24)
    wv, wm = M.mvue_pack(codes, 3, 9)
    for cut in (8, 32, 56):
        sv, sm = M.mvue_pack(codes[cut:], 3, 9, first_token=cut)
        assert np.array_equal(sv, wv[:, cut // 2:]) and np.array_equal(sm, wm[:, cut // 8:])
    ids = M.group_ids(16, 24, first_token=4 * 1000)
    assert ids.shape == (4, 24) and int(ids[0, 0]) == 1000 * 24 and int(ids[3, 23]) == 1003 * 24 + 23
    with pytest.raises(ValueError):
        M.group_ids(16, 24, first_token=6)
