"""Minimum-variance unbiased 2:4 sparsifier for the output gradient (Sec. 5.1 of the paper).

Test infrastructure only (see the package header).

The paper names the estimator (MVUE applied to grad_Z^T in grad_W = MVUE(grad_Z^T) X) and states
its properties -- unbiased, minimum variance, 2:4 -- but gives no formula; it defers to the
work it cites.  The algorithm below is therefore specified from those properties alone:

For a group g in R^4 (four consecutive tokens of one output channel -- the contraction index of
grad_Z^T X is the token index, and hardware 2:4 sparsity lies along the contraction), an
estimator theta with two recorded positions, theta_i = g_i / pi_i when i is recorded (inclusion
probability pi_i, sum pi_i = 2, pi_i <= 1) and 0 otherwise, is unbiased with total variance
sum_i g_i^2 (1/pi_i - 1).  Minimising over pi gives pi_i proportional to |g_i|, capped at 1:

  m_i = |g_i|, mx = max m, c = an index attaining mx, r = sum of the other three.
  capped case (mx > r):   pi_c = 1, pi_i = m_i / r;   theta_c = g_c, theta_i = sign(g_i) r.
  uncapped case:          pi_i = 2 m_i / s, s = sum m; theta_i = sign(g_i) s / 2.

Several joint distributions have these marginals; the one fixed here is systematic sampling
with one uniform u in [0,1) per group, written so that both cases share one branch-free
sequence of steps:

  1. Lo = sum of the three non-maximal magnitudes, taken as (b + d) + mid with
     a = max(m0,m1), b = min(m0,m1), cc = max(m2,m3), d = min(m2,m3), mx = max(a,cc), mid = min(a,cc).
  2. clamp = mx if Lo == 0 else Lo;  l_i = min(m_i, clamp).   (Capped case: the maximum is cut
     down to the total of the others, so its interval is half of the line and is always hit;
     uncapped case and single-nonzero groups: nothing changes.)
  3. Lay l on a line in index order: P0 = l0, P1 = P0 + l1, P2 = P1 + l2, L = P2 + l3; h = L / 2.
  4. tau0 = u * h, tau1 = tau0 + h; the interval holding tau is #{k in {0,1,2} : P_k <= tau}.
     i0 = min(interval(tau0), 2); i1 = min(3, max(interval(tau1), i0 + 1)).  The min / max only act
     when rounding or a degenerate line (zeros) breaks the exact-arithmetic guarantee i0 < i1.
  5. The value recorded at position p is g_p itself when m_p > h (the capped maximum) or m_p == 0
     (a zero dragged in by step 4), else sign(g_p) * h.

In exact arithmetic this gives the marginals above (capped: L = 2 Lo, h = Lo = r; uncapped: l = m,
h = s/2 and every m_i <= h).

Arithmetic order (bit-spec, float32, no fused multiply-add): exactly the operations written in
steps 1-4, each rounded to float32; comparisons are exact.
  bf16 storage: sign(g_p) * h is stored as sign bit | RNE_bf16(h); g_p itself keeps its pattern.
  e4m3 storage: theta can reach twice the largest input, so the stored operand is theta/2
  (sign | RNE_e4m3(0.5*h), or sign | RNE_e4m3(0.5*m_p) where g_p itself is recorded) and the GEMM
  epilogue multiplies by 2.
  e5m2 storage (the backward format of Sec. 5.2): the same with e5m2 codes and RNE_e5m2.

``mvue_definition`` is the same estimator written straight from the definition above (two-case
probabilities, cumulative probabilities on [0, 2), owners of u and u + 1, values g / pi), with no
code in common with the branch-free sequence; ``mvue_sample`` and the bit-spec layer are checked
against it draw by draw.

Pinned (tests/test_oracle_mvue.py): worked groups, the per-draw agreement of the branch-free
sequence with ``mvue_definition`` on random, tied, zero-laden and capped-boundary groups,
exactly-two-positions invariant, empirical
inclusion frequencies against the closed-form pi, Monte-Carlo mean against g with the closed-
form variance, optimality of pi against random feasible alternatives, continuity of the law
at mx == r, groups with one, two or no nonzeros, and a maximum that dwarfs the other elements.
Whether this joint distribution equals the one used by the work the paper cites is unpinned
(that text is not available here); every property the paper itself states is pinned.
"""
import numpy as np

from . import formats
from . import rng as _rng


# --------------------------------------------------------------------------- closed forms

def inclusion_probabilities(g):
    """(n, 4) float64 groups -> (n, 4) optimal inclusion probabilities."""
    m = np.abs(np.asarray(g, dtype=np.float64)).reshape(-1, 4)
    n = m.shape[0]
    rows = np.arange(n)
    mx = m.max(axis=1)
    c = np.argmax(m == mx[:, None], axis=1)
    mo = m.copy()
    mo[rows, c] = 0.0
    r = mo.sum(axis=1)
    s = m.sum(axis=1)
    capped = mx > r
    with np.errstate(divide="ignore", invalid="ignore"):
        pi_unc = np.where(s[:, None] > 0, 2.0 * m / s[:, None], 0.0)
        pi_cap = np.where(r[:, None] > 0, mo / r[:, None], 0.0)
    pi_cap[rows, c] = 1.0
    return np.where(capped[:, None], pi_cap, pi_unc)


def total_variance(g):
    """Closed-form sum_i Var(theta_i) = sum_i g_i^2 (1/pi_i - 1) over elements with g_i != 0."""
    g = np.asarray(g, dtype=np.float64).reshape(-1, 4)
    pi = inclusion_probabilities(g)
    with np.errstate(divide="ignore", invalid="ignore"):
        term = np.where(g != 0, g * g * (1.0 / pi - 1.0), 0.0)
    return term.sum(axis=1)


# --------------------------------------------------------------------------- selection core

def _select(m, u, ft):
    """Steps 1-4 of the module header on magnitudes m (n,4) with uniforms u (n,), all in dtype ft.
    Returns the recorded positions pos0 < pos1 and h."""
    m = np.ascontiguousarray(m, dtype=ft)
    u = np.ascontiguousarray(u, dtype=ft)
    a = np.maximum(m[:, 0], m[:, 1])
    b = np.minimum(m[:, 0], m[:, 1])
    cc = np.maximum(m[:, 2], m[:, 3])
    d = np.minimum(m[:, 2], m[:, 3])
    mx = np.maximum(a, cc)
    mid = np.minimum(a, cc)
    Lo = ((b + d) + mid).astype(ft)
    clamp = np.where(Lo == 0, mx, Lo).astype(ft)
    line = np.minimum(m, clamp[:, None])
    P0 = line[:, 0]
    P1 = (P0 + line[:, 1]).astype(ft)
    P2 = (P1 + line[:, 2]).astype(ft)
    L = (P2 + line[:, 3]).astype(ft)
    h = (ft(0.5) * L).astype(ft)
    tau0 = (u * h).astype(ft)
    tau1 = (tau0 + h).astype(ft)
    i0 = (P0 <= tau0).astype(np.int64) + (P1 <= tau0) + (P2 <= tau0)
    i1 = (P0 <= tau1).astype(np.int64) + (P1 <= tau1) + (P2 <= tau1)
    pos0 = np.minimum(i0, 2)
    pos1 = np.minimum(3, np.maximum(i1, pos0 + 1))
    return pos0, pos1, h


# --------------------------------------------------------------------------- plain definition

def mvue_definition(g, u):
    """The estimator written out from its definition, in float64, one group at a time.

    It shares nothing with ``_select``: no clamped line, no common threshold h.  For each group:
      * the optimal inclusion probabilities in their two-case closed form (capped iff the largest
        magnitude exceeds the sum of the other three; the largest is the lowest index attaining it);
      * the probabilities laid end to end on [0, 2) in index order: element i owns
        [C_{i-1}, C_i) with C_i = pi_0 + ... + pi_i;
      * systematic sampling: the recorded positions are the owners of the points u and u + 1;
      * a recorded element holds g_i / pi_i.
    Groups with fewer than two nonzeros leave the end of [0, 2) unowned (sum pi < 2).  The rule
    there: a point that no interval contains belongs to the last element with pi > 0 (element 3 if
    there is none); the first position is at most 2 and the second lies after the first (the next
    index when both points have the same owner); an element with pi_i = 0 that is recorded this
    way holds g_i = 0 itself.
    Returns dense theta (n, 4) and positions (n, 2); a per-group Python loop, for tests."""
    g = np.asarray(g, dtype=np.float64).reshape(-1, 4)
    u = np.asarray(u, dtype=np.float64).reshape(-1)
    theta = np.zeros_like(g)
    positions = np.zeros((g.shape[0], 2), dtype=np.int64)
    for n in range(g.shape[0]):
        m = [abs(float(x)) for x in g[n]]
        c = m.index(max(m))
        r = sum(m[i] for i in range(4) if i != c)
        if m[c] > r:                                   # capped: the largest element is always kept
            pi = [1.0 if i == c else (m[i] / r if r > 0 else 0.0) for i in range(4)]
        else:                                          # proportional to magnitude, sum = 2
            s = r + m[c]
            pi = [2.0 * m[i] / s if s > 0 else 0.0 for i in range(4)]
        C = [pi[0], pi[0] + pi[1], pi[0] + pi[1] + pi[2], pi[0] + pi[1] + pi[2] + pi[3]]
        owners = [i for i in range(4) if pi[i] > 0]

        def owner(point):
            for i in range(4):
                if point < C[i]:
                    return i
            return owners[-1] if owners else 3

        p0 = min(owner(float(u[n])), 2)
        p1 = min(3, max(owner(float(u[n]) + 1.0), p0 + 1))
        for p in (p0, p1):
            theta[n, p] = g[n, p] / pi[p] if pi[p] > 0 else g[n, p]
        positions[n] = (p0, p1)
    return theta, positions


def definition_edge_distance(g, u):
    """min over the interval ends C_0..C_2 and the two sampling points u, u + 1 of |C_k - point|,
    per group (float64).  Tests use it to tell groups whose draw sits on an interval end -- where
    two correctly rounded evaluations of the same rule may legitimately differ -- from the rest."""
    pi = inclusion_probabilities(g)
    C = np.cumsum(pi, axis=1)[:, :3]
    u = np.asarray(u, dtype=np.float64).reshape(-1, 1)
    return np.minimum(np.abs(C - u), np.abs(C - (u + 1.0))).min(axis=1)


# --------------------------------------------------------------------------- math layer

def mvue_sample(g, u):
    """float64 estimator: groups g (n,4), uniforms u (n,) -> dense theta (n,4) and positions (n,2)."""
    g = np.asarray(g, dtype=np.float64).reshape(-1, 4)
    m = np.abs(g)
    pos0, pos1, h = _select(m, np.asarray(u, dtype=np.float64), np.float64)
    n = g.shape[0]
    rows = np.arange(n)
    theta = np.zeros_like(g)
    for pos in (pos0, pos1):
        gi = g[rows, pos]
        mi = m[rows, pos]
        theta[rows, pos] = np.where((mi > h) | (mi == 0), gi, np.copysign(h, gi))
    return theta, np.stack([pos0, pos1], axis=1)


# --------------------------------------------------------------------------- bit-spec layer

def mvue_groups_bits(g_codes, u, dtype="bf16"):
    """Bit-exact estimator on stored patterns.

    g_codes : (n,4) uint16 bf16 patterns or uint8 e4m3 / e5m2 codes; u : (n,) float32 in [0,1).
    Returns (vals (n,2) patterns in ascending position order, nibble (n,) = pos0 | pos1 << 2).
    For e4m3 and e5m2 the returned codes hold theta/2."""
    if dtype == "bf16":
        g_codes = np.asarray(g_codes, dtype=np.uint16).reshape(-1, 4)
        gf = formats.bf16_to_f32(g_codes)
        sign_mask = np.uint16(0x8000)
    elif dtype in ("e4m3", "e5m2"):
        g_codes = np.asarray(g_codes, dtype=np.uint8).reshape(-1, 4)
        gf = formats.e4m3_to_f32(g_codes) if dtype == "e4m3" else formats.e5m2_to_f32(g_codes)
        encode8 = formats.f32_to_e4m3_rne_sat if dtype == "e4m3" else formats.f32_to_e5m2_rne_sat
        sign_mask = np.uint8(0x80)
    else:
        raise ValueError("dtype must be 'bf16', 'e4m3' or 'e5m2'")
    m = np.abs(gf).astype(np.float32)
    pos0, pos1, h = _select(m, np.asarray(u, dtype=np.float32), np.float32)
    n = m.shape[0]
    rows = np.arange(n)
    if dtype == "bf16":
        hq = formats.f32_to_bf16_rne(h)
    else:
        hq = encode8((np.float32(0.5) * h).astype(np.float32))
    out = []
    for pos in (pos0, pos1):
        code = g_codes[rows, pos]
        mi = m[rows, pos]
        common = ((code & sign_mask) | hq).astype(g_codes.dtype)
        if dtype == "bf16":
            own = code
        else:
            own = (code & sign_mask) | encode8((np.float32(0.5) * mi).astype(np.float32))
        out.append(np.where((mi > h) | (mi == 0), own, common).astype(g_codes.dtype))
    vals = np.stack(out, axis=1)
    nib = (pos0 | (pos1 << 2)).astype(np.uint8)
    return vals, nib


def group_ids(T, O, first_token=0):
    """gid[k, o] = (first_token // 4 + k) * O + o for token group k = t // 4 and output channel o.
    first_token is the global index of the tensor's first token row (a multiple of 4): a shard of
    the token axis draws the numbers the whole tensor would draw for the same tokens."""
    if first_token % 4 != 0:
        raise ValueError("first_token must be a multiple of 4 (whole groups)")
    k = np.arange(T // 4, dtype=np.uint64) + np.uint64(first_token // 4)
    return k[:, None] * np.uint64(O) + np.arange(O, dtype=np.uint64)[None, :]


def mvue_pack(dy_codes, seed, offset, dtype="bf16", first_token=0):
    """MVUE(dY^T) in packed 2:4 form.

    dy_codes : (T, O) stored patterns of the output gradient (bf16 uint16 / e4m3 or e5m2 uint8).
    Returns vals (O, T/2) and meta (O, T/8): row o holds, for token groups k = 0.. in order, the two
    recorded values and the nibble pos0 | pos1 << 2 (even k in the low nibble of byte k // 2)."""
    dy_codes = np.asarray(dy_codes)
    T, O = dy_codes.shape
    if T % 8 != 0:
        raise ValueError("T must be a multiple of 8 (two groups per metadata byte)")
    g = dy_codes.reshape(T // 4, 4, O).transpose(0, 2, 1).reshape(-1, 4)       # [(k, o), 4]
    u = _rng.uniform24(seed, offset, group_ids(T, O, first_token).reshape(-1))
    vals, nib = mvue_groups_bits(g, u, dtype)
    vals = vals.reshape(T // 4, O, 2).transpose(1, 0, 2).reshape(O, T // 2)
    nib = nib.reshape(T // 4, O).T.reshape(O, T // 8, 2)
    meta = (nib[:, :, 0] | (nib[:, :, 1] << 4)).astype(np.uint8)
    return np.ascontiguousarray(vals), np.ascontiguousarray(meta)
