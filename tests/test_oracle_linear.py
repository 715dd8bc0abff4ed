"""Pins for oracle/linear.py: the two products of Sec. 5.1 against brute force and their algebra."""
import numpy as np

from oracle import formats as F
from oracle import linear as Lin
from oracle import mvue as M
from oracle import projection as P


def _bf16(rng, shape, std):
    return F.f32_to_bf16_rne((rng.standard_normal(shape) * std).astype(np.float32))


def test_forward_against_triple_loop_and_dense_with_zeros():
    rng = np.random.default_rng(0)
    wb = _bf16(rng, (8, 16), 0.02)
    xb = _bf16(rng, (12, 16), 1.0)
    vals, meta, _ = P.project_pack(wb, 1.5)
    Z = Lin.linear_fwd(xb, vals, meta)
    Wd = P.decode_packed(vals, meta)
    X = F.bf16_to_f32(xb).astype(np.float64)
    assert np.allclose(Z, Lin.linear_fwd_loops(X, Wd), rtol=1e-13, atol=1e-18)
    # a transposed operand or a wrong contraction axis would fail this non-square case
    assert Z.shape == (12, 8)
    # against the float64 definition of S(W) (before bf16 storage rounding of the values)
    exact = X @ (1.5 * P.soft_threshold(F.bf16_to_f32(wb).astype(np.float64))).T
    assert np.abs(Z - exact).max() <= 2.0 ** -8 * np.abs(X).sum(axis=1).max() * np.abs(Wd).max()


def test_forward_scales_and_linearity():
    rng = np.random.default_rng(1)
    wb = _bf16(rng, (8, 32), 0.02)
    vals, meta, _ = P.project_pack(wb, 1.0)
    x1 = F.f32_to_bf16_rne(np.round(rng.standard_normal((4, 32)) * 4).astype(np.float32))
    x2 = F.f32_to_bf16_rne(np.round(rng.standard_normal((4, 32)) * 4).astype(np.float32))
    xs = F.f32_to_bf16_rne(F.bf16_to_f32(x1) + F.bf16_to_f32(x2))      # small integers: exact sum
    Z1, Z2, Zs = (Lin.linear_fwd(x, vals, meta) for x in (x1, x2, xs))
    assert np.allclose(Z1 + Z2, Zs, rtol=1e-13, atol=1e-18)
    assert np.allclose(Lin.linear_fwd(x1, vals, meta, x_scale=0.5, w_scale=4.0), 2.0 * Z1)


def test_forward_e4m3_decodes_codes():
    rng = np.random.default_rng(2)
    wb = _bf16(rng, (8, 16), 0.02)
    vals, meta, amax = P.project_pack(wb, 1.5, "e4m3", np.float32(0.0002))
    x = F.f32_to_e4m3_rne_sat((rng.standard_normal((4, 16)) * 50).astype(np.float32))
    Z = Lin.linear_fwd(x, vals, meta, "e4m3", x_scale=0.02, w_scale=0.0002)
    Wd = P.decode_packed(vals, meta, "e4m3")
    want = Lin.linear_fwd_loops(F.e4m3_to_f32(x).astype(np.float64), Wd) * (np.float64(np.float32(0.02)) * np.float64(np.float32(0.0002)))
    assert np.allclose(Z, want, rtol=1e-13)


def test_wgrad_against_loops_on_the_sparsified_operand():
    rng = np.random.default_rng(3)
    T, O, I = 16, 8, 8
    dy = _bf16(rng, (T, O), 1e-3)
    xb = _bf16(rng, (T, I), 1.0)
    dW = Lin.linear_wgrad(dy, xb, 7, 1)
    theta = Lin.mvue_dense(dy, 7, 1)                       # (T, O)
    X = F.bf16_to_f32(xb).astype(np.float64)
    want = Lin.linear_fwd_loops(theta.T, X.T)              # dW[o][i] = sum_t theta[t][o] X[t][i]
    assert dW.shape == (O, I)
    assert np.allclose(dW, want, rtol=1e-13, atol=1e-20)
    # theta is 2:4 along tokens for every channel
    assert np.all(np.count_nonzero(theta.reshape(T // 4, 4, O), axis=1) <= 2)


def test_wgrad_mean_over_seeds_converges_to_dense_gradient():
    rng = np.random.default_rng(4)
    T, O, I = 32, 8, 8
    dy = _bf16(rng, (T, O), 1e-3)
    xb = _bf16(rng, (T, I), 1.0)
    dense = Lin.linear_wgrad_dense(dy, xb)
    n = 10000
    acc = np.zeros_like(dense)
    acc2 = np.zeros_like(dense)
    for seed in range(n):
        d = Lin.linear_wgrad(dy, xb, seed, 0)
        acc += d
        acc2 += d * d
    mean = acc / n
    sd = np.sqrt(np.maximum(acc2 / n - mean ** 2, 0) / n)
    # unbiased up to the deterministic bf16 rounding of the kept magnitudes (relative 2^-8 per term)
    X = np.abs(F.bf16_to_f32(xb).astype(np.float64))
    G = np.abs(F.bf16_to_f32(dy).astype(np.float64))
    rounding = 2.0 ** -8 * (G.T @ X)
    assert np.all(np.abs(mean - dense) <= 5 * sd + rounding)
    # and the estimate is genuinely noisy for a single seed (it is a sparsifier, not the identity)
    assert np.abs(Lin.linear_wgrad(dy, xb, 0, 0) - dense).max() > 10 * np.abs(mean - dense).max()


def test_wgrad_e4m3_doubles_the_stored_half_theta():
    rng = np.random.default_rng(5)
    T, O, I = 16, 8, 8
    dy = F.f32_to_e4m3_rne_sat((rng.standard_normal((T, O)) * 60).astype(np.float32))
    x = F.f32_to_e4m3_rne_sat((rng.standard_normal((T, I)) * 60).astype(np.float32))
    dW = Lin.linear_wgrad(dy, x, 2, 3, "e4m3", dy_scale=0.5, x_scale=0.25)
    vals, meta = M.mvue_pack(dy, 2, 3, "e4m3")
    half_theta = P.decode_packed(vals, meta, "e4m3").T
    want = (half_theta.T @ F.e4m3_to_f32(x).astype(np.float64)) * 2 * 0.5 * 0.25
    assert np.allclose(dW, want, rtol=1e-13)


def test_dgrad_against_triple_loop_and_shape():
    rng = np.random.default_rng(7)
    wb = _bf16(rng, (8, 16), 0.02)                  # O = 8, I = 16
    dyb = _bf16(rng, (12, 8), 1e-3)                 # T = 12
    vals, meta, _ = P.project_pack(wb, 1.5)
    dX = Lin.linear_dgrad(dyb, vals, meta)
    Wd = P.decode_packed(vals, meta)
    dY = F.bf16_to_f32(dyb).astype(np.float64)
    assert dX.shape == (12, 16)                     # a transposed weight or a wrong contraction axis fails here
    assert np.allclose(dX, Lin.linear_dgrad_loops(dY, Wd), rtol=1e-13, atol=1e-22)
    # a zero in S(W) column i for every channel gives a zero input gradient there: the 2:4 structure shows
    pruned_everywhere = np.all(Wd == 0.0, axis=0)
    assert np.all(dX[:, pruned_everywhere] == 0.0)
    assert np.allclose(Lin.linear_dgrad(dyb, vals, meta, dy_scale=0.25, w_scale=8.0), 2.0 * dX)


def test_dgrad_is_the_adjoint_of_the_forward_product():
    """<dY, X S(W)^T> = <dY S(W), X> for any X, dY: ties the input gradient to the forward oracle."""
    rng = np.random.default_rng(8)
    for dtype, wscale in (("bf16", 1.0), ("e4m3", 0.0002)):
        wb = _bf16(rng, (24, 32), 0.02)
        vals, meta, _ = P.project_pack(wb, 1.4, dtype, np.float32(wscale))
        if dtype == "bf16":
            x, dy = _bf16(rng, (10, 32), 1.0), _bf16(rng, (10, 24), 1e-3)
        else:
            x = F.f32_to_e4m3_rne_sat((rng.standard_normal((10, 32)) * 40).astype(np.float32))
            dy = F.f32_to_e4m3_rne_sat((rng.standard_normal((10, 24)) * 40).astype(np.float32))
        Z = Lin.linear_fwd(x, vals, meta, dtype, x_scale=1.0, w_scale=wscale)
        dX = Lin.linear_dgrad(dy, vals, meta, dtype, dy_scale=1.0, w_scale=wscale)
        lhs = np.sum(Lin.decode_activations(dy, dtype) * Z)
        rhs = np.sum(dX * Lin.decode_activations(x, dtype))
        assert abs(lhs - rhs) <= 1e-12 * max(abs(lhs), abs(rhs))


def test_e5m2_gradients_against_e4m3_operands():
    """Sec. 5.2's backward formats: e5m2 output gradients with e4m3 activations / weights.  The weight
    gradient is the loop product of the decoded half-theta operand, doubled; its mean over seeds
    approaches the dense product; the input gradient equals the loop product on the decoded operands."""
    rng = np.random.default_rng(31)
    T, O, I = 16, 8, 16
    dy = F.f32_to_e5m2_rne_sat((rng.standard_normal((T, O)) * 3000).astype(np.float32))
    x = F.f32_to_e4m3_rne_sat((rng.standard_normal((T, I)) * 60).astype(np.float32))
    dW = Lin.linear_wgrad(dy, x, 2, 3, "e5m2", dy_scale=0.5, x_scale=0.25, x_dtype="e4m3")
    vals, meta = M.mvue_pack(dy, 2, 3, "e5m2")
    half_theta = P.decode_packed(vals, meta, "e5m2")                       # (O, T)
    want = Lin.linear_fwd_loops(F.e4m3_to_f32(x).astype(np.float64).T, half_theta).T * 2 * 0.5 * 0.25
    assert np.allclose(dW, want, rtol=1e-12, atol=0)
    mean = sum(Lin.linear_wgrad(dy, x, s, 0, "e5m2", x_dtype="e4m3") for s in range(3000)) / 3000
    dense = F.e5m2_to_f32(dy).astype(np.float64).T @ F.e4m3_to_f32(x).astype(np.float64)
    assert np.max(np.abs(mean - dense)) <= 0.08 * np.max(np.abs(dense))
    wb = F.f32_to_bf16_rne((rng.standard_normal((O, I)) * 0.02).astype(np.float32)).reshape(O, I)
    wv, wm, _ = P.project_pack(wb, 1.5, "e4m3", np.float32(0.0002))
    dX = Lin.linear_dgrad(dy, wv, wm, "e5m2", dy_scale=0.5, w_scale=0.0002, w_dtype="e4m3")
    want = Lin.linear_dgrad_loops(F.e5m2_to_f32(dy).astype(np.float64), P.decode_packed(wv, wm, "e4m3")) * (0.5 * np.float64(np.float32(0.0002)))
    assert np.allclose(dX, want, rtol=1e-12, atol=0)


# ------------------------------------------------------------------ 8-bit output of the forward product

def _tiny_layer(rs, T=6, O=8, I=16):
    w = F.f32_to_bf16_rne((rs.standard_normal((O, I)) * 0.5).astype(np.float32)).reshape(O, I)
    vals, meta, _ = P.project_pack(w, np.float32(1.25))
    x = F.f32_to_bf16_rne(rs.standard_normal((T, I)).astype(np.float32)).reshape(T, I)
    return x, vals, meta


def test_e4m3_output_is_the_rounded_rescaled_product():
    """decode(codes) * z_scale is the float64 product to within half a step of the e4m3 grid; amax is the
    product's largest magnitude; a scale that is too small saturates at +-448 instead of wrapping."""
    rs = np.random.default_rng(5)
    x, vals, meta = _tiny_layer(rs)
    Z = Lin.linear_fwd(x, vals, meta)
    amax_true = np.max(np.abs(Z))
    z_scale = np.float32(amax_true / 448.0)
    codes, amax = Lin.linear_fwd_e4m3_out(x, vals, meta, z_scale=z_scale)
    assert codes.shape == Z.shape and codes.dtype == np.uint8
    assert abs(float(amax) - amax_true) <= 1e-6 * amax_true
    back = F.e4m3_to_f32(codes).astype(np.float64) * float(z_scale)
    q = np.abs(Z) / float(z_scale)
    step = np.where(q < 2.0 ** -6, 2.0 ** -9, 2.0 ** (np.floor(np.log2(np.maximum(q, 1e-300))) - 3))     # grid spacing at |q|
    assert np.all(np.abs(back - Z) <= (0.5 * step * float(z_scale)) * (1 + 1e-6) + 1e-12)
    assert np.max(F.e4m3_to_f32(codes)) <= 448.0 and np.any(np.abs(F.e4m3_to_f32(codes)) >= 416.0)     # the range is used
    # scale 16 times too small: everything beyond the range clamps, signs are kept
    sat, _ = Lin.linear_fwd_e4m3_out(x, vals, meta, z_scale=np.float32(z_scale / 16.0))
    big = np.abs(Z) >= 448.0 * float(z_scale) / 16.0 * 1.04
    assert np.all((sat[big] & 0x7F) == 0x7E) and np.array_equal(sat[big] >> 7, (Z[big] < 0).astype(np.uint8))


def test_e4m3_output_hand_values_and_ties():
    """A 1 x 1 layer makes the accumulator a single known product: exact codes, ties to even, operand scales."""
    one = F.f32_to_bf16_rne(np.array([[1.0, 0, 0, 0, 0, 0, 0, 0]], dtype=np.float32)).reshape(1, 8)
    vals, meta, _ = P.project_pack(one, np.float32(1.0))              # S_soft keeps the 1 (t = 0): weight row (1, 0, ...)
    assert P.decode_packed(vals, meta)[0, 0] == 1.0

    def code_for(xval, **kw):
        x = F.f32_to_bf16_rne(np.array([[xval, 0, 0, 0, 0, 0, 0, 0]], dtype=np.float32)).reshape(1, 8)
        c, amax = Lin.linear_fwd_e4m3_out(x, vals, meta, **kw)
        return int(c[0, 0]), float(amax)

    assert code_for(1.0) == (0x38, 1.0)                               # 1.0 = exponent field 7, mantissa 0
    assert code_for(-1.5)[0] == 0xBC                                  # sign | 1.5
    assert code_for(1.0625)[0] == 0x38 and code_for(1.1875)[0] == 0x3A   # halfway 1.0|1.125 -> even (1.0); halfway 1.125|1.25 -> even (1.25)
    assert code_for(3.0, z_scale=np.float32(2.0))[0] == 0x3C          # stored 1.5, read back as 1.5 * 2
    assert code_for(3.0, x_scale=np.float32(0.5), w_scale=np.float32(4.0)) == (0x4C, 6.0)    # real value 6 = 1.5 * 2^2
    assert code_for(1000.0)[0] == 0x7E                                # saturates at 448


def test_delayed_scale_window():
    assert F.delayed_scale([], "e4m3") == np.float32(1.0)
    assert F.delayed_scale([0.0, 0.0], "e5m2") == np.float32(1.0)
    assert F.delayed_scale([1.0, 448.0, 3.0], "e4m3") == np.float32(1.0)
    assert F.delayed_scale([2.0, 1.0], "e4m3") == np.float32(np.float32(2.0) / np.float32(448.0))
    assert F.delayed_scale([57344.0 * 3], "e5m2") == np.float32(3.0)


# ------------------------------------------------------------------ feed-forward block

def test_ffn_backward_is_the_gradient_of_the_forward_pass():
    """Numerical differentiation of L = <dY, Y(X, W1, W2)>: central differences in X, W1 and W2 reproduce dX,
    dW1 and dW2 of the chained backward pass (a wrong transpose, a missing activation derivative or a swapped
    operand fails this)."""
    rs = np.random.default_rng(8)
    T, d, h, d2 = 5, 6, 7, 4
    X, W1, W2, dY = rs.standard_normal((T, d)), rs.standard_normal((h, d)), rs.standard_normal((d2, h)), rs.standard_normal((T, d2))
    ref = Lin.ffn_reference(X, W1, W2, dY)

    def loss(X_, W1_, W2_):
        return float(np.sum(dY * Lin.ffn_reference(X_, W1_, W2_, dY)["Y"]))

    eps = 1e-6
    for name, base, grad in (("X", X, ref["dX"]), ("W1", W1, ref["dW1"]), ("W2", W2, ref["dW2"])):
        num = np.zeros_like(base)
        for idx in np.ndindex(base.shape):
            p, m = base.copy(), base.copy()
            p[idx] += eps
            m[idx] -= eps
            args_p = {"X": (p, W1, W2), "W1": (X, p, W2), "W2": (X, W1, p)}[name]
            args_m = {"X": (m, W1, W2), "W1": (X, m, W2), "W2": (X, W1, m)}[name]
            num[idx] = (loss(*args_p) - loss(*args_m)) / (2 * eps)
        assert np.allclose(num, grad, rtol=1e-6, atol=1e-7), name
    # the stages are the single-layer products of this module
    assert np.allclose(ref["H"], X @ W1.T) and np.allclose(ref["dA"], dY @ W2)
