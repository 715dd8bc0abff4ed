"""The sparse linear layer of Sec. 5.1: Z = X S(W)^T, grad_W = MVUE(grad_Z^T) X and grad_X = grad_Z S(W).

Test infrastructure only (see the package header).  Both products are the plain definitions,
evaluated in float64 on exactly the quantised operands the storage formats hold (bf16 or e4m3
decoded without error), so the only difference to a finite-precision GEMM is accumulation
rounding.  Pinned (tests/test_oracle_linear.py): a pure-Python triple loop on tiny shapes,
linearity, and -- for the weight gradient -- convergence of the mean over seeds to the dense
product grad_Z^T X; the input gradient is pinned by its own loop and by the adjoint identity
<grad_Z, X S(W)^T> = <grad_Z S(W), X> that ties it to the forward product.
"""
import numpy as np

from . import activation
from . import formats
from . import projection
from . import mvue


def decode_activations(codes, dtype="bf16"):
    """Stored activation / gradient patterns -> exact float64 values."""
    if dtype == "bf16":
        return formats.bf16_to_f32(codes).astype(np.float64)
    if dtype == "e4m3":
        return formats.e4m3_to_f32(codes).astype(np.float64)
    if dtype == "e5m2":
        return formats.e5m2_to_f32(codes).astype(np.float64)
    raise ValueError("dtype must be 'bf16', 'e4m3' or 'e5m2'")


def linear_fwd(x_codes, vals, meta, dtype="bf16", x_scale=1.0, w_scale=1.0):
    """Z = (x_scale * w_scale) * X . decode(vals, meta)^T   in float64.  X: (T, I), result (T, O)."""
    X = decode_activations(x_codes, dtype)
    Wd = projection.decode_packed(vals, meta, dtype)
    return (X @ Wd.T) * (np.float64(np.float32(x_scale)) * np.float64(np.float32(w_scale)))


def linear_fwd_e4m3_out(x_codes, vals, meta, dtype="bf16", x_scale=1.0, w_scale=1.0, z_scale=1.0):
    """The forward product with an 8-bit output (Sec. 5.2: every operand of an FP8 GEMM is rescaled per
    tensor and cast; the output of one layer is an operand of the next).

    acc = X . decode(vals, meta)^T in float64 (the exact product of the stored operands);
    real = x_scale * w_scale (one float32 product);  q = real / z_scale (one float32 division);
    code = RNE_e4m3(clamp(float32(acc * q), +-448));  amax = max |acc| * real  (float32).
    Returns (codes uint8 (T, O), amax float32).  The consumer reads the codes with scale z_scale."""
    X = decode_activations(x_codes, dtype)
    Wd = projection.decode_packed(vals, meta, dtype)
    acc = X @ Wd.T
    real = np.float32(np.float32(x_scale) * np.float32(w_scale))
    q = np.float32(real / np.float32(z_scale))
    with np.errstate(over="ignore"):
        stored = (acc * np.float64(q)).astype(np.float32)
    codes = formats.f32_to_e4m3_rne_sat(stored).reshape(acc.shape)
    amax = np.float32(np.float32(np.max(np.abs(acc))) * real) if acc.size else np.float32(0.0)
    return codes, amax


def linear_fwd_loops(X, Wd):
    """Triple loop Z[t][o] = sum_i X[t][i] Wd[o][i] for tiny shapes (pure Python floats)."""
    T, I = X.shape
    O = Wd.shape[0]
    Z = [[0.0] * O for _ in range(T)]
    for t in range(T):
        for o in range(O):
            acc = 0.0
            for i in range(I):
                acc += float(X[t][i]) * float(Wd[o][i])
            Z[t][o] = acc
    return np.array(Z, dtype=np.float64)


def mvue_dense(dy_codes, seed, offset, dtype="bf16", first_token=0):
    """theta = MVUE(dY^T)^T as a dense-with-zeros (T, O) float64 matrix of the STORED operand values
    (for e4m3 these are theta/2; the factor 2 belongs to the epilogue scale)."""
    vals, meta = mvue.mvue_pack(dy_codes, seed, offset, dtype, first_token)
    return projection.decode_packed(vals, meta, dtype).T            # (O, T) -> (T, O)


def linear_wgrad(dy_codes, x_codes, seed, offset, dtype="bf16", dy_scale=1.0, x_scale=1.0, x_dtype=None, first_token=0):
    """grad_W = scale * MVUE(dY^T) X in float64: (O, I).  scale = dy_scale * x_scale, times 2 for the
    8-bit formats because the stored sparse operand holds theta / 2.  `dtype` is the format of dY;
    X has the same format unless x_dtype says otherwise (Sec. 5.2: e5m2 gradients against e4m3
    activations)."""
    theta = mvue_dense(dy_codes, seed, offset, dtype, first_token)  # (T, O); first_token: dY is a shard of the token axis
    X = decode_activations(x_codes, x_dtype or dtype)
    scale = np.float64(np.float32(dy_scale)) * np.float64(np.float32(x_scale))
    if dtype in ("e4m3", "e5m2"):
        scale = scale * 2.0
    return (theta.T @ X) * scale


def linear_wgrad_dense(dy_codes, x_codes, dtype="bf16", dy_scale=1.0, x_scale=1.0):
    """The dense product grad_Z^T X that MVUE estimates without bias."""
    dY = decode_activations(dy_codes, dtype)
    X = decode_activations(x_codes, dtype)
    return (dY.T @ X) * (np.float64(np.float32(dy_scale)) * np.float64(np.float32(x_scale)))


def linear_dgrad(dy_codes, vals, meta, dtype="bf16", dy_scale=1.0, w_scale=1.0, w_dtype=None):
    """grad_X = (dy_scale * w_scale) * grad_Z . decode(vals, meta)   in float64 (Sec. 5.1: the input
    gradient is the dense product with the projected weight; it is not sparsified).  dY: (T, O) in
    `dtype`, the packed weight in w_dtype (default: the same), result (T, I)."""
    dY = decode_activations(dy_codes, dtype)
    Wd = projection.decode_packed(vals, meta, w_dtype or dtype)     # (O, I)
    return (dY @ Wd) * (np.float64(np.float32(dy_scale)) * np.float64(np.float32(w_scale)))


def linear_dgrad_loops(dY, Wd):
    """Triple loop dX[t][i] = sum_o dY[t][o] Wd[o][i] for tiny shapes (pure Python floats)."""
    T, O = dY.shape
    I = Wd.shape[1]
    dX = [[0.0] * I for _ in range(T)]
    for t in range(T):
        for i in range(I):
            acc = 0.0
            for o in range(O):
                acc += float(dY[t][o]) * float(Wd[o][i])
            dX[t][i] = acc
    return np.array(dX, dtype=np.float64)


def ffn_reference(X, Wd1, Wd2, dY):
    """The feed-forward block fc1 -> activation -> fc2 and its backward pass, all in float64 with no rounding
    in between (Sec. 5.1 gives each linear layer's three products; the block chains two of them through the
    activation of ``oracle.activation``).  X (T, d), Wd1 (h, d) and Wd2 (d2, h) dense-with-zeros projected
    weights, dY (T, d2) the gradient of the block's output.  The weight gradients returned are the DENSE
    products grad_Z^T X that the estimator of Sec. 5.1 approximates without bias."""
    X = np.asarray(X, dtype=np.float64)
    H = X @ Wd1.T
    A = activation.gelu_tanh(H)
    Y = A @ Wd2.T
    dA = np.asarray(dY, dtype=np.float64) @ Wd2
    dH = dA * activation.gelu_tanh_grad(H)
    return {"H": H, "A": A, "Y": Y, "dA": dA, "dH": dH, "dX": dH @ Wd1, "dW2": np.asarray(dY, dtype=np.float64).T @ A, "dW1": dH.T @ X}
