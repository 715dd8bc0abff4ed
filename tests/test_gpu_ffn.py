"""The feed-forward block fc1 -> GELU -> fc2, forward and backward, chained through the C ABI on one stream
with the activation fused into fc1's forward epilogue and its derivative into fc2's input-gradient epilogue.
Every stage is checked against the oracle evaluated on that stage's inputs as the GPU holds them; the ends of
the chain are also checked against the float64 block with no rounding in between."""
import numpy as np
import pytest
import torch

from oracle import activation as OA
from oracle import formats as F
from oracle import linear as OL
from oracle import native as ON
from oracle import projection as OP
from paper_2409_09099_amd import workloads as WL

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sste():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2409_09099_amd as lib
    lib.library()
    return lib


def bf16_dev(bits):
    return torch.from_numpy(np.ascontiguousarray(bits.view(np.int16))).cuda().view(torch.bfloat16)


def bits_of(t):
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def f64(bits):
    return F.bf16_to_f32(bits).astype(np.float64)


def close_bf16(name, got_bits, ref, roundings=1, slack=1e-4):
    """|got - ref| <= roundings * 2^-8 |ref| + slack * max |ref| for every element."""
    got = f64(got_bits)
    rmax = float(np.max(np.abs(ref)))
    err = np.abs(got - ref)
    bad = err > roundings * 2.0 ** -8 * np.abs(ref) + slack * rmax
    k = int(np.argmax(err))
    print(f"  {name}: max|err| {err.flat[k] / rmax:.2e} of max|ref|", flush=True)
    assert not bad.any(), (name, int(bad.sum()), np.argwhere(bad)[:4])


@pytest.mark.parametrize("T,d,h", [(512, 256, 1024),        # the tiny workload's layer, as a block
                                    (320, 192, 320),         # ragged tails everywhere
                                    (16384, 1024, 4096)])    # the GPT-2-350M FFN pair at full size
def test_ffn_block_bf16(sste, T, d, h):
    wl = WL.WORKLOADS[3]
    print(f"FFN block T={T} d={d} h={h}", flush=True)
    w1, w2 = WL.weight_bits(wl, 0, O=h, I=d), WL.weight_bits(wl, 1, O=d, I=h)
    xb = WL.activations(wl, 0, T=T, I=d)[0]
    dyb = WL.output_gradient(wl, 1, T=T, O=d)[0]
    beta = np.float32(1.4830322)
    rv1, rm1, _ = OP.project_pack(w1, beta)
    rv2, rm2, _ = OP.project_pack(w2, beta)
    Wd1, Wd2 = OP.decode_packed(rv1, rm1), OP.decode_packed(rv2, rm2)
    v1, m1 = sste.project_pack(bf16_dev(w1), float(beta))
    v2, m2 = sste.project_pack(bf16_dev(w2), float(beta))
    X, dY = bf16_dev(xb), bf16_dev(dyb)

    # ---- forward: fc1 with the activation in its epilogue, then fc2 on the activation output
    H, A, _ = sste.linear_fwd_act(X, v1, m1, h)
    Y = sste.linear_fwd(A, v2, m2, d)
    hb, ab = bits_of(H), bits_of(A)
    assert torch.equal(H, sste.linear_fwd(X, v1, m1, h))                     # the stored pre-activation is the plain forward result
    close_bf16("H", hb, f64(xb) @ Wd1.T)
    close_bf16("A = gelu(H)", ab, OA.gelu_tanh(f64(hb)), slack=1e-6)         # on the H the GPU holds: one rounding
    _, A_only, _ = sste.linear_fwd_act(X, v1, m1, h, store_pre=False)        # inference: no pre-activation kept
    assert torch.equal(A_only, A)
    close_bf16("Y", bits_of(Y), f64(ab) @ Wd2.T)

    # ---- backward: fc2's input gradient with the activation's derivative in its epilogue, both weight gradients,
    # fc1's input gradient
    dH = sste.linear_dgrad_act(dY, v2, m2, h, H)
    dhb = bits_of(dH)
    close_bf16("dH = (dY S(W2)) gelu'(H)", dhb, (f64(dyb) @ Wd2) * OA.gelu_tanh_grad(f64(hb)), roundings=2)
    plain = sste.linear_dgrad(dY, v2, m2, h)                                 # the unfused pair of operations, same roundings
    unfused = f64(bits_of(plain)) * OA.gelu_tanh_grad(f64(hb))
    close_bf16("dH vs dgrad then gelu'", dhb, unfused, roundings=1, slack=1e-6)
    dW2 = sste.linear_wgrad(dY, A, 31, 0)
    theta2 = ON.decode_packed(*ON.mvue_pack(dyb, 31, 0, "bf16"), "bf16")     # (d, T)
    ref = theta2 @ f64(ab)
    assert np.max(np.abs(dW2.cpu().numpy() - ref)) <= 1e-4 * np.max(np.abs(ref))
    dW1 = sste.linear_wgrad(dH, X, 31, 1)
    theta1 = ON.decode_packed(*ON.mvue_pack(dhb, 31, 1, "bf16"), "bf16")     # (h, T)
    ref = theta1 @ f64(xb)
    assert np.max(np.abs(dW1.cpu().numpy() - ref)) <= 1e-4 * np.max(np.abs(ref))
    dX = sste.linear_dgrad(dH, v1, m1, d)
    close_bf16("dX", bits_of(dX), f64(dhb) @ Wd1)

    # ---- the ends of the chain against the float64 block (bf16 intermediates add their roundings)
    blk = OL.ffn_reference(f64(xb), Wd1, Wd2, f64(dyb))
    for name, got, want in (("Y end to end", bits_of(Y), blk["Y"]), ("dX end to end", bits_of(dX), blk["dX"])):
        err = np.max(np.abs(f64(got) - want)) / np.max(np.abs(want))
        print(f"  {name}: {err:.2e}", flush=True)
        assert err <= 1e-2


def test_ffn_block_8bit(sste):
    """The same block in the 8-bit formats of Sec. 5.2: e4m3 activations and weights, the activation written as
    e4m3 by fc1's epilogue with a delayed scale and its largest magnitude, e5m2 output gradients."""
    wl = WL.WORKLOADS[5]
    T, d, h = 1024, 256, 1024
    w1, w2 = WL.weight_bits(wl, 2, O=h, I=d), WL.weight_bits(wl, 3, O=d, I=h)
    xb = WL.activations(wl, 2, T=T, I=d)[0]
    dyb = WL.output_gradient(wl, 3, T=T, O=d)[0]
    beta = np.float32(1.4830322)

    def pack8(wb):
        _, _, amax = OP.project_pack(wb, beta)
        ws = np.float32(float(amax) / 448.0)
        rv, rm, _ = OP.project_pack(wb, beta, "e4m3", ws)
        v, m = sste.project_pack(bf16_dev(wb), float(beta), sste.F8E4M3, float(ws))
        return OP.decode_packed(rv, rm, "e4m3"), ws, v, m

    Wd1, ws1, v1, m1 = pack8(w1)
    Wd2, ws2, v2, m2 = pack8(w2)

    def quant(bits, fmt, code, fmax):
        amax = np.float32(np.max(np.abs(F.bf16_to_f32(bits))))
        scale = np.float32(float(amax) / fmax)
        codes, _ = F.cast_fp8(bits, scale, fmt)
        q, _ = sste.cast_fp8(bf16_dev(bits), float(scale), code)
        assert np.array_equal(q.cpu().numpy(), codes)
        return codes, scale, q

    xc, xs, Xq = quant(xb, "e4m3", sste.F8E4M3, 448.0)
    dyc, dys, dYq = quant(dyb, "e5m2", sste.F8E5M2, 57344.0)
    Xf, dYf = F.e4m3_to_f32(xc).astype(np.float64), F.e5m2_to_f32(dyc).astype(np.float64)

    a_scale = np.float32(2.0 / 448.0)                                        # "from earlier iterations": some headroom
    H, A8, amax = sste.linear_fwd_act(Xq, v1, m1, h, sste.F8E4M3, float(xs), float(ws1), a_dtype=sste.F8E4M3, a_scale=float(a_scale))
    hb = bits_of(H)
    close_bf16("H", hb, (Xf @ Wd1.T) * float(xs) * float(ws1), slack=1e-4)
    a_ref = OA.gelu_tanh(f64(hb))
    assert abs(float(amax.cpu()[0]) - np.max(np.abs(a_ref))) <= 1e-5 * np.max(np.abs(a_ref))
    inv = np.float32(np.float32(1.0) / a_scale)
    want = F.f32_to_e4m3_rne_sat((a_ref.astype(np.float32) * inv).astype(np.float32)).reshape(a_ref.shape)
    got = A8.cpu().numpy()
    diff = got != want
    assert diff.mean() <= 2e-3, diff.mean()                                  # the two sides round a value that differs by ~1e-6
    back = F.e4m3_to_f32(got).astype(np.float64) * float(a_scale)
    q = np.abs(a_ref) / float(a_scale)
    step = np.where(q < 2.0 ** -6, 2.0 ** -9, 2.0 ** (np.floor(np.log2(np.maximum(q, 1e-300))) - 3)) * float(a_scale)
    assert np.all(np.abs(back - a_ref) <= 0.5 * step * (1 + 1e-3) + 2e-6)
    Y = sste.linear_fwd(A8, v2, m2, d, sste.F8E4M3, float(a_scale), float(ws2))
    close_bf16("Y", bits_of(Y), (F.e4m3_to_f32(got).astype(np.float64) @ Wd2.T) * float(a_scale) * float(ws2), slack=1e-4)

    dH = sste.linear_dgrad_act(dYq, v2, m2, h, H, sste.F8E5M2, float(dys), float(ws2))
    ref = (dYf @ Wd2) * float(dys) * float(ws2) * OA.gelu_tanh_grad(f64(hb))
    close_bf16("dH", bits_of(dH), ref, roundings=2, slack=1e-4)


def test_ffn_calls_validate_their_arguments(sste):
    X = torch.zeros((64, 64), dtype=torch.bfloat16, device="cuda")
    v, m = sste.packed_buffers(16, 64, sste.BF16, "cuda")
    v.zero_()
    m.fill_(0x44)
    with pytest.raises(sste.SsteError) as ei:
        sste.linear_fwd_act(X, v, m, 16, act=7)
    assert ei.value.status == 5
    with pytest.raises(sste.SsteError) as ei:
        sste.linear_fwd_act(X, v, m, 16, a_scale=0.5)                       # a bf16 activation output has no scale
    assert ei.value.status == 5
    H, A, _ = sste.linear_fwd_act(X, v, m, 16)
    assert float(H.float().abs().max()) == 0.0 and float(A.float().abs().max()) == 0.0
    dY = torch.zeros((64, 16), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sste.SsteError) as ei:
        sste.linear_dgrad_act(dY, v, m, 64, torch.zeros((64, 32), dtype=torch.bfloat16, device="cuda"))     # H narrower than dX
    assert ei.value.status == 2
    with pytest.raises(sste.SsteError) as ei:
        sste.linear_dgrad_act(dY, v, m, 64, X, act=9)
    assert ei.value.status == 5
