"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on identical seeded inputs.

Bars: bit-exact for packed values, metadata and the sparsified operand; max |err| / max |ref| <= 1e-2
(bf16 operands) and <= 6e-2 (e4m3 operands) for the GEMM outputs, both sides using float32-or-better
accumulation on the same quantised operands.
"""
import numpy as np
import pytest
import torch

from oracle import formats as F
from oracle import linear as OL
from oracle import mvue as OM
from oracle import projection as OP
from paper_2409_09099_amd import workloads as WL

pytestmark = pytest.mark.gpu

TOL = {"bf16": 1e-2, "e4m3": 6e-2}


@pytest.fixture(scope="module")
def sste():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2409_09099_amd as lib
    lib.library()
    return lib


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.view(dtype) if dtype is not None else t


def host(t):
    return t.detach().cpu().contiguous()


def dt(lib, name):
    return {"bf16": lib.BF16, "e4m3": lib.F8E4M3, "e5m2": lib.F8E5M2}[name]


def bf16_dev(bits):
    return dev(bits.view(np.int16), torch.bfloat16)


def act_dev(codes, dtype):
    return bf16_dev(codes) if dtype == "bf16" else dev(codes)


FMT_MAX = {"e4m3": 448.0, "e5m2": 57344.0}


def operand(lib, bits, dtype):
    """bf16 patterns -> (the oracle's copy of the operand, its scale, the GPU's copy) in storage format
    `dtype`.  For the 8-bit formats each side runs its OWN per-tensor rescale + cast of Sec. 5.2 (oracle:
    formats.cast_fp8; GPU: sste_cast_fp8) with scale = largest magnitude / format maximum, and the two
    must agree bit for bit before anything is built on them."""
    bits = np.ascontiguousarray(bits)
    if dtype == "bf16":
        return bits, np.float32(1.0), bf16_dev(bits)
    xd = bf16_dev(bits)
    _, amax = lib.cast_fp8(xd, 1.0, dt(lib, dtype), store=False)
    amax_ref = np.float32(np.max(np.abs(F.bf16_to_f32(bits)))) if bits.size else np.float32(0.0)
    assert float(host(amax)[0]) == float(amax_ref)
    scale = np.float32(float(amax_ref) / FMT_MAX[dtype]) if amax_ref > 0 else np.float32(1.0)
    codes, _ = F.cast_fp8(bits, scale, dtype)
    q, _ = lib.cast_fp8(xd, float(scale), dt(lib, dtype))
    assert np.array_equal(host(q).numpy(), codes)
    return codes, scale, q


def rel_err(got, ref):
    return float(np.max(np.abs(got - ref)) / max(np.max(np.abs(ref)), 1e-300))


def z_to_f64(Z):
    return host(Z).view(torch.int16).numpy().view(np.uint16).astype(np.uint32).__lshift__(16).view(np.float32).astype(np.float64)


# ------------------------------------------------------------------------------------------ project + pack

def _edge_weights():
    """Groups that exercise ties, zeros, signed zeros, subnormals, huge values."""
    rows = [
        [1, -3, 0.5, 2], [2, -2, 1, 1], [3, 1, 1, 0], [1, 1, 1, 1], [0, 0, 0, 5], [0, 0, 0, 0],
        [-0.0, 0, -0.0, 0], [-1, -1, -1, -1], [1e-40, -2e-40, 3e-40, 0], [1e38, -3e38, 2e38, 1e-38],
        [6, 5, -5, 1], [-4, 0.25, -0.5, 8], [1.5, 1.5, -1.5, 0.1], [7, 7, 7, -7.5],
        [1e-3, 1.0000001e-3, 0.999e-3, -1e-3], [65280, 1, -65280, 3],
    ]
    w = np.array(rows, dtype=np.float32).reshape(1, -1)               # 64 weights
    w = np.concatenate([w, w[:, ::-1]], axis=1)                         # 128: one e4m3 column step
    return F.f32_to_bf16_rne(np.concatenate([w, -w, w * 0.5], axis=0))


@pytest.mark.parametrize("case", ["cfg1", "ragged", "edges", "strided"])
def test_project_pack_bf16_bit_exact(sste, case):
    wl = WL.WORKLOADS[1]
    if case == "cfg1":
        wb = WL.weight_bits(wl, 0)
    elif case == "ragged":
        wb = WL.weight_bits(wl, 0, O=77, I=1088)          # spans several workgroups, ragged row tail
    elif case == "edges":
        wb = _edge_weights()
    else:
        wb = WL.weight_bits(wl, 0, O=33, I=256)
    beta = np.float32(OP.beta_mse(F.bf16_to_f32(wb).astype(np.float64))) if case != "edges" else np.float32(1.37)
    if case == "strided":
        big = torch.zeros((33, 320), dtype=torch.bfloat16, device="cuda")
        big[:, :256] = bf16_dev(wb)
        Wd = big[:, :256]
    else:
        Wd = bf16_dev(wb)
    amax = torch.full((1,), -1.0, dtype=torch.float32, device="cuda")
    vals, meta = sste.project_pack(Wd, float(beta), amax_out=amax)
    rv, rm, ra = OP.project_pack(wb, beta)
    fv, fm = OP.to_fragment_major(rv, rm)
    assert np.array_equal(host(meta).numpy().reshape(-1), fm)
    assert np.array_equal(host(vals).numpy().view(np.uint16).reshape(-1), fv)
    assert host(amax).numpy().view(np.uint32)[0] == np.float32(ra).view(np.uint32)


@pytest.mark.parametrize("case", ["cfg1", "edges"])
def test_project_pack_e4m3_bit_exact(sste, case):
    wl = WL.WORKLOADS[1]
    wb = WL.weight_bits(wl, 0) if case == "cfg1" else _edge_weights()
    beta = np.float32(1.4830322)
    _, _, amax = OP.project_pack(wb, beta)
    scale = np.float32(amax / np.float32(448.0)) if case == "cfg1" else np.float32(0.37)
    vals, meta = sste.project_pack(bf16_dev(wb), float(beta), sste.F8E4M3, float(scale))
    rv, rm, ra = OP.project_pack(wb, beta, "e4m3", scale)
    fv, fm = OP.to_fragment_major(rv, rm, "e4m3")
    assert np.array_equal(host(meta).numpy().reshape(-1), fm)
    got = host(vals).numpy().reshape(-1)
    assert np.array_equal(got, fv), np.argwhere(got != fv)[:5]
    # the same call reporting the largest projected magnitude (another instantiation of the kernel)
    amax_d = torch.full((1,), -1.0, dtype=torch.float32, device="cuda")
    v2, m2 = sste.project_pack(bf16_dev(wb), float(beta), sste.F8E4M3, float(scale), amax_out=amax_d)
    assert torch.equal(v2, vals) and torch.equal(m2, meta)
    assert host(amax_d).numpy().view(np.uint32)[0] == np.float32(ra).view(np.uint32)


@pytest.mark.parametrize("dtype", ["bf16", "e4m3"])
@pytest.mark.parametrize("gamma", [0.33, 0.67, 1.0])
def test_project_pack_threshold_interpolation_bit_exact(sste, dtype, gamma):
    """The threshold ablation of Sec. 4.1 (t between the third- and the second-largest magnitude): packed values,
    positions and largest magnitude are the oracle's, bit for bit; gamma = 0 is the plain call."""
    wl = WL.WORKLOADS[1]
    for wb in (WL.weight_bits(wl, 0, O=77, I=1152), _edge_weights()):
        beta = np.float32(1.37)
        scale = np.float32(1.0) if dtype == "bf16" else np.float32(0.0009 if wb.shape[0] == 77 else 0.37)
        amax = torch.full((1,), -1.0, dtype=torch.float32, device="cuda")
        vals, meta = sste.project_pack(bf16_dev(wb), float(beta), dt(sste, dtype), float(scale), amax_out=amax, gamma=gamma)
        rv, rm, ra = OP.project_pack(wb, beta, dtype, scale, gamma=gamma)
        fv, fm = OP.to_fragment_major(rv, rm, dtype)
        assert np.array_equal(host(meta).numpy().reshape(-1), fm)
        assert np.array_equal(host(vals).numpy().view(fv.dtype).reshape(-1), fv)
        assert host(amax).numpy().view(np.uint32)[0] == np.float32(ra).view(np.uint32)
        # without the largest magnitude (another instantiation of the kernel): the same packed form
        v2, m2 = sste.project_pack(bf16_dev(wb), float(beta), dt(sste, dtype), float(scale), gamma=gamma)
        assert torch.equal(v2, vals) and torch.equal(m2, meta)
    W = bf16_dev(WL.weight_bits(wl, 0))
    v0, m0 = sste.project_pack(W, 1.37)
    lib = sste.library()
    v1, m1 = sste.packed_buffers(256, 1024, sste.BF16, "cuda")
    assert lib.sste_project_pack_gamma(W.data_ptr(), 256, 1024, 1024, 1.37, 0.0, sste.BF16, 1.0, v1.data_ptr(), m1.data_ptr(), None,
                                       torch.cuda.current_stream().cuda_stream) == 0
    assert torch.equal(v0, v1) and torch.equal(m0, m1)
    with pytest.raises(sste.SsteError) as ei:
        sste.project_pack(W, 1.37, gamma=1.5)
    assert ei.value.status == 5


def test_compute_beta_variants(sste):
    """The two scales Sec. 4.2 compares, for several thresholds: GPU reduction against the float64 definitions."""
    wl = WL.WORKLOADS[1]
    wb = WL.weight_bits(wl, 0, O=200, I=1024)
    W = bf16_dev(wb)
    w64 = F.bf16_to_f32(wb).astype(np.float64)
    for gamma in (0.0, 0.33, 1.0):
        # the kernel forms t in float32 from gamma as a float32: evaluate the definition at that gamma
        g32 = float(np.float32(gamma))
        for kind, ref in ((sste.BETA_MSE, OP.beta_mse(w64, g32)), (sste.BETA_L1, OP.beta_l1(w64, g32))):
            got = float(host(sste.compute_beta(W, kind, gamma))[0])
            assert abs(got - ref) <= 2e-5 * ref, (gamma, kind, got, ref)
    assert 1.45 < float(host(sste.compute_beta(W))[0]) < 1.52 and 2.3 < float(host(sste.compute_beta(W, sste.BETA_L1))[0]) < 2.7
    with pytest.raises(sste.SsteError) as ei:
        sste.compute_beta(W, 5)
    assert ei.value.status == 5


@pytest.mark.parametrize("dtype", ["bf16", "e4m3"])
def test_project_pack_batch_bit_exact(sste, dtype):
    """Many tensors in one launch: every tensor's packed form is the oracle's, bit for bit (shapes with a
    ragged row tail, a strided tensor, an empty tensor and the edge-case groups among them)."""
    wl = WL.WORKLOADS[1]
    shapes = [(256, 1024), (77, 1152), (16, 128), (0, 128), (33, 256), (40, 384)]
    wbs = [WL.weight_bits(wl, k % len(wl.layers), O=O, I=I) if O else np.zeros((0, I), dtype=np.uint16)
           for k, (O, I) in enumerate(shapes)] + [_edge_weights()]
    betas = [np.float32(1.25 + 0.125 * k) for k in range(len(wbs))]
    scales = [np.float32(1.0)] * len(wbs) if dtype == "bf16" else [np.float32(0.004 * (k + 1)) for k in range(len(wbs))]
    Ws = []
    for k, wb in enumerate(wbs):
        if k == 4:                                        # a view into a wider buffer
            big = torch.zeros((wb.shape[0], wb.shape[1] + 64), dtype=torch.bfloat16, device="cuda")
            big[:, :wb.shape[1]] = bf16_dev(wb)
            Ws.append(big[:, :wb.shape[1]])
        elif wb.shape[0] == 0:
            Ws.append(torch.empty((0, wb.shape[1]), dtype=torch.bfloat16, device="cuda"))
        else:
            Ws.append(bf16_dev(wb))
    batch = sste.PackBatch(Ws, [float(b) for b in betas], dt(sste, dtype), [float(x) for x in scales])
    for rep in range(2):                                  # the table is reusable
        for v, m in zip(batch.vals, batch.metas):
            v.fill_(0x55)
            m.fill_(0xAA)
        vals, metas = batch.launch()
        for k, wb in enumerate(wbs):
            if wb.shape[0] == 0:
                continue
            rv, rm, _ = OP.project_pack(wb, betas[k]) if dtype == "bf16" else OP.project_pack(wb, betas[k], "e4m3", scales[k])
            fv, fm = OP.to_fragment_major(rv, rm, dtype)
            assert np.array_equal(host(metas[k]).numpy().reshape(-1), fm), k
            assert np.array_equal(host(vals[k]).numpy().view(fv.dtype).reshape(-1), fv), k


@pytest.mark.parametrize("dtype", ["bf16", "e4m3"])
def test_project_pack_batch_whole_model_sized_launch(sste, dtype):
    """A launch of more than 2^18 blocks (the size from which the multi-tensor kernels write their packed
    values with the streaming hint): one tensor is compared with the oracle, every tensor with the
    single-tensor launch of the same weight and scale (itself held to the oracle above), bit for bit."""
    wl = WL.WORKLOADS[3]
    O, I = 4096, 1024
    n = 66 if dtype == "bf16" else 130                        # 4096 / 2048 blocks per tensor
    wbs = [WL.weight_bits(wl, 0, O=O, I=I), WL.weight_bits(wl, 1, O=O, I=I)]
    Wsrc = [bf16_dev(w) for w in wbs]
    Ws = [Wsrc[k % 2] for k in range(n)]                      # inputs are only read: tensors may share them
    betas = [float(np.float32(1.0 + k / 256.0)) for k in range(n)]
    scales = [1.0] * n if dtype == "bf16" else [float(np.float32(0.0005 * (1 + k % 7))) for k in range(n)]
    batch = sste.PackBatch(Ws, betas, dt(sste, dtype), scales)
    assert batch.total_blocks > (1 << 18)
    for v, m in zip(batch.vals, batch.metas):
        v.fill_(0x55)
        m.fill_(0xAA)
    vals, metas = batch.launch()
    for k in range(n):
        v1, m1 = sste.project_pack(Ws[k], betas[k], dt(sste, dtype), scales[k])
        assert torch.equal(v1.view(torch.uint8), vals[k].view(torch.uint8)) and torch.equal(m1, metas[k]), k
    k = n - 1
    rv, rm, _ = (OP.project_pack(wbs[k % 2], np.float32(betas[k])) if dtype == "bf16"
                 else OP.project_pack(wbs[k % 2], np.float32(betas[k]), "e4m3", np.float32(scales[k])))
    fv, fm = OP.to_fragment_major(rv, rm, dtype)
    assert np.array_equal(host(metas[k]).numpy().reshape(-1), fm)
    assert np.array_equal(host(vals[k]).numpy().view(fv.dtype).reshape(-1), fv)


@pytest.mark.parametrize("dtype", ["bf16", "e4m3"])
@pytest.mark.parametrize("master", ["bf16", "f32"])
def test_sgd_project_pack_batch_whole_model_sized_launch(sste, master, dtype):
    """The fused update + re-projection in a launch of more than 2^18 blocks: every tensor equals the
    single-tensor call on a copy of the same weight and gradient, bit for bit; one is held to the oracle."""
    wl = WL.WORKLOADS[3]
    O, I, n = 4096, 1024, (66 if dtype == "bf16" else 130)
    vscale = 1.0 if dtype == "bf16" else float(np.float32(0.0007))
    rng = np.random.default_rng(31)
    wb = WL.weight_bits(wl, 0, O=O, I=I)
    g = (rng.standard_normal((O, I)) * 2e-2).astype(np.float32)
    w0 = wb if master == "bf16" else (F.bf16_to_f32(wb) + (rng.standard_normal((O, I)) * 1e-5).astype(np.float32))
    W0 = bf16_dev(w0) if master == "bf16" else dev(w0)
    G = dev(g)
    Wd = [W0.clone() for _ in range(n)]
    betas = [float(np.float32(1.0 + k / 256.0)) for k in range(n)]
    alpha = 0.3
    batch = sste.UpdateBatch(Wd, [G] * n, betas, dt(sste, dtype), [vscale] * n)
    assert batch.total_blocks > (1 << 18)
    vals, metas = batch.launch(alpha)
    for k in range(n):
        Wk = W0.clone()
        v1, m1 = sste.sgd_project_pack(Wk, G, alpha, betas[k], dt(sste, dtype), vscale)
        assert torch.equal(Wk, Wd[k]) and torch.equal(v1, vals[k]) and torch.equal(m1, metas[k]), k
    k = n - 1
    w_next, rv, rm = OP.sgd_project_pack(w0, g, alpha, np.float32(betas[k]), master, dtype, np.float32(vscale))
    if master == "bf16":
        assert np.array_equal(host(Wd[k]).view(torch.int16).numpy().view(np.uint16), w_next)
    else:
        assert np.array_equal(host(Wd[k]).numpy().view(np.uint32), w_next.view(np.uint32))
    fv, fm = OP.to_fragment_major(rv, rm, dtype)
    assert np.array_equal(host(metas[k]).numpy().reshape(-1), fm)
    assert np.array_equal(host(vals[k]).numpy().view(fv.dtype).reshape(-1), fv)


@pytest.mark.parametrize("master", ["bf16", "f32"])
@pytest.mark.parametrize("dtype", ["bf16", "e4m3"])
@pytest.mark.parametrize("case", ["cfg1", "ragged_strided", "alpha0"])
def test_sgd_project_pack_bit_exact(sste, master, dtype, case):
    """Eq. (7) step fused with project + pack: the updated dense weight, the packed values and the
    metadata are the oracle's, bit for bit; padding outside strided views is untouched."""
    wl = WL.WORKLOADS[1]
    O, I = (256, 1024) if case != "ragged_strided" else (77, 1152)
    wb = WL.weight_bits(wl, 0, O=O, I=I)
    rng = np.random.default_rng(11)
    # gradients large enough that a step moves many weights across rounding and flip boundaries
    g = (rng.standard_normal((O, I)) * 2e-2).astype(np.float32)
    alpha = 0.0 if case == "alpha0" else 0.3
    beta = np.float32(1.31)
    scale = np.float32(1.0) if dtype == "bf16" else np.float32(0.0007)
    w0 = wb if master == "bf16" else (F.bf16_to_f32(wb) + (rng.standard_normal((O, I)) * 1e-5).astype(np.float32))
    pad = 64 if case == "ragged_strided" else 0
    if master == "bf16":
        Wbig = torch.full((O, I + pad), 7.0, dtype=torch.bfloat16, device="cuda")
        Wbig[:, :I] = bf16_dev(w0)
    else:
        Wbig = torch.full((O, I + pad), 7.0, dtype=torch.float32, device="cuda")
        Wbig[:, :I] = dev(w0)
    Gbig = torch.full((O, I + pad // 2), 3.0, dtype=torch.float32, device="cuda")
    Gbig[:, :I] = dev(g)
    Wd, Gd = Wbig[:, :I], Gbig[:, :I]
    vals, meta = sste.sgd_project_pack(Wd, Gd, alpha, float(beta), dt(sste, dtype), float(scale))
    w_next, rv, rm = OP.sgd_project_pack(w0, g, alpha, beta, master, dtype, scale)
    if master == "bf16":
        got_w = host(Wd).view(torch.int16).numpy().view(np.uint16)
        assert np.array_equal(got_w, w_next)
    else:
        assert np.array_equal(host(Wd).numpy().view(np.uint32), w_next.view(np.uint32))
    if pad:
        assert bool((Wbig[:, I:] == 7.0).all()) and bool((Gbig[:, I:] == 3.0).all())
    assert np.array_equal(host(Gd).numpy(), g)
    fv, fm = OP.to_fragment_major(rv, rm, dtype)
    assert np.array_equal(host(meta).numpy().reshape(-1), fm)
    assert np.array_equal(host(vals).numpy().view(fv.dtype).reshape(-1), fv)
    if case == "alpha0" and master == "bf16":
        v2, m2 = sste.project_pack(bf16_dev(wb), float(beta), dt(sste, dtype), float(scale))
        assert torch.equal(v2, vals) and torch.equal(m2, meta)


@pytest.mark.parametrize("master", ["bf16", "f32"])
@pytest.mark.parametrize("dtype", ["bf16", "e4m3"])
def test_sgd_project_pack_batch_bit_exact(sste, master, dtype):
    """Many tensors, one launch, two iterations with different learning rates: weights and packed forms
    follow the oracle's iteration bit for bit (ragged rows, a strided tensor and an empty one included)."""
    wl = WL.WORKLOADS[1]
    shapes = [(256, 1024), (77, 1152), (16, 128), (0, 128), (33, 256)]
    rng = np.random.default_rng(21)
    ws, gs = [], []
    for k, (O, I) in enumerate(shapes):
        wb = WL.weight_bits(wl, k % len(wl.layers), O=O, I=I) if O else np.zeros((0, I), dtype=np.uint16)
        ws.append(wb if master == "bf16" else (F.bf16_to_f32(wb) + (rng.standard_normal((O, I)) * 1e-5).astype(np.float32)))
        gs.append((rng.standard_normal((O, I)) * 2e-2).astype(np.float32))
    betas = [np.float32(1.25 + 0.125 * k) for k in range(len(ws))]
    scales = [np.float32(1.0)] * len(ws) if dtype == "bf16" else [np.float32(0.0006 * (k + 1)) for k in range(len(ws))]
    tdt = torch.bfloat16 if master == "bf16" else torch.float32
    Wd, Gd = [], []
    for k, (w, g) in enumerate(zip(ws, gs)):
        O, I = g.shape
        pad = 64 if k == 4 else 0
        Wbig = torch.zeros((O, I + pad), dtype=tdt, device="cuda")
        Gbig = torch.zeros((O, I + pad), dtype=torch.float32, device="cuda")
        if O:
            Wbig[:, :I] = bf16_dev(w) if master == "bf16" else dev(w)
            Gbig[:, :I] = dev(g)
        Wd.append(Wbig[:, :I])
        Gd.append(Gbig[:, :I])
    batch = sste.UpdateBatch(Wd, Gd, [float(b) for b in betas], dt(sste, dtype), [float(x) for x in scales])
    for alpha in (0.3, -0.11):
        vals, metas = batch.launch(alpha)
        for k in range(len(ws)):
            if ws[k].shape[0] == 0:
                continue
            ws[k], rv, rm = OP.sgd_project_pack(ws[k], gs[k], alpha, betas[k], master, dtype, scales[k])
            if master == "bf16":
                assert np.array_equal(host(Wd[k]).view(torch.int16).numpy().view(np.uint16), ws[k]), k
            else:
                assert np.array_equal(host(Wd[k]).numpy().view(np.uint32), ws[k].view(np.uint32)), k
            fv, fm = OP.to_fragment_major(rv, rm, dtype)
            assert np.array_equal(host(metas[k]).numpy().reshape(-1), fm), k
            assert np.array_equal(host(vals[k]).numpy().view(fv.dtype).reshape(-1), fv), k


def test_sgd_project_pack_errors(sste):
    W = torch.zeros((16, 64), dtype=torch.bfloat16, device="cuda")
    G = torch.zeros((16, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(sste.SsteError) as ei:
        sste.sgd_project_pack(W, G, float("inf"), 1.0)
    assert ei.value.status == 5
    with pytest.raises(sste.SsteError) as ei:
        sste.sgd_project_pack(W, torch.zeros((16, 66), dtype=torch.float32, device="cuda")[:, :64], 0.1, 1.0)
    assert ei.value.status == 3
    e = torch.empty((0, 64), dtype=torch.float32, device="cuda")
    vals, meta = sste.sgd_project_pack(e, e.clone(), 0.1, 1.0)
    assert vals.shape == (0, 32)


def test_project_pack_empty_and_errors(sste):
    e = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda")
    vals, meta = sste.project_pack(e, 1.0)
    assert vals.shape == (0, 32) and meta.shape == (0, 8)
    w = torch.zeros((4, 12), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sste.SsteError) as ei:
        sste.project_pack(w, 1.0, vals=torch.empty((16, 6), dtype=torch.int16, device="cuda"),
                          meta=torch.empty((16, 2), dtype=torch.uint8, device="cuda"))
    assert ei.value.status == 2
    w = torch.zeros((4, 96), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sste.SsteError) as ei:
        sste.project_pack(w, 1.0)
    assert ei.value.status == 7
    w = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sste.SsteError) as ei:
        sste.project_pack(w, float("nan"))
    assert ei.value.status == 5


def test_compute_beta_and_flip_count(sste):
    wl = WL.WORKLOADS[1]
    wb = WL.weight_bits(wl, 0)
    beta = float(host(sste.compute_beta(bf16_dev(wb)))[0])
    ref = OP.beta_mse(F.bf16_to_f32(wb).astype(np.float64))
    assert abs(beta - ref) <= 1e-5 * ref
    assert np.isnan(float(host(sste.compute_beta(torch.ones((4, 64), dtype=torch.bfloat16, device="cuda")))[0]))
    w2 = WL.weight_update_bits(wb, wl, 0, step=1)
    _, m1 = sste.project_pack(bf16_dev(wb), beta)
    _, m2 = sste.project_pack(bf16_dev(w2), beta)
    got = int(host(sste.flip_count(m1, m2, wb.shape[0]))[0])
    _, r1, _ = OP.project_pack(wb, np.float32(beta))
    _, r2, _ = OP.project_pack(w2, np.float32(beta))
    want = int(np.count_nonzero(OP.structural_mask(r1) ^ OP.structural_mask(r2)))
    assert got == want and got > 0
    assert int(host(sste.flip_count(m1, m1, wb.shape[0]))[0]) == 0


# ------------------------------------------------------------------------------------------ 8-bit cast

@pytest.mark.parametrize("fmt", ["e4m3", "e5m2"])
@pytest.mark.parametrize("case", ["activations", "strided_ragged", "saturating"])
def test_cast_fp8_bit_exact(sste, fmt, case):
    """Per-tensor rescale + cast: codes and largest magnitude are the oracle's, bit for bit; the two-call
    use (largest magnitude first, then the cast with the scale derived from it) reproduces the host-side
    quantisation of the workloads."""
    wl = WL.WORKLOADS[1]
    mx = 448.0 if fmt == "e4m3" else 57344.0
    R, C = (512, 1024) if case != "strided_ragged" else (77, 264)
    xb = WL.activations(wl, 0, T=R, I=C)[0]                               # bf16 patterns ~ N(0, 1)
    xb[0, :4] = [0x0000, 0x8000, 0x0001, 0x7F7F]                          # +0, -0, smallest subnormal, bf16 maximum
    pad = 24 if case == "strided_ragged" else 0
    Xbig = torch.full((R, C + pad), 9.0, dtype=torch.bfloat16, device="cuda")
    Xbig[:, :C] = bf16_dev(xb)
    Qbig = torch.full((R, C + pad), 0x55, dtype=torch.uint8, device="cuda")
    X, Q = Xbig[:, :C], Qbig[:, :C]
    _, amax = sste.cast_fp8(X, 1.0, dt(sste, fmt), store=False)
    amax_ref = np.float32(np.max(np.abs(F.bf16_to_f32(xb))))
    assert host(amax).numpy().view(np.uint32)[0] == amax_ref.view(np.uint32)
    assert bool((Qbig == 0x55).all())
    scale = np.float32(2.0 ** -20) if case == "saturating" else np.float32(float(amax_ref) / mx)
    amax2 = torch.full((1,), -1.0, dtype=torch.float32, device="cuda")
    sste.cast_fp8(X, float(scale), dt(sste, fmt), Q=Q, amax_out=amax2)
    codes, _ = F.cast_fp8(xb, scale, fmt)
    assert np.array_equal(host(Q).numpy(), codes)
    assert host(amax2).numpy().view(np.uint32)[0] == amax_ref.view(np.uint32)
    if pad:
        assert bool((Qbig[:, C:] == 0x55).all())
    if case == "activations" and fmt == "e4m3":
        # the same tensor through PyTorch's CPU cast (an independent implementation of the same rounding)
        t = torch.from_numpy(F.bf16_to_f32(xb).copy()) / float(scale)
        ref_codes = t.clamp_(-448.0, 448.0).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        assert np.array_equal(codes, ref_codes)


@pytest.mark.parametrize("fmt", ["e4m3", "e5m2"])
def test_cast_fp8_every_finite_bf16_value(sste, fmt):
    """Every finite bf16 pattern (both zeros, subnormals, the largest value) under scales with awkward
    significands, inside and outside the range in which the kernel forms the quotient without a division
    instruction sequence, at its edges, and far enough out that results saturate or vanish: codes are the
    oracle's (a float32 division, then the encoder) for every one."""
    pats = np.arange(65536, dtype=np.uint32)
    pats = pats[(pats & 0x7F80) != 0x7F80].astype(np.uint16)               # no infinities, no NaNs
    assert pats.size == 65280
    xb = pats.reshape(255, 256)
    X = bf16_dev(xb)
    scales = [1.0, 0.012345679, 3.0000001e-5, 0.99999994, 1.9999999, 447.99997, 2.0 ** -40, 2.0 ** -41, 2.0 ** 40, 2.0 ** 41,
              7.77e11, 1.7e-13, 2.0 ** -100, 3.1e30, 1.0000001, 5.960465e-8]
    for sc in scales:
        scale = np.float32(sc)
        q, _ = sste.cast_fp8(X, float(scale), dt(sste, fmt))
        codes, _ = F.cast_fp8(xb, scale, fmt)
        got = host(q).numpy()
        bad = np.argwhere(got != codes)
        assert bad.size == 0, (float(scale), bad[:4], [hex(int(xb[tuple(b)])) for b in bad[:4]])
    # a strided view takes the row-addressed instantiations through the same values
    big = torch.zeros((255, 256 + 32), dtype=torch.bfloat16, device="cuda")
    big[:, :256] = X
    for sc in (0.012345679, 2.0 ** -41):
        q, _ = sste.cast_fp8(big[:, :256], float(np.float32(sc)), dt(sste, fmt))
        assert np.array_equal(host(q).numpy(), F.cast_fp8(xb, np.float32(sc), fmt)[0])


def test_cast_fp8_largest_magnitude_of_tiny_tensors(sste):
    """The reported largest magnitude is exact also when it is a subnormal bf16 value or zero."""
    for top in (0x0000, 0x0001, 0x007F, 0x0080, 0x8003):
        xb = np.zeros((16, 64), dtype=np.uint16)
        xb[3, 5] = top
        xb[9, 60] = 0x8001 if top else 0x8000
        _, amax = sste.cast_fp8(bf16_dev(xb), 1.0, sste.F8E4M3, store=False)
        want = np.float32(np.max(np.abs(F.bf16_to_f32(xb))))
        assert host(amax).numpy().view(np.uint32)[0] == want.view(np.uint32), hex(top)
        q, amax2 = sste.cast_fp8(bf16_dev(xb), 1.0, sste.F8E4M3)
        assert host(amax2).numpy().view(np.uint32)[0] == want.view(np.uint32), hex(top)
        assert np.array_equal(host(q).numpy(), F.cast_fp8(xb, np.float32(1.0), "e4m3")[0])


def test_cast_fp8_empty_and_errors(sste):
    e = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda")
    q, amax = sste.cast_fp8(e, 1.0)
    assert q.shape == (0, 64) and float(host(amax)[0]) == 0.0
    x = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sste.SsteError) as ei:
        sste.cast_fp8(x, 0.0)
    assert ei.value.status == 5
    with pytest.raises(sste.SsteError) as ei:
        sste.cast_fp8(x, 1.0, sste.BF16)
    assert ei.value.status == 4
    with pytest.raises(sste.SsteError) as ei:
        sste.cast_fp8(torch.zeros((4, 60), dtype=torch.bfloat16, device="cuda"), 1.0)
    assert ei.value.status == 2


# ------------------------------------------------------------------------------------------ MVUE

def _edge_gradients(dtype):
    g = np.array([[1, 1, 1, 1], [10, 1, 1, 1], [3, 1, 1, 1], [0, 0, 0, 0], [0, 0, 7, 0], [7, 0, 0, 0], [0, 0, 0, -7],
                  [2, 0, 2, 0], [-1, 2, -3, 4], [1, -8, 2, 1], [1, 2.0 ** -30, 0, 0], [-0.0, 0, -5, 0],
                  [1e-3, -1e-3, 1e-3, -1e-3], [448, 448, 448, 448], [448, -1, 0.5, 0.25], [3, -3, 1, 0]], dtype=np.float32)
    cols = g.T                      # (4 tokens, 16 channels): each column is one group
    cols = np.concatenate([cols, cols[::-1]], axis=0)     # 8 tokens
    cols = np.tile(cols, (16, 1))                         # 128 tokens: one e4m3 column step
    if dtype == "e5m2":
        cols = np.where(np.abs(cols) == 448, np.sign(cols) * 57344, cols).astype(np.float32)    # top of the range
        cols[1, 10] = 2.0 ** -16                                                                  # smallest subnormal
        return F.f32_to_e5m2_rne_sat(cols)
    return F.f32_to_bf16_rne(cols) if dtype == "bf16" else F.f32_to_e4m3_rne_sat(cols)


@pytest.mark.parametrize("dtype", ["bf16", "e4m3", "e5m2"])
@pytest.mark.parametrize("case", ["cfg1", "ragged", "edges"])
def test_mvue_materialize_bit_exact(sste, dtype, case):
    wl = WL.WORKLOADS[1] if dtype == "bf16" else WL.WORKLOADS[5]
    if case == "cfg1":
        codes, _, dYd = operand(sste, WL.output_gradient(wl, 0, T=512, O=256)[0], dtype)
    elif case == "ragged":             # 2.6 tiles of 128 channels, a half-filled last block of 16 rows (bf16: 8-channel pieces)
        codes, _, dYd = operand(sste, WL.output_gradient(wl, 0, T=384, O=328 if dtype == "bf16" else 336)[0], dtype)
    else:
        codes = _edge_gradients(dtype)
        dYd = act_dev(codes, dtype)
    for seed, offset in [(0, 0), (1, 0), (12345678901234567, 99)]:
        vals, meta = sste.mvue_materialize(dYd, seed, offset, dt(sste, dtype))
        rv, rm = OM.mvue_pack(codes, seed, offset, dtype)
        T_, O_ = codes.shape
        gv, gm = OP.from_fragment_major(host(vals).numpy().view(rv.dtype).reshape(-1), host(meta).numpy().reshape(-1), O_, T_, dtype)
        assert np.array_equal(gm, rm), (case, seed, np.argwhere(gm != rm)[:5])
        assert np.array_equal(gv, rv), (case, seed, np.argwhere(gv != rv)[:5])


@pytest.mark.parametrize("dtype", ["bf16", "e4m3"])
def test_mvue_group_ids_beyond_32_bits_and_token_shards(sste, dtype):
    """The draw takes the 64-bit group id ((first_token + t) / 4) * O + o.  Shards of the token axis placed
    where the ids cross 2^32 inside the tensor, and far beyond it, against the oracle bit for bit; and a
    tensor cut into two shards gives the very operand of the whole."""
    wl = WL.WORKLOADS[1]
    T, O = 512, 256
    codes, _, dYd = operand(sste, WL.output_gradient(wl, 0, T=T, O=O)[0], dtype)
    for first_token in (4 * ((1 << 24) - 3), 1 << 40, 4 * ((1 << 54) + 5)):       # (2^24 - 3) * 256 = 2^32 - 768: ids cross 2^32 at group row 3
        vals, meta = sste.mvue_materialize(dYd, 9, 3, dt(sste, dtype), first_token=first_token)
        rv, rm = OM.mvue_pack(codes, 9, 3, dtype, first_token=first_token)
        gv, gm = OP.from_fragment_major(host(vals).numpy().view(rv.dtype).reshape(-1), host(meta).numpy().reshape(-1), O, T, dtype)
        assert np.array_equal(gm, rm) and np.array_equal(gv, rv), first_token
    whole_v, whole_m = OM.mvue_pack(codes, 9, 3, dtype)
    half = T // 2
    v2, m2 = sste.mvue_materialize(dYd[half:], 9, 3, dt(sste, dtype), first_token=half)
    gv, gm = OP.from_fragment_major(host(v2).numpy().view(whole_v.dtype).reshape(-1), host(m2).numpy().reshape(-1), O, half, dtype)
    assert np.array_equal(gv, whole_v[:, half // 2:]) and np.array_equal(gm, whole_m[:, half // 8:])
    with pytest.raises(sste.SsteError) as ei:
        sste.mvue_materialize(dYd, 9, 3, dt(sste, dtype), first_token=6)
    assert ei.value.status == 2


@pytest.mark.parametrize("T,O,I", [(512, 256, 128), (4096, 512, 256)])       # in-GEMM estimator; pre-pass + packed GEMM
def test_linear_wgrad_token_shards_add_up_to_the_whole(sste, T, O, I):
    wl = WL.WORKLOADS[1]
    dyb, xb = WL.output_gradient(wl, 0, T=T, O=O)[0], WL.activations(wl, 0, T=T, I=I)[0]
    dY, X = bf16_dev(dyb), bf16_dev(xb)
    whole = sste.linear_wgrad(dY, X, 5, 8)
    half = T // 2
    parts = sste.linear_wgrad(dY[:half], X[:half], 5, 8)
    sste.linear_wgrad(dY[half:], X[half:], 5, 8, dW=parts, accumulate=True, first_token=half)
    ref = OL.linear_wgrad(dyb, xb, 5, 8)
    assert rel_err(host(parts).numpy().astype(np.float64), ref) <= 1e-4
    assert rel_err(host(whole).numpy().astype(np.float64), ref) <= 1e-4
    ref2 = OL.linear_wgrad(dyb[half:], xb[half:], 5, 8, first_token=half)
    got2 = sste.linear_wgrad(dY[half:], X[half:], 5, 8, first_token=half)
    assert rel_err(host(got2).numpy().astype(np.float64), ref2) <= 1e-4
    wrong = sste.linear_wgrad(dY[half:], X[half:], 5, 8)                      # without its place in the batch: other draws
    assert not torch.equal(wrong, got2)


def test_mvue_materialize_refuses_partial_pieces(sste):
    """The estimator kernel reads dY in 16-byte pieces: channel counts and leading dimensions that are not
    whole pieces, and misaligned bases, are refused before anything is launched."""
    for dtype, tdt, O in (("bf16", torch.bfloat16, 333), ("e4m3", torch.uint8, 328), ("e5m2", torch.uint8, 24)):
        dY = torch.zeros((128, O), dtype=tdt, device="cuda")
        with pytest.raises(sste.SsteError) as ei:
            sste.mvue_materialize(dY, 0, 0, dt(sste, dtype))
        assert ei.value.status == 7, dtype
    wide = torch.zeros((128, 72), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sste.SsteError) as ei:          # rows of 72 elements, 68-element stride is impossible; 8-element view of a 12-stride buffer
        sste.mvue_materialize(torch.zeros((128, 12), dtype=torch.bfloat16, device="cuda")[:, :8], 0, 0)
    assert ei.value.status == 3
    with pytest.raises(sste.SsteError) as ei:          # base pointer 8 bytes into a row
        sste.mvue_materialize(wide[:, 4:68], 0, 0)
    assert ei.value.status == 3


# ------------------------------------------------------------------------------------------ forward GEMM

def _fwd_case(sste, dtype, T, O, I, seed_layer=0):
    wl = WL.WORKLOADS[1] if dtype == "bf16" else WL.WORKLOADS[5]
    wb = WL.weight_bits(wl, seed_layer, O=O, I=I)
    xc, xs, Xd = operand(sste, WL.activations(wl, seed_layer, T=T, I=I)[0], dtype)
    beta = np.float32(1.4830322)
    if dtype == "bf16":
        ws = np.float32(1.0)
        rv, rm, _ = OP.project_pack(wb, beta)
        vals, meta = sste.project_pack(bf16_dev(wb), float(beta))
    else:
        _, _, amax = OP.project_pack(wb, beta)
        ws = np.float32(max(float(amax), 1e-30) / 448.0)
        rv, rm, _ = OP.project_pack(wb, beta, "e4m3", ws)
        vals, meta = sste.project_pack(bf16_dev(wb), float(beta), sste.F8E4M3, float(ws))
    Z = sste.linear_fwd(Xd, vals, meta, O, dt(sste, dtype), float(xs), float(ws))
    ref = OL.linear_fwd(xc, rv, rm, dtype, xs, ws)
    return z_to_f64(Z), ref


@pytest.mark.parametrize("dtype,T,O,I", [
    ("bf16", 512, 256, 1024),        # the tiny workload
    ("bf16", 200, 136, 192),         # ragged T and O tails inside one and across two tiles
    ("bf16", 1, 8, 64),              # single token, one k-step
    ("bf16", 300, 264, 64),
    ("e4m3", 512, 256, 1024),
    ("e4m3", 130, 72, 256),
    # pipelined 256 x 256 kernel (128 .. 256 tiles), ragged token and channel tails
    ("bf16", 16424, 520, 128),
    ("e4m3", 16424, 520, 128),
    # two tile shapes in one grid (262 tiles: 256 full + 12 halves), last token tile 64 rows: its second half is empty
    ("bf16", 33344, 264, 64),
    ("e4m3", 33344, 264, 128),
])
def test_linear_fwd_matches_oracle(sste, dtype, T, O, I):
    got, ref = _fwd_case(sste, dtype, T, O, I)
    assert got.shape == ref.shape
    err = rel_err(got, ref)
    assert err <= TOL[dtype], err
    # tighter sanity bound: bf16 output rounding (2^-9 of the value) plus float32 accumulation noise
    assert np.all(np.abs(got - ref) <= np.abs(ref) * 2.0 ** -8 + np.max(np.abs(ref)) * 1e-4)


@pytest.mark.parametrize("dtype,T,O,I", [
    ("bf16", 512, 256, 1024),        # one-wave tiles
    ("e4m3", 300, 272, 256),         # ragged token and channel tails
    ("e4m3", 2100, 1040, 256),       # 256 x 128 four-wave tiles
    ("bf16", 16424, 528, 128),       # pipelined 256 x 256 tiles, ragged tails
    ("e4m3", 33344, 272, 128),       # two tile shapes in one grid
    ("bf16", 2100, 1040, 128),       # 256 x 128 four-wave tiles, bf16 operands
    ("bf16", 33344, 272, 128),       # two tile shapes in one grid, bf16 operands
    ("e4m3", 16424, 528, 128),       # pipelined 256 x 256 tiles, 8-bit operands
])
def test_linear_fwd_e4m3_output_and_amax(sste, dtype, T, O, I):
    """The forward product cast to e4m3 where it is produced (Sec. 5.2) and its largest magnitude.  Both sides
    round the same product, the GPU from a float32 accumulator and the oracle from float64, so codes may differ
    where the product sits on a rounding boundary: they must agree almost everywhere, differ by one step where
    they do not, and decode to the float64 product within half a step of the grid plus the accumulation noise.  The bf16 output with amax_out is the
    plain forward result, bit for bit."""
    wl = WL.WORKLOADS[1] if dtype == "bf16" else WL.WORKLOADS[5]
    wb = WL.weight_bits(wl, 0, O=O, I=I)
    xc, xs, Xd = operand(sste, WL.activations(wl, 0, T=T, I=I)[0], dtype)
    beta = np.float32(1.4830322)
    if dtype == "bf16":
        ws = np.float32(1.0)
        rv, rm, _ = OP.project_pack(wb, beta)
    else:
        _, _, amax_w = OP.project_pack(wb, beta)
        ws = np.float32(float(amax_w) / 448.0)
        rv, rm, _ = OP.project_pack(wb, beta, "e4m3", ws)
    vals, meta = sste.project_pack(bf16_dev(wb), float(beta), dt(sste, dtype), float(ws))
    ref = OL.linear_fwd(xc, rv, rm, dtype, xs, ws)
    amax_ref = float(np.max(np.abs(ref)))

    # bf16 output + amax: the same Z as sste_linear_fwd, and the largest magnitude of the unrounded product
    Z16, amax16 = sste.linear_fwd_ex(Xd, vals, meta, O, dt(sste, dtype), float(xs), float(ws),
                                     amax_out=torch.full((1,), -1.0, dtype=torch.float32, device="cuda"))
    assert torch.equal(Z16, sste.linear_fwd(Xd, vals, meta, O, dt(sste, dtype), float(xs), float(ws)))
    assert abs(float(host(amax16)[0]) - amax_ref) <= 2e-5 * amax_ref

    # e4m3 output with a scale from "earlier iterations": a little headroom over the true maximum
    z_scale = np.float32(1.25 * amax_ref / 448.0)
    Z8, amax8 = sste.linear_fwd_ex(Xd, vals, meta, O, dt(sste, dtype), float(xs), float(ws), sste.F8E4M3, float(z_scale))
    assert float(host(amax8)[0]) == float(host(amax16)[0])
    want, amax_o = OL.linear_fwd_e4m3_out(xc, rv, rm, dtype, xs, ws, z_scale)
    assert abs(float(amax_o) - float(host(amax8)[0])) <= 2e-5 * amax_ref
    got = host(Z8).numpy()
    assert got.shape == want.shape
    diff = got != want
    assert diff.mean() <= 2e-3, diff.mean()
    # Where the codes differ, the two roundings saw products that differ by the float32 accumulation noise of
    # the matrix pipe (the same allowance as for the bf16 output: 1e-4 of the largest output); for most outputs
    # that is less than a step of the grid (neighbouring codes), for outputs near zero it can span a few steps.
    back = F.e4m3_to_f32(got).astype(np.float64) * float(z_scale)
    q = np.abs(ref) / float(z_scale)
    step = np.where(q < 2.0 ** -6, 2.0 ** -9, 2.0 ** (np.floor(np.log2(np.maximum(q, 1e-300))) - 3)) * float(z_scale)
    excess = np.abs(back - ref) - 0.5 * step * (1 + 1e-3)
    print(f"e4m3 output: {diff.mean():.2e} of the codes differ, worst excess over half a step {excess.max() / amax_ref:.2e} of max|Z|", flush=True)
    assert np.all(excess <= 1e-4 * amax_ref)
    gm, wm = got[diff].astype(np.int32), want[diff].astype(np.int32)
    near = (np.abs((gm & 0x7F) - (wm & 0x7F)) == 1) & ((gm >> 7) == (wm >> 7)) | ((gm & 0x7F) + (wm & 0x7F) <= 1)
    assert near.mean() >= 0.9 if near.size else True
    # saturation instead of overflow when the scale is far too small
    Zs, _ = sste.linear_fwd_ex(Xd, vals, meta, O, dt(sste, dtype), float(xs), float(ws), sste.F8E4M3, float(z_scale) / 64.0)
    sat = host(Zs).numpy()
    assert np.all((sat & 0x7F) <= 0x7E) and np.any((sat & 0x7F) == 0x7E)
    # strided e4m3 output: the padding columns stay untouched
    big = torch.full((T, O + 32), 0x55, dtype=torch.uint8, device="cuda")
    sste.linear_fwd_ex(Xd, vals, meta, O, dt(sste, dtype), float(xs), float(ws), sste.F8E4M3, float(z_scale), Z=big[:, :O],
                       amax_out=amax8)
    assert torch.equal(big[:, :O], Z8) and bool((big[:, O:] == 0x55).all())


def test_fp8_output_feeds_the_next_layer_with_delayed_scaling(sste):
    """Two chained 8-bit layers over three iterations: layer 1 writes its output as e4m3 with a scale taken from
    the amax history of earlier iterations, layer 2 consumes those codes directly.  Each stage against the oracle
    on the inputs the GPU holds."""
    wl = WL.WORKLOADS[5]
    T, I, H, O = 256, 256, 384, 128
    w1, w2 = WL.weight_bits(wl, 2, O=H, I=I), WL.weight_bits(wl, 3, O=O, I=H)
    beta = np.float32(1.4830322)
    packs = []
    for wb in (w1, w2):
        _, _, amax_w = OP.project_pack(wb, beta)
        ws = np.float32(float(amax_w) / 448.0)
        rv, rm, _ = OP.project_pack(wb, beta, "e4m3", ws)
        v, m = sste.project_pack(bf16_dev(wb), float(beta), sste.F8E4M3, float(ws))
        packs.append((rv, rm, ws, v, m))
    hist = sste.AmaxHistory(2)
    z_scale = 1.0                                                   # first iteration: nothing known yet
    for it in range(3):
        xb = F.f32_to_bf16_rne((F.bf16_to_f32(WL.activations(wl, 0, T=T, I=I)[0]) * np.float32(1.0 + it)).astype(np.float32)).reshape(T, I)
        xc, xs, Xd = operand(sste, xb, "e4m3")
        rv, rm, ws, v, m = packs[0]
        Z8, amax = sste.linear_fwd_ex(Xd, v, m, H, sste.F8E4M3, float(xs), float(ws), sste.F8E4M3, z_scale)
        zc = host(Z8).numpy()
        want, amax_o = OL.linear_fwd_e4m3_out(xc, rv, rm, "e4m3", xs, ws, np.float32(z_scale))
        assert (zc != want).mean() <= 5e-3
        assert abs(float(host(amax)[0]) - float(amax_o)) <= 2e-5 * float(amax_o)
        # layer 2 reads the codes the GPU wrote, with the scale they were written with
        rv2, rm2, ws2, v2, m2 = packs[1]
        Y = sste.linear_fwd(Z8, v2, m2, O, sste.F8E4M3, z_scale, float(ws2))
        assert rel_err(z_to_f64(Y), OL.linear_fwd(zc, rv2, rm2, "e4m3", np.float32(z_scale), ws2)) <= TOL["e4m3"]
        z_scale = hist.push(float(host(amax)[0]), 448.0)           # scale of the next iteration
        assert z_scale == float(F.delayed_scale([float(host(amax)[0])] if it == 0 else prev + [float(host(amax)[0])], "e4m3"))
        prev = [float(host(amax)[0])]


def test_linear_fwd_empty_and_errors(sste):
    X = torch.zeros((0, 64), dtype=torch.bfloat16, device="cuda")
    vals = torch.zeros((16, 32), dtype=torch.int16, device="cuda")
    meta = torch.full((16, 8), 0x44, dtype=torch.uint8, device="cuda")
    assert sste.linear_fwd(X, vals, meta, 8).shape == (0, 8)
    X = torch.zeros((4, 96), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sste.SsteError) as ei:
        sste.linear_fwd(X, torch.zeros((16, 48), dtype=torch.int16, device="cuda"), torch.zeros((16, 12), dtype=torch.uint8, device="cuda"), 8)
    assert ei.value.status == 7


# ------------------------------------------------------------------------------------------ weight-gradient GEMM

def _wgrad_case(sste, dtype, T, O, I, seed=3, offset=5, **kw):
    wl = WL.WORKLOADS[1] if dtype == "bf16" else WL.WORKLOADS[5]
    dyc, dys, dYd = operand(sste, WL.output_gradient(wl, 0, T=T, O=O)[0], dtype)
    xc, xs, Xd = operand(sste, WL.activations(wl, 0, T=T, I=I)[0], "e4m3" if dtype == "e5m2" else dtype)
    dW = sste.linear_wgrad(dYd, Xd, seed, offset, dt(sste, dtype), float(dys), float(xs), **kw)
    ref = OL.linear_wgrad(dyc, xc, seed, offset, dtype, dys, xs, x_dtype="e4m3" if dtype == "e5m2" else None)
    return dW, ref


@pytest.mark.parametrize("dtype,T,O,I", [
    ("bf16", 512, 256, 1024),        # the tiny workload
    ("bf16", 64, 8, 8),              # one k-step, one partial tile
    ("bf16", 192, 136, 200),         # ragged O and I tails
    ("bf16", 4096, 128, 128),        # one tile, token axis split across workgroups
    ("bf16", 2048, 264, 328),        # estimator pre-pass + packed GEMM, ragged channel and feature tails
    ("bf16", 4096, 512, 256),        # pre-pass path, several tiles and splits
    ("e4m3", 512, 256, 1024),
    ("e4m3", 256, 144, 80),
    ("e4m3", 8192, 128, 128),
    ("e4m3", 2048, 272, 320),        # pre-pass path, ragged tails
    ("e5m2", 512, 256, 1024),        # e5m2 gradients against e4m3 activations (Sec. 5.2): fused kernel
    ("e5m2", 256, 144, 80),
    ("e5m2", 2048, 272, 320),        # pre-pass + packed GEMM
    ("e5m2", 4096, 512, 256),
])
def test_linear_wgrad_matches_oracle(sste, dtype, T, O, I):
    dW, ref = _wgrad_case(sste, dtype, T, O, I)
    got = host(dW).numpy().astype(np.float64)
    assert got.shape == ref.shape
    err = rel_err(got, ref)
    assert err <= TOL.get(dtype, 6e-2), err
    # the sparse operand is bit-identical on both sides, so only float32 accumulation order differs
    assert err <= 1e-4, err


@pytest.mark.parametrize("dtype", ["bf16", "e4m3", "e5m2"])
@pytest.mark.parametrize("mi,ni,splits", [(8, 4, 1), (8, 4, 3), (8, 3, 2), (8, 3, 5), (6, 3, 4)])
def test_linear_wgrad_every_tile_shape_with_ragged_tails(sste, dtype, mi, ni, splits):
    """The large-problem path with each workgroup tile (256 x 256, 256 x 192, 192 x 192) and several split
    counts forced, on shapes whose channel and feature counts end inside a tile and inside a 16-row block:
    every element against the oracle, and the split count must not change the estimator's draws."""
    T, O, I = (2560, 520, 456) if dtype == "bf16" else (2560, 528, 464)
    try:
        sste.wgrad_plan_override(mi, ni, splits)
        dW, ref = _wgrad_case(sste, dtype, T, O, I, seed=17, offset=2)
        got = host(dW).numpy().astype(np.float64)
    finally:
        sste.wgrad_plan_override(0, 0, 0)
    assert got.shape == ref.shape
    assert rel_err(got, ref) <= 1e-4
    with pytest.raises(sste.SsteError) as ei:
        sste.wgrad_plan_override(4, 4, 0)
    assert ei.value.status == 5


def test_linear_wgrad_accumulate_and_reproducible(sste):
    T, O, I = 4096, 128, 256
    dW1, ref = _wgrad_case(sste, "bf16", T, O, I)
    dW2, _ = _wgrad_case(sste, "bf16", T, O, I)
    assert torch.equal(dW1, dW2)                                   # fixed-order split reduction
    base = torch.full((O, I), 0.5, dtype=torch.float32, device="cuda")
    dW3, _ = _wgrad_case(sste, "bf16", T, O, I, dW=base, accumulate=True)
    assert rel_err(host(dW3).numpy().astype(np.float64), ref + 0.5) <= 1e-5
    # a different seed gives a different estimate of the same dense gradient
    dW4, ref4 = _wgrad_case(sste, "bf16", T, O, I, seed=4)
    assert not torch.equal(dW1, dW4)
    assert rel_err(host(dW4).numpy().astype(np.float64), ref4) <= 1e-4


def test_linear_wgrad_strided_output_and_errors(sste):
    T, O, I = 128, 16, 24
    big = torch.zeros((O, 40), dtype=torch.float32, device="cuda")
    dW, ref = _wgrad_case(sste, "bf16", T, O, I, dW=big[:, :I])
    assert rel_err(host(big[:, :I]).numpy().astype(np.float64), ref) <= 1e-4
    assert float(big[:, I:].abs().max()) == 0.0
    dY = torch.zeros((100, 16), dtype=torch.bfloat16, device="cuda")
    X = torch.zeros((100, 16), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sste.SsteError) as ei:
        sste.linear_wgrad(dY, X, 0, 0)
    assert ei.value.status == 7
    dY = torch.zeros((102, 16), dtype=torch.bfloat16, device="cuda")
    X = torch.zeros((102, 16), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sste.SsteError) as ei:
        sste.linear_wgrad(dY, X, 0, 0)
    assert ei.value.status == 2


def test_linear_wgrad_of_an_empty_batch(sste):
    """T = 0: the sum over no tokens is zero -- dW is cleared (its padding columns are not), or left as it
    is when the call accumulates."""
    O, I = 48, 40
    dY = torch.empty((0, O), dtype=torch.bfloat16, device="cuda")
    X = torch.empty((0, I), dtype=torch.bfloat16, device="cuda")
    big = torch.full((O, I + 8), 2.5, dtype=torch.float32, device="cuda")
    sste.linear_wgrad(dY, X, 1, 2, dW=big[:, :I], accumulate=True)
    assert bool((big == 2.5).all())
    sste.linear_wgrad(dY, X, 1, 2, dW=big[:, :I])
    assert bool((big[:, :I] == 0.0).all()) and bool((big[:, I:] == 2.5).all())


# ------------------------------------------------------------------------------------------ strided operands, large-problem kernels

def test_large_kernels_with_strided_operands(sste):
    """X, dY, Z and dW are views into wider buffers (leading dimension > row length) at sizes that take the
    pipelined forward kernel and the pre-pass + packed GEMM of the weight gradient; the padding columns of the
    outputs must stay untouched."""
    T, O, I = 16448, 520, 320
    wl = WL.WORKLOADS[1]
    wb = WL.weight_bits(wl, 0, O=O, I=I)
    xc, xs = WL.activations(wl, 0, T=T, I=I)
    dyc, dys = WL.output_gradient(wl, 0, T=T, O=O)
    beta = np.float32(1.4830322)
    rv, rm, _ = OP.project_pack(wb, beta)
    vals, meta = sste.project_pack(bf16_dev(wb), float(beta))

    Xbig = torch.full((T, I + 64), 7.0, dtype=torch.bfloat16, device="cuda")
    Xbig[:, :I] = act_dev(xc, "bf16")
    dYbig = torch.full((T, O + 24), 3.0, dtype=torch.bfloat16, device="cuda")
    dYbig[:, :O] = act_dev(dyc, "bf16")
    Zbig = torch.full((T, O + 8), -5.0, dtype=torch.bfloat16, device="cuda")
    dWbig = torch.full((O, I + 12), 9.0, dtype=torch.float32, device="cuda")

    sste.linear_fwd(Xbig[:, :I], vals, meta, O, sste.BF16, float(xs), 1.0, Z=Zbig[:, :O])
    ref = OL.linear_fwd(xc, rv, rm, "bf16", xs, np.float32(1.0))
    assert rel_err(z_to_f64(Zbig[:, :O]), ref) <= TOL["bf16"]
    assert float((Zbig[:, O:].float() + 5.0).abs().max()) == 0.0

    sste.linear_wgrad(dYbig[:, :O], Xbig[:, :I], 11, 2, sste.BF16, float(dys), float(xs), dW=dWbig[:, :I])
    refw = OL.linear_wgrad(dyc, xc, 11, 2, "bf16", dys, xs)
    assert rel_err(host(dWbig[:, :I]).numpy().astype(np.float64), refw) <= 1e-4
    assert float((dWbig[:, I:] - 9.0).abs().max()) == 0.0


# ------------------------------------------------------------------------------------------ HIP graph capture

def test_step_under_graph_capture_replays_bit_exact(sste):
    """The library only enqueues kernels on the caller's stream (no allocation, no synchronisation, no
    memset nodes), so a whole step can be captured into a HIP graph.  Every replay must reproduce the eager
    result bit for bit, with eager work and synchronisations between the replays."""
    T, O, I = 4096, 512, 256                       # takes the estimator pre-pass + packed GEMM + reduction
    wl = WL.WORKLOADS[1]
    W = bf16_dev(WL.weight_bits(wl, 0, O=O, I=I))
    X = bf16_dev(WL.activations(wl, 0, T=T, I=I)[0])
    dY = bf16_dev(WL.output_gradient(wl, 0, T=T, O=O)[0])
    beta = 1.4830322
    vals, meta = sste.packed_buffers(O, I, sste.BF16, "cuda")
    Z = torch.empty((T, O), dtype=torch.bfloat16, device="cuda")
    dW = torch.empty((O, I), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(sste.wgrad_workspace_bytes(T, O, I, sste.BF16), 16), dtype=torch.uint8, device="cuda")

    def step():
        sste.project_pack(W, beta, vals=vals, meta=meta)
        sste.linear_fwd(X, vals, meta, O, Z=Z)
        sste.linear_wgrad(dY, X, 5, 9, dW=dW, workspace=ws)

    step()
    torch.cuda.synchronize()
    ref = [t.clone() for t in (vals, meta, Z, dW)]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                     # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for rep in range(4):
        for t in (vals, meta, Z, dW, ws):
            t.view(torch.uint8).fill_(0x3C + rep)  # eager work between replays; also proves the replay rewrites everything
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip((vals, meta, Z, dW), ref):
            assert torch.equal(got.view(torch.uint8), want.view(torch.uint8)), rep


# ------------------------------------------------------------------------------------------ input gradient

@pytest.mark.parametrize("dtype", ["bf16", "e4m3", "e5m2"])
@pytest.mark.parametrize("T,O,I", [
    (512, 256, 1024),          # the tiny workload's shapes
    (300, 272, 384),           # ragged token tile, channel count not a multiple of the k-step, ragged feature tile
    (1, 16, 128),              # single token, one partial k-step
    (1000, 528, 640),          # several k-steps, three feature tiles
    (8, 0, 128),               # no channels: zeros
    (16384, 144, 128),         # many token tiles: the 256 x 256 tile kernel
    (65892, 32, 128),          # 258 tiles: a whole round of 256 x 256 tiles + the rest as 256 x 128 halves, ragged tail
])
def test_linear_dgrad_matches_oracle(sste, dtype, T, O, I):
    wl = WL.WORKLOADS[1] if dtype == "bf16" else WL.WORKLOADS[5]
    beta = np.float32(1.4830322)
    dys = np.float32(1.0)
    if O:
        dyc, dys, dY = operand(sste, WL.output_gradient(wl, 0, T=T, O=O)[0], dtype)
    ws = np.float32(1.0)
    wdt = "e4m3" if dtype == "e5m2" else dtype                 # e5m2 gradients meet an e4m3 weight (Sec. 5.2)
    if O:
        wb = WL.weight_bits(wl, 0, O=O, I=I)
        if wdt == "e4m3":
            _, _, amax = OP.project_pack(wb, beta)
            ws = np.float32(amax / np.float32(448.0))
        rv, rm, _ = OP.project_pack(wb, beta, wdt, ws)
        vals, meta = sste.project_pack(bf16_dev(wb), float(beta), dt(sste, wdt), float(ws))
        ref = OL.linear_dgrad(dyc, rv, rm, dtype, dys, ws, w_dtype=wdt)
    else:
        vals, meta = sste.packed_buffers(0, I, dt(sste, wdt), "cuda")
        ref = np.zeros((T, I))
        dY = torch.zeros((T, 16), dtype=torch.bfloat16 if dtype == "bf16" else torch.uint8, device="cuda")[:, :0]
    dX = torch.full((T, I), 7.0, dtype=torch.bfloat16, device="cuda")
    sste.linear_dgrad(dY, vals, meta, I, dt(sste, dtype), float(dys), float(ws), dX=dX)
    got = z_to_f64(dX)
    if O == 0:
        assert np.all(got == 0.0)
        return
    assert rel_err(got, ref) <= TOL.get(dtype, 6e-2)
    # operands are identical on both sides: only float32 accumulation order and the bf16 output rounding differ
    assert np.all(np.abs(got - ref) <= np.abs(ref) * 2.0 ** -8 + np.max(np.abs(ref)) * 1e-4)


def test_linear_dgrad_strided_and_errors(sste):
    T, O, I = 260, 72, 128
    wl = WL.WORKLOADS[1]
    wb = WL.weight_bits(wl, 0, O=O, I=I)
    dyc, dys = WL.output_gradient(wl, 0, T=T, O=O)
    rv, rm, _ = OP.project_pack(wb, np.float32(1.25))
    vals, meta = sste.project_pack(bf16_dev(wb), 1.25)
    dYbig = torch.full((T, O + 24), 3.0, dtype=torch.bfloat16, device="cuda")
    dYbig[:, :O] = bf16_dev(dyc)
    dXbig = torch.full((T, I + 8), -5.0, dtype=torch.bfloat16, device="cuda")
    sste.linear_dgrad(dYbig[:, :O], vals, meta, I, sste.BF16, float(dys), 1.0, dX=dXbig[:, :I])
    ref = OL.linear_dgrad(dyc, rv, rm, "bf16", dys, np.float32(1.0))
    assert rel_err(z_to_f64(dXbig[:, :I]), ref) <= TOL["bf16"]
    assert float((dXbig[:, I:].float() + 5.0).abs().max()) == 0.0
    with pytest.raises(sste.SsteError) as ei:          # e4m3 rows are 16 channels to the 16 bytes
        sste.linear_dgrad(torch.zeros((T, 72), dtype=torch.uint8, device="cuda"), vals, meta, I, sste.F8E4M3)
    assert ei.value.status == 7
    with pytest.raises(sste.SsteError) as ei:
        sste.linear_dgrad(dYbig[:, :O], vals, meta, 96)
    assert ei.value.status == 7


# ------------------------------------------------------------------------------------------ whole iterations

def test_training_iterations_chain(sste):
    """Three iterations of one layer through the C ABI: project+pack -> forward -> weight gradient and
    input gradient -> dense-weight step fused with the next projection (Sec. 2, the three steps of an
    iteration).  Every stage is checked against the oracle evaluated on that stage's inputs as the GPU
    holds them: packed weight, weights after the step and estimator draws are bit-exact; GEMM outputs meet
    the bf16 bar.  The recorded positions must change somewhere over the iterations (flips, Sec. 3.3)."""
    wl = WL.WORKLOADS[1]
    T, O, I = 512, 256, 1024
    wb = WL.weight_bits(wl, 0)
    xc, xs = WL.activations(wl, 0)
    dyc, dys = WL.output_gradient(wl, 0)
    beta = np.float32(OP.beta_mse(F.bf16_to_f32(wb).astype(np.float64)))
    W = bf16_dev(wb)
    X, dY = bf16_dev(xc), bf16_dev(dyc)
    vals, meta = sste.project_pack(W, float(beta))
    w_host = wb.copy()
    rv, rm, _ = OP.project_pack(w_host, beta)
    first_meta = rm.copy()
    alpha = 0.2                                              # steps of about a quarter of a typical weight: groups flip
    for it in range(3):
        fv, fm = OP.to_fragment_major(rv, rm)
        assert np.array_equal(host(meta).numpy().reshape(-1), fm), it
        assert np.array_equal(host(vals).numpy().view(np.uint16).reshape(-1), fv), it
        Z = sste.linear_fwd(X, vals, meta, O)
        assert rel_err(z_to_f64(Z), OL.linear_fwd(xc, rv, rm, "bf16", xs, np.float32(1.0))) <= TOL["bf16"]
        dX = sste.linear_dgrad(dY, vals, meta, I, sste.BF16, float(dys), 1.0)
        assert rel_err(z_to_f64(dX), OL.linear_dgrad(dyc, rv, rm, "bf16", dys, np.float32(1.0))) <= TOL["bf16"]
        dW = sste.linear_wgrad(dY, X, 77, it, sste.BF16, float(dys), float(xs))
        ref_dw = OL.linear_wgrad(dyc, xc, 77, it, "bf16", dys, xs)
        assert rel_err(host(dW).numpy().astype(np.float64), ref_dw) <= 1e-4
        g = host(dW).numpy()                                 # the step is checked on the gradient the GPU holds
        vals, meta = sste.sgd_project_pack(W, dW, alpha, float(beta), vals=vals, meta=meta)
        w_host, rv, rm = OP.sgd_project_pack(w_host, g, alpha, beta)
        assert np.array_equal(host(W).view(torch.int16).numpy().view(np.uint16), w_host), it
    fv, fm = OP.to_fragment_major(rv, rm)
    assert np.array_equal(host(meta).numpy().reshape(-1), fm)
    assert np.count_nonzero(OP.structural_mask(first_meta) ^ OP.structural_mask(rm)) > 0


def test_fp8_iteration_with_gpu_side_casts(sste):
    """The 8-bit recipe of Sec. 5.2 end to end through the C ABI: bf16 activations and output gradients
    are rescaled per tensor and cast on the GPU (e4m3 / e5m2, scale from the tensor's own largest
    magnitude), the weight is projected to e4m3 with its own scale, then forward, weight gradient and
    input gradient run on the 8-bit operands.  Every stage against the oracle on that stage's inputs."""
    wl = WL.WORKLOADS[1]
    T, O, I = 512, 256, 1024
    wb = WL.weight_bits(wl, 0)
    xb = WL.activations(wl, 0)[0]                                   # bf16 patterns
    dyb = WL.output_gradient(wl, 0)[0]
    beta = np.float32(1.4830322)
    W, X, dY = bf16_dev(wb), bf16_dev(xb), bf16_dev(dyb)

    def cast(t, bits, fmt, mx):
        _, amax = sste.cast_fp8(t, 1.0, dt(sste, fmt), store=False)
        scale = np.float32(float(host(amax)[0]) / mx)
        q, _ = sste.cast_fp8(t, float(scale), dt(sste, fmt))
        codes, amax_ref = F.cast_fp8(bits, scale, fmt)
        assert float(host(amax)[0]) == float(amax_ref)
        assert np.array_equal(host(q).numpy(), codes)
        return q, codes, scale

    Xq, xc, xs = cast(X, xb, "e4m3", 448.0)
    dYq, dyc, dys = cast(dY, dyb, "e5m2", 57344.0)
    amax = torch.zeros(1, dtype=torch.float32, device="cuda")
    sste.project_pack(W, float(beta), amax_out=amax)
    ws = np.float32(float(host(amax)[0]) / 448.0)
    vals, meta = sste.project_pack(W, float(beta), sste.F8E4M3, float(ws))
    rv, rm, ra = OP.project_pack(wb, beta, "e4m3", ws)
    assert np.float32(float(ra) / 448.0) == ws
    fv, fm = OP.to_fragment_major(rv, rm, "e4m3")
    assert np.array_equal(host(vals).numpy().reshape(-1), fv) and np.array_equal(host(meta).numpy().reshape(-1), fm)
    Z = sste.linear_fwd(Xq, vals, meta, O, sste.F8E4M3, float(xs), float(ws))
    assert rel_err(z_to_f64(Z), OL.linear_fwd(xc, rv, rm, "e4m3", xs, ws)) <= TOL["e4m3"]
    dW = sste.linear_wgrad(dYq, Xq, 3, 1, sste.F8E5M2, float(dys), float(xs))
    assert rel_err(host(dW).numpy().astype(np.float64), OL.linear_wgrad(dyc, xc, 3, 1, "e5m2", dys, xs, x_dtype="e4m3")) <= 1e-4
    dX = sste.linear_dgrad(dYq, vals, meta, I, sste.F8E5M2, float(dys), float(ws))
    assert rel_err(z_to_f64(dX), OL.linear_dgrad(dyc, rv, rm, "e5m2", dys, ws, w_dtype="e4m3")) <= TOL["e4m3"]
    # the 8-bit forward stays close to the bf16 one (quantisation noise only)
    v16, m16 = sste.project_pack(W, float(beta))
    Z16 = sste.linear_fwd(X, v16, m16, O)
    assert rel_err(z_to_f64(Z), z_to_f64(Z16)) <= 0.1
