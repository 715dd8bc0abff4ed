"""The hot path under HIP graph capture: project + pack, forward and weight gradient of a layer (and of an 8-bit
layer with its output cast and largest magnitude) are recorded once on a capture stream and replayed; every
replay must reproduce the eagerly computed results bit for bit.  The library launches only kernels on the
caller's stream (values that must start at zero are cleared by small fill kernels, never by memset nodes), so a
caller may capture it; the replays below are separated by eager work and synchronisations on purpose."""
import numpy as np
import pytest
import torch

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


@pytest.mark.parametrize("dtype,T,O,I", [("bf16", 512, 256, 1024),      # small: the fused weight-gradient kernel
                                          ("bf16", 4096, 512, 768),      # estimator pre-pass + packed GEMM + reduction
                                          ("e4m3", 4096, 528, 768)])     # 8-bit operands, e4m3 output with its maximum
def test_layer_step_replays_bit_exact(sste, dtype, T, O, I):
    wl = WL.WORKLOADS[1]
    fp8 = dtype == "e4m3"
    dt = sste.F8E4M3 if fp8 else sste.BF16
    W = bf16_dev(WL.weight_bits(wl, 0, O=O, I=I))
    Xb = bf16_dev(WL.activations(wl, 0, T=T, I=I)[0])
    dYb = bf16_dev(WL.output_gradient(wl, 0, T=T, O=O)[0])
    beta, ws = 1.4830322, (0.0009 if fp8 else 1.0)
    if fp8:
        xs, dys = 0.011, 1.1e-5
        X, _ = sste.cast_fp8(Xb, xs, dt)
        dY, _ = sste.cast_fp8(dYb, dys, dt)
    else:
        xs, dys, X, dY = 1.0, 1.0, Xb, dYb
    vals, meta = sste.packed_buffers(O, I, dt, "cuda")
    Z = torch.empty((T, O), dtype=torch.uint8 if fp8 else torch.bfloat16, device="cuda")
    amax = torch.empty(1, dtype=torch.float32, device="cuda")
    dW = torch.empty((O, I), dtype=torch.float32, device="cuda")
    ws_bytes = sste.wgrad_workspace_bytes(T, O, I, dt)
    wsb = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")

    def step():
        sste.project_pack(W, beta, dt, ws, vals=vals, meta=meta)
        if fp8:
            sste.linear_fwd_ex(X, vals, meta, O, dt, xs, ws, sste.F8E4M3, 0.02, Z=Z, amax_out=amax)
        else:
            sste.linear_fwd_ex(X, vals, meta, O, dt, xs, ws, Z=Z, amax_out=amax)
        sste.linear_wgrad(dY, X, 7, 3, dt, dys, xs, dW=dW, workspace=wsb)

    step()
    torch.cuda.synchronize()
    want = [t.clone() for t in (vals, meta, Z, amax, dW)]
    assert float(amax[0]) > 0

    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=side):
        step()
    for rep in range(4):
        for t in (vals, meta, Z, dW, wsb):       # eager work between the replays: the outputs are wiped
            t.view(torch.uint8).fill_(0x5A)
        amax.fill_(-1.0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for name, got, ref in zip(("vals", "meta", "Z", "amax", "dW"), (vals, meta, Z, amax, dW), want):
            assert torch.equal(got.view(torch.uint8), ref.view(torch.uint8)), (rep, name)
