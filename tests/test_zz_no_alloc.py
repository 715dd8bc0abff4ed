"""The weight-gradient entry point that allocates nothing (sste_linear_wgrad_noalloc) against
sste_linear_wgrad: same kernels, so the results must be bitwise equal; two calls in a row share the
library's built-in scratch, the second with a smaller problem; problems beyond the scratch are refused."""
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


def _bf16(bits):
    return torch.from_numpy(np.ascontiguousarray(bits.view(np.int16))).cuda().view(torch.bfloat16)


@pytest.mark.parametrize("dtype", ["bf16", "e4m3"])
def test_noalloc_equals_workspace_entry_point_on_two_calls_in_a_row(sste, dtype):
    wl = WL.WORKLOADS[1]
    code = sste.BF16 if dtype == "bf16" else sste.F8E4M3
    # both problems take the pre-pass + packed GEMM + split reduction, i.e. they use every part of the scratch
    shapes = [(4096, 512, 512), (2048, 256, 384)]
    operands = []
    for T, O, I in shapes:
        assert sste.wgrad_workspace_bytes(T, O, I, code) > 0
        dY = _bf16(WL.output_gradient(wl, 0, T=T, O=O)[0])
        X = _bf16(WL.activations(wl, 0, T=T, I=I)[0])
        if dtype == "e4m3":
            dY, _ = sste.cast_fp8(dY, 1e-5, code)
            X, _ = sste.cast_fp8(X, 0.01, code)
        want = sste.linear_wgrad(dY, X, 21, 4, code, 1e-5 if dtype == "e4m3" else 1.0, 0.01 if dtype == "e4m3" else 1.0)
        operands.append((dY, X, want))
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    outs = [torch.full_like(want, 3.0) for _, _, want in operands]
    torch.cuda.synchronize()
    free_mid = torch.cuda.mem_get_info()[0]
    for (dY, X, want), out in zip(operands, outs):                 # back to back on one stream, larger problem first
        sste.linear_wgrad_noalloc(dY, X, 21, 4, out, code, 1e-5 if dtype == "e4m3" else 1.0, 0.01 if dtype == "e4m3" else 1.0)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_mid <= free_before   # the calls took no device memory
    for (dY, X, want), out in zip(operands, outs):
        assert torch.equal(out, want)
    # accumulate, and once more in the opposite order (smaller first)
    for (dY, X, want), out in reversed(list(zip(operands, outs))):
        out.fill_(0.25)
        sste.linear_wgrad_noalloc(dY, X, 21, 4, out, code, 1e-5 if dtype == "e4m3" else 1.0, 0.01 if dtype == "e4m3" else 1.0, accumulate=True)
        assert torch.allclose(out, want + 0.25, rtol=0, atol=1e-6 * float(want.abs().max()) + 1e-7)


def test_noalloc_refuses_what_does_not_fit_and_checks_arguments(sste):
    T, O, I = 16384, 5120, 1280
    assert sste.wgrad_workspace_bytes(T, O, I, sste.BF16) > sste.binding.NOALLOC_SCRATCH_BYTES
    dY = torch.zeros((T, O), dtype=torch.bfloat16, device="cuda")
    X = torch.zeros((T, I), dtype=torch.bfloat16, device="cuda")
    dW = torch.full((O, I), 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(sste.SsteError) as ei:
        sste.linear_wgrad_noalloc(dY, X, 0, 0, dW)
    assert ei.value.status == 6 and "scratch" in str(ei.value)
    assert float(dW.min()) == 7.0                                     # nothing was launched
    with pytest.raises(sste.SsteError) as ei:
        sste.linear_wgrad_noalloc(dY[:100], X[:100], 0, 0, dW)
    assert ei.value.status == 7
    # a small problem that needs no scratch at all
    small = sste.linear_wgrad_noalloc(dY[:64, :8], X[:64, :8].contiguous(), 0, 0, torch.ones((8, 8), dtype=torch.float32, device="cuda"))
    assert float(small.abs().max()) == 0.0
