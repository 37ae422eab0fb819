"""GPU check of the benchmark-harness glue (SwiGLU elementwise forward and backward).  This is not
part of the paper's method, so the reference is the textbook definition written out here in fp64:
silu(v) = v / (1 + exp(-v)); the backward is checked both against the analytic derivative and
against central finite differences of that same definition."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def silu64(v):
    return v / (1.0 + np.exp(-v))


def bf16_inputs(n, seed):
    g = torch.Generator().manual_seed(seed)
    gate = (torch.randn(n, generator=g) * 2.0).to(torch.bfloat16)
    up = torch.randn(n, generator=g).to(torch.bfloat16)
    dh = torch.randn(n, generator=g).to(torch.bfloat16)
    return gate, up, dh


@pytest.mark.parametrize("n", [8, 4096 + 8, 1 << 20])
def test_swiglu_matches_definition(gpu_api, n):
    gate, up, dh = bf16_inputs(n, seed=5)
    g64, u64, d64 = (t.double().numpy() for t in (gate, up, dh))
    h = gpu_api.swiglu_forward(gate.cuda(), up.cuda()).float().cpu().double().numpy()
    dg, du = gpu_api.swiglu_backward(dh.cuda(), gate.cuda(), up.cuda())
    dg, du = dg.float().cpu().double().numpy(), du.float().cpu().double().numpy()

    ref_h = silu64(g64) * u64
    eps = 1e-6
    dsilu_fd = (silu64(g64 + eps) - silu64(g64 - eps)) / (2 * eps)
    ref_dg = d64 * u64 * dsilu_fd
    ref_du = d64 * silu64(g64)
    # one bf16 rounding of the result (2^-9 relative) plus fp32 evaluation noise
    for got, ref in ((h, ref_h), (dg, ref_dg), (du, ref_du)):
        assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-6)


def test_swiglu_rejects_ragged_length(gpu_api):
    gate, up, _ = bf16_inputs(16, seed=1)
    with pytest.raises(Exception):
        gpu_api.swiglu_forward(gate.cuda()[:12], up.cuda()[:12])


def test_swiglu_wide_layout_matches_separate_tensors(gpu_api):
    """[gate | up] in one tensor (the output of a wide gate/up layer): same values as the
    two-tensor form, bit for bit."""
    rows, cols = 37, 264
    gate, up, dh = bf16_inputs(rows * cols, seed=9)
    gate, up, dh = (t.view(rows, cols).cuda() for t in (gate, up, dh))
    gu = torch.cat([gate, up], dim=1).contiguous()
    h = gpu_api.swiglu_forward_strided(gu, cols)
    assert torch.equal(h, gpu_api.swiglu_forward(gate.contiguous(), up.contiguous()))
    dgu = gpu_api.swiglu_backward_strided(dh.contiguous(), gu, cols)
    dg, du = gpu_api.swiglu_backward(dh.contiguous(), gate.contiguous(), up.contiguous())
    assert torch.equal(dgu[:, :cols], dg) and torch.equal(dgu[:, cols:], du)
