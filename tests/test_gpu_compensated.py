"""Error-compensated code selection on the GPU (qalora_quantize_compensated) against the oracle:
the operation order is part of the definition, so codes, alpha and beta must agree bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2309_14717_amd import synth
from helpers import dev
from test_oracle_compensated import hessian, hessian_error

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("bits,g,d_in,d_out", [(4, 32, 384, 40), (3, 64, 256, 16), (2, 128, 512, 72), (4, 16, 208, 24)])
def test_compensated_bit_exact(gpu_api, bits, g, d_in, d_out):
    W = synth.make_inputs(synth.LayerConfig("t", 1, d_in, d_out, bits, g, 1, seed=40 + bits), want=("W",))["W"]
    H, U = hessian(d_in, 4 * d_in, seed=bits)
    U32 = np.ascontiguousarray(U.astype(np.float32))
    desc = gpu_api.make_desc(d_in, d_out, bits, g)
    if gpu_api.check_desc(desc) != gpu_api.OK:
        pytest.skip("group size outside the packed format for this code width")
    packed, alpha, beta = gpu_api.quantize_compensated(desc, dev(W), dev(U32))
    codes = gpu_api.unpack(desc, packed).cpu().numpy()
    c, a, b = oracle.quantize_compensated(W, U32, bits, g, block=128)
    assert np.array_equal(codes, c)
    assert np.array_equal(alpha.cpu().numpy().view(np.uint32), a.view(np.uint32))
    assert np.array_equal(beta.cpu().numpy().view(np.uint32), b.view(np.uint32))
    # and it does what it is for: less output error under H than plain rounding
    e_rtn = hessian_error(W, *oracle.quantize(W, bits, g), g, H)
    assert hessian_error(W, codes, a, b, g, H) < e_rtn


def test_compensated_many_blocks_and_rerun(gpu_api):
    """A layer of sixteen lazy row blocks and 128 column blocks (all compute units busy, two
    block generations), bit for bit against the oracle, and twice: the row lanes of a column
    live in different wavefronts, so an ordering mistake between them would show as a result
    that differs between runs or from the oracle."""
    bits, g, d_in, d_out = 4, 32, 2048, 2048
    W = synth.make_inputs(synth.LayerConfig("t", 1, d_in, d_out, bits, g, 1, seed=61), want=("W",))["W"]
    _, U = hessian(d_in, 2 * d_in, seed=9)
    U32 = np.ascontiguousarray(U.astype(np.float32))
    desc = gpu_api.make_desc(d_in, d_out, bits, g)
    Wd, Ud = dev(W), dev(U32)
    p1, a1, b1 = gpu_api.quantize_compensated(desc, Wd, Ud)
    p2, a2, b2 = gpu_api.quantize_compensated(desc, Wd, Ud)
    assert torch.equal(p1, p2) and torch.equal(a1, a2) and torch.equal(b1, b2)
    c, a, b = oracle.quantize_compensated(W, U32, bits, g, block=128)
    assert np.array_equal(gpu_api.unpack(desc, p1).cpu().numpy(), c)
    assert np.array_equal(a1.cpu().numpy().view(np.uint32), a.view(np.uint32))
    assert np.array_equal(b1.cpu().numpy().view(np.uint32), b.view(np.uint32))


def test_compensated_identity_is_plain_quantize(gpu_api):
    d_in, d_out = 256, 64
    W = synth.make_inputs(synth.LayerConfig("t", 1, d_in, d_out, 4, 32, 1, seed=50), want=("W",))["W"]
    desc = gpu_api.make_desc(d_in, d_out, 4, 32)
    p1, a1, b1 = gpu_api.quantize_compensated(desc, dev(W), torch.eye(d_in, device="cuda"))
    p0, a0, b0 = gpu_api.quantize(desc, dev(W))
    assert torch.equal(p1, p0) and torch.equal(a1, a0) and torch.equal(b1, b0)


def test_compensated_layer_runs_on_the_result(gpu_api):
    """The triple feeds the layer like any other: forward parity against the oracle on it."""
    d_in, d_out, T = 512, 128, 33
    cfg = synth.LayerConfig("t", T, d_in, d_out, 4, 32, 8, 0.5, seed=51)
    d = synth.make_inputs(cfg)
    _, U = hessian(d_in, 2048, seed=6)
    U32 = np.ascontiguousarray(U.astype(np.float32))
    desc = gpu_api.make_desc(d_in, d_out, 4, 32, 8, 0.5)
    packed, alpha, beta = gpu_api.quantize_compensated(desc, dev(d["W"]), dev(U32))
    c, a, b = oracle.quantize_compensated(d["W"], U32, 4, 32)
    y = gpu_api.forward(desc, dev(d["x"], torch.bfloat16), packed, alpha, beta, dev(d["A"]), dev(d["B"]))
    ref = oracle.forward(d["x"], c, a, b, 32, d["A"], d["B"], 0.5)
    assert np.abs(y.cpu().numpy() - ref).max() <= 2e-3 * np.abs(ref).max()


def test_compensated_rejects_groups_that_straddle_blocks(gpu_api):
    desc = gpu_api.make_desc(384, 64, 4, 96)
    with pytest.raises(gpu_api.QaloraError) as e:
        gpu_api.quantize_compensated(desc, torch.zeros(384, 64, device="cuda"), torch.eye(384, device="cuda"))
    assert e.value.status == gpu_api.EUNSUPPORTED
