"""Seeded random layer shapes through every entry point against the oracle: code width, group
size, number of groups, output width, token count and rank are drawn together, so that tile
edges, ragged tails, the streaming / matrix-path switch and the rank padding meet in
combinations the hand-picked cases do not list.  (A sweep of several hundred such draws was run
while the kernels were written; these are a fixed sample of it.)"""
import numpy as np
import pytest
import torch

import oracle
from paper_2309_14717_amd import synth
from helpers import TOL, layer_on_gpu, record, rel_err

pytestmark = pytest.mark.gpu

TOKENS = [1, 2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 31, 63, 64, 65, 100, 129, 255, 256, 257, 300, 513]
RANKS = [0, 1, 2, 3, 8, 16, 31, 64, 100, 128]


def draw(case):
    rng = np.random.default_rng(7000 + case)
    bits = int(rng.choice([2, 3, 4]))
    group = int({4: 8, 2: 16, 3: 32}[bits] * rng.choice([1, 2, 4, 8]))
    L = int(rng.integers(1, 40)) if case % 3 else int(rng.integers(40, 160))
    d_out = 8 * int(rng.integers(1, 120)) if case % 5 else 8 * int(rng.integers(120, 400))
    return synth.LayerConfig(f"rnd{case}", int(rng.choice(TOKENS)), group * L, d_out, bits, group,
                             int(rng.choice(RANKS)), float(rng.choice([0.25, 1.0, 2.0])), seed=7000 + case)


@pytest.mark.parametrize("case", range(32))
def test_random_layer(gpu_api, case):
    cfg = draw(case)
    L = layer_on_gpu(gpu_api, cfg)
    d = L["np"]
    assert np.array_equal(gpu_api.unpack(L["desc"], L["packed"]).cpu().numpy(), L["codes"])
    assert np.array_equal(L["g_alpha"].cpu().numpy().view(np.uint32), L["alpha"].view(np.uint32))
    assert np.array_equal(L["g_beta"].cpu().numpy().view(np.uint32), L["beta"].view(np.uint32))
    A, B = L.get("A"), L.get("B")
    hA, hB = (d["A"], d["B"]) if cfg.rank else (None, None)
    errs = {}
    y = gpu_api.forward(L["desc"], L["x"], L["packed"], L["g_alpha"], L["g_beta"], A, B)
    ref = oracle.forward(d["x"], L["codes"], L["alpha"], L["beta"], cfg.group, hA, hB, cfg.s)
    errs["y"] = rel_err(y.cpu().numpy(), ref)
    yb = gpu_api.forward(L["desc"], L["x"], L["packed"], L["g_alpha"], L["g_beta"], A, B, out_dtype=torch.bfloat16)
    assert torch.equal(yb, y.to(torch.bfloat16))
    dx, dA, dB = gpu_api.backward(L["desc"], L["dy"], L["x"], L["packed"], L["g_alpha"], L["g_beta"], A, B)
    rdx, rdA, rdB = oracle.backward(d["dy"], d["x"], L["codes"], L["alpha"], L["beta"], cfg.group, hA, hB, cfg.s)
    errs["dx"] = rel_err(dx.cpu().numpy(), rdx)
    if cfg.rank:
        errs["dA"] = rel_err(dA.cpu().numpy(), rdA)
        errs["dB"] = rel_err(dB.cpu().numpy(), rdB)
        # the pair that keeps the pooled activations instead of x: the same bits
        yk, kept = gpu_api.forward_keep(L["desc"], L["x"], L["packed"], L["g_alpha"], L["g_beta"], A, B)
        gk = gpu_api.backward_kept(L["desc"], L["dy"], kept, L["packed"], L["g_alpha"], L["g_beta"], A, B)
        assert torch.equal(yk, y) and all(torch.equal(p, q) for p, q in zip(gk, (dx, dA, dB)))
        beta_m = gpu_api.merge(L["desc"], L["g_beta"], A, B)
        assert rel_err(beta_m.cpu().numpy(), oracle.merge(L["beta"], hA, hB, cfg.group, cfg.s)) <= 1e-5
        y_m = gpu_api.forward(L["desc"], L["x"], L["packed"], L["g_alpha"], beta_m)
        errs["y_merged"] = rel_err(y_m.cpu().numpy(), ref)
    fac = gpu_api.pack_factors16(L["desc"], L["g_alpha"], L["g_beta"])
    a16 = L["alpha"].astype(np.float16).astype(np.float32)
    b16 = L["beta"].astype(np.float16).astype(np.float32)
    y16 = gpu_api.forward_factors16(L["desc"], L["x"], L["packed"], fac)
    errs["y_factors16"] = rel_err(y16.cpu().numpy(), oracle.forward(d["x"], L["codes"], a16, b16, cfg.group))
    record(f"random N={cfg.bits} g={cfg.group} {cfg.d_in}x{cfg.d_out} T={cfg.tokens} r={cfg.rank}", **errs)
    assert max(errs.values()) <= TOL, errs


@pytest.mark.parametrize("case", range(16))
def test_random_small_token_layer(gpu_api, case):
    """The streaming kernels on drawn shapes: up to sixteen tokens, every code width, 1 to 70
    chunks of input rows, output widths that end anywhere inside a slab; fp32 and 16-bit
    factors; exact operands, so the bar is 1e-5; reruns bit-identical."""
    from helpers import dev
    rng = np.random.default_rng(9000 + case)
    bits, group = int(rng.choice([2, 3, 4])), int(rng.choice([32, 64, 128]))
    d_in, d_out, T = 128 * int(rng.integers(1, 70)), 8 * int(rng.integers(1, 1500)), int(rng.integers(1, 17))
    L = d_in // group
    codes = rng.integers(0, 1 << bits, size=(d_in, d_out), dtype=np.uint8)
    alpha = (rng.random((L, d_out), dtype=np.float32) * 0.01 + 0.001).astype(np.float32)
    beta = (-rng.random((L, d_out), dtype=np.float32) * 0.05).astype(np.float32)
    x = torch.from_numpy(rng.standard_normal((T, d_in)).astype(np.float32)).to(torch.bfloat16)
    x64 = x.float().numpy().astype(np.float64)
    desc = gpu_api.make_desc(d_in, d_out, bits, group)
    packed, ga, gb, xd = gpu_api.pack(desc, dev(codes)), dev(alpha), dev(beta), x.cuda()
    y = gpu_api.forward(desc, xd, packed, ga, gb)
    e32 = rel_err(y.cpu().numpy(), oracle.forward(x64, codes, alpha, beta, group))
    assert torch.equal(y, gpu_api.forward(desc, xd, packed, ga, gb))
    fac = gpu_api.pack_factors16(desc, ga, gb)
    a16, b16 = (v.astype(np.float16).astype(np.float32) for v in (alpha, beta))
    y16 = gpu_api.forward_factors16(desc, xd, packed, fac)
    e16 = rel_err(y16.cpu().numpy(), oracle.forward(x64, codes, a16, b16, group))
    record(f"random small-token N={bits} g={group} {d_in}x{d_out} T={T}", y=e32, y_factors16=e16)
    assert max(e32, e16) <= 1e-5
