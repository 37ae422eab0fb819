"""Linears that share their input, evaluated as one wide layer (qalora_forward_shared /
qalora_backward_shared): q/k/v and gate/up.  The oracle runs every linear on its own (Alg. 1
per layer) and the results are concatenated (y, dA, dB) or added (dx): it never sees the wide
layer.  The single-layer entry points of the library give the same y bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2309_14717_amd import synth
from helpers import TOL, dev, record, rel_err

pytestmark = pytest.mark.gpu


def make_parts(d_in, widths, ranks, ss, bits, group, tokens, seed):
    """Per-linear seeded inputs (W, A, B) and a shared x / per-linear dy."""
    parts = []
    for q, (w, r, s) in enumerate(zip(widths, ranks, ss)):
        cfg = synth.LayerConfig(f"p{q}", tokens, d_in, w, bits, group, r, s, seed=seed + 7 * q, outlier_frac=0.004)
        parts.append((cfg, synth.make_inputs(cfg)))
    return parts


def run_case(gpu_api, d_in, widths, ranks, ss, bits, group, tokens, seed, rows=None, keep=False):
    parts = make_parts(d_in, widths, ranks, ss, bits, group, tokens, seed)
    x = parts[0][1]["x"]                                   # the shared input
    dy = np.concatenate([d["dy"] for _, d in parts], axis=1)
    W = np.concatenate([d["W"] for _, d in parts], axis=1)
    desc = gpu_api.make_desc(d_in, sum(widths), bits, group)
    packed, alpha, beta = gpu_api.quantize(desc, dev(W))
    adapters = [(dev(d["A"]), dev(d["B"]), cfg.s) for cfg, d in parts]
    gx, gdy = dev(x, torch.bfloat16), dev(dy, torch.bfloat16)
    if keep:
        y, kept = gpu_api.forward_shared(desc, gx, packed, alpha, beta, adapters, keep=True)
        dx, grads = gpu_api.backward_shared(desc, gdy, None, kept, packed, alpha, beta, adapters)
    else:
        y = gpu_api.forward_shared(desc, gx, packed, alpha, beta, adapters)
        dx, grads = gpu_api.backward_shared(desc, gdy, gx, None, packed, alpha, beta, adapters)
    rows = np.arange(tokens) if rows is None else rows
    sel = torch.from_numpy(rows).cuda()
    y_np, dx_np = y[sel].cpu().numpy(), dx[sel].cpu().numpy()
    errs, col = {}, 0
    dx_ref = 0.0
    for q, (cfg, d) in enumerate(parts):
        codes, al, be = oracle.quantize(d["W"], bits, group)
        # the wide layer's quantization is the concatenation of the per-linear ones
        assert np.array_equal(alpha.cpu().numpy()[:, col:col + cfg.d_out], al)
        assert np.array_equal(beta.cpu().numpy()[:, col:col + cfg.d_out], be)
        ref = oracle.forward(x[rows], codes, al, be, group, d["A"], d["B"], cfg.s)
        errs[f"y{q}"] = rel_err(y_np[:, col:col + cfg.d_out], ref)
        rdx, _, _ = oracle.backward(d["dy"][rows], x[rows], codes, al, be, group, d["A"], d["B"], cfg.s,
                                    want_dAdB=False)
        dx_ref = dx_ref + rdx
        _, rdA, rdB = oracle.backward(d["dy"], x, codes, al, be, group, d["A"], d["B"], cfg.s, want_dx=False)
        errs[f"dA{q}"] = rel_err(grads[q][0].cpu().numpy(), rdA)
        errs[f"dB{q}"] = rel_err(grads[q][1].cpu().numpy(), rdB)
        col += cfg.d_out
    errs["dx"] = rel_err(dx_np, dx_ref)
    return errs, (desc, gx, gdy, packed, alpha, beta, adapters, y, dx, grads, parts)


@pytest.mark.parametrize("keep", [False, True])
@pytest.mark.parametrize("bits,group", [(4, 32), (2, 64), (3, 32)])
def test_shared_small(gpu_api, bits, group, keep):
    errs, st = run_case(gpu_api, 512, (64, 96, 32), (8, 16, 4), (0.5, 2.0, 1.0), bits, group, 130, seed=70,
                        keep=keep)
    record(f"shared small N={bits} g={group} keep={keep}", **errs)
    assert max(errs.values()) <= TOL, errs
    # each part's y equals the single-layer call on that part, bit for bit
    desc, gx, _, _, _, _, adapters, y, _, _, parts = st
    col = 0
    for (cfg, d), (A, B, s) in zip(parts, adapters):
        dq = gpu_api.make_desc(512, cfg.d_out, bits, group, cfg.rank, cfg.s)
        pk, al, be = gpu_api.quantize(dq, dev(d["W"]))
        yq = gpu_api.forward(dq, gx, pk, al, be, A, B)
        assert torch.equal(yq, y[:, col:col + cfg.d_out])
        col += cfg.d_out


def test_shared_rejects_bad_parts(gpu_api):
    d_in = 256
    desc = gpu_api.make_desc(d_in, 96, 4, 32)
    W = torch.randn(d_in, 96, device="cuda") * 0.02
    packed, alpha, beta = gpu_api.quantize(desc, W)
    x = torch.randn(8, d_in, device="cuda").to(torch.bfloat16)
    A = torch.zeros(8, 4, device="cuda")
    with pytest.raises(ValueError):      # widths do not add up
        gpu_api.forward_shared(desc, x, packed, alpha, beta, [(A, torch.zeros(4, 64, device="cuda"), 1.0)])
    with pytest.raises(gpu_api.QaloraError) as e:  # a width that is not a multiple of 32
        gpu_api.forward_shared(desc, x, packed, alpha, beta,
                               [(A, torch.zeros(4, 48, device="cuda"), 1.0), (A, torch.zeros(4, 48, device="cuda"), 1.0)])
    assert e.value.status == gpu_api.EUNSUPPORTED


def test_shared_qkv_full_size(gpu_api):
    """q/k/v of a LLaMA-7B attention block as one 4096 x 12288 layer, 4096 tokens: y and dx on
    sampled token rows, the three dA and dB in full."""
    from test_gpu_fullsize import sample_rows
    rows = sample_rows(4096, extra=3, seed=11)
    errs, _ = run_case(gpu_api, 4096, (4096, 4096, 4096), (64, 64, 64), (0.25, 0.25, 0.25), 4, 32, 4096, seed=80,
                       rows=rows, keep=True)
    record("shared q/k/v 4096 x 3*4096 T=4096", **errs)
    assert max(errs.values()) <= TOL, errs
