"""GPU parity at the full benchmark sizes, in the launch configurations bench.py times.

The dense outputs (y, dx) are compared on sampled token rows -- every output row depends on its
own input row only, so the oracle evaluates exactly those rows, over ALL columns (tile-edge rows
0/255/256/... are always in the sample).  The adapter gradients (dA, dB) reduce over all tokens
and are compared in full.  Codes, alpha, beta are compared bit for bit in full."""
import numpy as np
import pytest
import torch

import oracle
from paper_2309_14717_amd import synth
from helpers import TOL, dev, layer_on_gpu, record, rel_err

pytestmark = pytest.mark.gpu


def sample_rows(T, extra=6, seed=0):
    edge = [0, 1, 31, 32, 63, 64, 127, 128, 255, 256, 257, T // 2, T - 257, T - 256, T - 1]
    rng = np.random.default_rng(seed)
    rows = sorted(set([r for r in edge if 0 <= r < T] + rng.integers(0, T, extra).tolist()))
    return np.array(rows)


def check_layer(gpu_api, cfg, rows=None, check_grads=True):
    L = layer_on_gpu(gpu_api, cfg)
    d = L["np"]
    assert np.array_equal(gpu_api.unpack(L["desc"], L["packed"]).cpu().numpy(), L["codes"])
    assert np.array_equal(L["g_alpha"].cpu().numpy().view(np.uint32), L["alpha"].view(np.uint32))
    assert np.array_equal(L["g_beta"].cpu().numpy().view(np.uint32), L["beta"].view(np.uint32))
    rows = sample_rows(cfg.tokens) if rows is None else rows
    y = gpu_api.forward(L["desc"], L["x"], L["packed"], L["g_alpha"], L["g_beta"], L["A"], L["B"])
    ref = oracle.forward(d["x"][rows], L["codes"], L["alpha"], L["beta"], cfg.group, d["A"], d["B"], cfg.s)
    errs = dict(y=rel_err(y[torch.from_numpy(rows).cuda()].cpu().numpy(), ref))
    dx, dA, dB = gpu_api.backward(L["desc"], L["dy"], L["x"], L["packed"], L["g_alpha"], L["g_beta"],
                                  L["A"], L["B"])
    rdx, _, _ = oracle.backward(d["dy"][rows], d["x"][rows], L["codes"], L["alpha"], L["beta"], cfg.group,
                                d["A"], d["B"], cfg.s, want_dAdB=False)
    errs["dx"] = rel_err(dx[torch.from_numpy(rows).cuda()].cpu().numpy(), rdx)
    if check_grads:
        _, rdA, rdB = oracle.backward(d["dy"], d["x"], L["codes"], L["alpha"], L["beta"], cfg.group,
                                      d["A"], d["B"], cfg.s, want_dx=False)
        errs["dA"] = rel_err(dA.cpu().numpy(), rdA)
        errs["dB"] = rel_err(dB.cpu().numpy(), rdB)
    record(f"fullsize {cfg.name} N={cfg.bits} g={cfg.group} T={cfg.tokens}", **errs)
    assert max(errs.values()) <= TOL, errs
    # the pair the benchmark times (pooled activations kept by the forward): the same bits
    w = (L["packed"], L["g_alpha"], L["g_beta"], L["A"], L["B"])
    yk, kept = gpu_api.forward_keep(L["desc"], L["x"], *w)
    gk = gpu_api.backward_kept(L["desc"], L["dy"], kept, *w)
    assert torch.equal(yk, y) and all(torch.equal(p, q) for p, q in zip(gk, (dx, dA, dB)))
    return L


def test_config2_attention_projection(gpu_api):
    L = check_layer(gpu_api, synth.CONFIGS["c2"])
    # the bf16 outputs the benchmark times are the fp32 outputs rounded to nearest even, bit for
    # bit, in both directions, at the full size and on the tile shape of the timed launch
    w = (L["packed"], L["g_alpha"], L["g_beta"], L["A"], L["B"])
    y32 = gpu_api.forward(L["desc"], L["x"], *w)
    y16 = gpu_api.forward(L["desc"], L["x"], *w, out_dtype=torch.bfloat16)
    assert torch.equal(y16, y32.to(torch.bfloat16))
    dx32, dA32, dB32 = gpu_api.backward(L["desc"], L["dy"], L["x"], *w)
    dx16, dA16, dB16 = gpu_api.backward(L["desc"], L["dy"], L["x"], *w, dx_dtype=torch.bfloat16)
    assert torch.equal(dx16, dx32.to(torch.bfloat16))
    assert torch.equal(dA16, dA32) and torch.equal(dB16, dB32)


@pytest.mark.parametrize("name", ["c3_gate", "c3_down"])
def test_config3_mlp_shapes(gpu_api, name):
    check_layer(gpu_api, synth.CONFIGS[name], rows=sample_rows(4096, extra=9, seed=3))


@pytest.mark.parametrize("bits,group", [(2, 32), (3, 32), (4, 32), (2, 64), (4, 64), (2, 128), (3, 128), (4, 128), (3, 64)])
def test_config4_low_bit_sweep(gpu_api, bits, group):
    cfg = synth.CONFIGS["c4"].scaled(bits=bits, group=group)
    L = check_layer(gpu_api, cfg, rows=sample_rows(cfg.tokens, extra=5, seed=bits * 1000 + group))
    # merge, then the post-merge quantized forward against the adapted one (App. B.3)
    d = L["np"]
    rows = np.array([0, 255, 256, cfg.tokens - 1])
    beta_m = gpu_api.merge(L["desc"], L["g_beta"], L["A"], L["B"])
    ref_m = oracle.merge(L["beta"], d["A"], d["B"], cfg.group, cfg.s)
    assert rel_err(beta_m.cpu().numpy(), ref_m) <= 1e-5
    y_m = gpu_api.forward(L["desc"], L["x"], L["packed"], L["g_alpha"], beta_m)
    ref = oracle.forward(d["x"][rows], L["codes"], L["alpha"], L["beta"], cfg.group, d["A"], d["B"], cfg.s)
    err = rel_err(y_m[torch.from_numpy(rows).cuda()].cpu().numpy(), ref)
    record(f"fullsize c4 post-merge N={bits} g={group}", y=err)
    assert err <= TOL


@pytest.mark.parametrize("name", ["c5_up", "c5_down"])
def test_config5_post_merge_inference(gpu_api, name):
    """Merged model, adapter-free forward at T in {1, 4, 16} (streaming path, full oracle) and
    T = 256, 128, 64 (matrix path at its three tile heights, sampled rows)."""
    cfg = synth.CONFIGS[name].scaled(tokens=256)
    L = layer_on_gpu(gpu_api, cfg)
    d = L["np"]
    beta_m = gpu_api.merge(L["desc"], L["g_beta"], L["A"], L["B"])
    ref_beta = oracle.merge(L["beta"], d["A"], d["B"], cfg.group, cfg.s)
    assert rel_err(beta_m.cpu().numpy(), ref_beta) <= 1e-5
    beta_np = beta_m.cpu().numpy()  # what the device will use from here on
    ref16 = oracle.forward(d["x"][:16], L["codes"], L["alpha"], beta_np, cfg.group)
    for T in (1, 4, 16):
        y = gpu_api.forward(L["desc"], L["x"][:T].contiguous(), L["packed"], L["g_alpha"], beta_m)
        err = rel_err(y.cpu().numpy(), ref16[:T])
        record(f"fullsize {name} post-merge T={T}", y=err)
        assert err <= 1e-5  # exact-operand path: only fp32 accumulation order differs
        yb = gpu_api.forward(L["desc"], L["x"][:T].contiguous(), L["packed"], L["g_alpha"], beta_m,
                             out_dtype=torch.bfloat16)
        assert torch.equal(yb, y.to(torch.bfloat16))
    rows = np.array([0, 17, 63, 64, 128, 255])
    y256 = gpu_api.forward(L["desc"], L["x"], L["packed"], L["g_alpha"], beta_m)
    ref = oracle.forward(d["x"][rows], L["codes"], L["alpha"], beta_np, cfg.group)
    err = rel_err(y256[torch.from_numpy(rows).cuda()].cpu().numpy(), ref)
    record(f"fullsize {name} post-merge T=256", y=err)
    assert err <= TOL
    # 64 and 128 tokens: the 64- and 128-row tiles with their own K splits (sampled rows)
    for T in (64, 128):
        r = rows[rows < T]
        yT = gpu_api.forward(L["desc"], L["x"][:T].contiguous(), L["packed"], L["g_alpha"], beta_m)
        err = rel_err(yT[torch.from_numpy(r).cuda()].cpu().numpy(), ref[: len(r)])
        record(f"fullsize {name} post-merge T={T}", y=err)
        assert err <= TOL


@pytest.mark.parametrize("name,bits", [("c5_up", 2), ("c5_up", 3), ("c5_down", 3)])
def test_config5_shapes_low_bit_small_token(gpu_api, name, bits):
    """The c5 shapes at INT2 / INT3: the streaming kernel at T in {1, 4, 8, 16} (one, two and
    four groups of four tokens) against the full oracle."""
    cfg = synth.CONFIGS[name].scaled(tokens=16, bits=bits)
    L = layer_on_gpu(gpu_api, cfg)
    d = L["np"]
    ref16 = oracle.forward(d["x"], L["codes"], L["alpha"], L["beta"], cfg.group)
    for T in (1, 4, 8, 16):
        y = gpu_api.forward(L["desc"], L["x"][:T].contiguous(), L["packed"], L["g_alpha"], L["g_beta"])
        err = rel_err(y.cpu().numpy(), ref16[:T])
        record(f"fullsize {name} INT{bits} small-token T={T}", y=err)
        assert err <= 1e-5


def test_small_token_share_longer_than_one_staged_piece(gpu_api):
    """8448 x 32768: 128 slabs of 256 columns leave two parts of 33 chunks each, one more than a
    block stages of x at a time -- the only way to reach the second-piece path of the two
    streaming kernels with the part count the launch planner picks (T = 3: one-column-per-lane
    kernel, T = 9: sixteen-token kernel).  Seeded codes and factors are uploaded as given (the
    quantizer is not what this test is about)."""
    d_in, d_out, g = 8448, 32768, 32
    rng = np.random.default_rng(77)
    codes = rng.integers(0, 16, size=(d_in, d_out), dtype=np.uint8)
    alpha = (rng.random((d_in // g, d_out), dtype=np.float32) * 0.01 + 0.001).astype(np.float32)
    beta = (-rng.random((d_in // g, d_out), dtype=np.float32) * 0.05).astype(np.float32)
    x = torch.from_numpy(rng.standard_normal((9, d_in)).astype(np.float32)).to(torch.bfloat16)
    x64 = x.float().numpy().astype(np.float64)
    desc = gpu_api.make_desc(d_in, d_out, 4, g)
    packed = gpu_api.pack(desc, dev(codes))
    ga, gb = dev(alpha), dev(beta)
    ref = oracle.forward(x64, codes, alpha, beta, g)
    for T in (3, 9):
        y = gpu_api.forward(desc, x[:T].contiguous().cuda(), packed, ga, gb)
        err = rel_err(y.cpu().numpy(), ref[:T])
        record(f"fullsize two-piece share T={T} {d_in}x{d_out}", y=err)
        assert err <= 1e-5


def _bf16(a):
    """fp64 array -> nearest-even bf16 values, back in fp64 (the block's activations are bf16)."""
    return torch.from_numpy(np.ascontiguousarray(a)).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()


def test_config3_mlp_block_end_to_end(gpu_api):
    """The block bench.py --workload c3 times, as one chain: gate and up on x, SwiGLU, down, and
    back (dx of gate and up added).  The oracle runs the same chain from the same seeded inputs
    -- fp64 linears, the textbook SwiGLU and its derivative in fp64, every activation that the
    block stores in bf16 rounded to bf16 at the same point -- and never sees a device value.
    y and dx on sampled token rows (all columns), the three dA and the three dB in full."""
    import bench

    def run_block(shared):
        """(y, dx, {linear: (dA, dB)}) of one step of the block as bench.py builds it: three
        separate layers, or gate and up as one wide layer sharing x (--shared)."""
        blk = (bench.MlpBlockShared if shared else bench.MlpBlock)(gpu_api, torch, synth, torch.bfloat16)
        dx = blk.step().float().cpu().numpy()
        y = blk.down.y.float().cpu().numpy()
        if shared:
            gr = {"gate": blk.grads[0], "up": blk.grads[1], "down": (blk.down.dA, blk.down.dB)}
        else:
            gr = {n: (l.dA, l.dB) for n, l in (("gate", blk.gate), ("up", blk.up), ("down", blk.down))}
        gr = {n: (a.cpu().numpy(), b.cpu().numpy()) for n, (a, b) in gr.items()}
        torch.cuda.synchronize()
        return y, dx, gr

    results = {"separate": run_block(False)}
    torch.cuda.empty_cache()
    results["shared"] = run_block(True)
    torch.cuda.empty_cache()

    q, host = {}, {}
    for name in ("gate", "up", "down"):
        cfg = synth.CONFIGS["c3_" + name]
        host[name] = synth.make_inputs(cfg)
        q[name] = oracle.quantize(host[name]["W"], cfg.bits, cfg.group)

    def fwd(name, x):
        cfg, d = synth.CONFIGS["c3_" + name], host[name]
        return oracle.forward(x, *q[name], cfg.group, d["A"], d["B"], cfg.s)

    def bwd(name, dy, x, **kw):
        cfg, d = synth.CONFIGS["c3_" + name], host[name]
        return oracle.backward(dy, x, *q[name], cfg.group, d["A"], d["B"], cfg.s, **kw)

    x = host["gate"]["x"].astype(np.float64)            # block input (bf16 values)
    dy = host["down"]["dy"].astype(np.float64)
    g, u = _bf16(fwd("gate", x)), _bf16(fwd("up", x))   # all tokens: dA, dB of gate / up need them
    sig = 1.0 / (1.0 + np.exp(-g))
    h = _bf16(g * sig * u)
    rows = sample_rows(4096, extra=3, seed=9)
    y_ref = _bf16(fwd("down", h[rows]))
    dh, dA_d, dB_d = bwd("down", dy, h)
    dh = _bf16(dh)
    dg = _bf16(dh * u * (sig * (1.0 + g * (1.0 - sig))))
    du = _bf16(dh * g * sig)
    _, dA_g, dB_g = bwd("gate", dg, x, want_dx=False)
    _, dA_u, dB_u = bwd("up", du, x, want_dx=False)
    dx1, _, _ = bwd("gate", dg[rows], x[rows], want_dAdB=False)
    dx2, _, _ = bwd("up", du[rows], x[rows], want_dAdB=False)
    dx_ref = _bf16(_bf16(dx1) + _bf16(dx2))

    all_errs = {}
    for kind, (y_gpu, dx_gpu, grads_gpu) in results.items():
        errs = dict(y=rel_err(y_gpu[rows], y_ref), dx=rel_err(dx_gpu[rows], dx_ref))
        for name, (rA, rB) in (("gate", (dA_g, dB_g)), ("up", (dA_u, dB_u)), ("down", (dA_d, dB_d))):
            errs["dA_" + name] = rel_err(grads_gpu[name][0], rA)
            errs["dB_" + name] = rel_err(grads_gpu[name][1], rB)
        record(f"fullsize c3 block end to end ({kind})", **errs)
        all_errs[kind] = errs
    # Bars of the chain.  Each contraction on the path to an output may be off by TOL of its own
    # maximum (the bar of a single layer), and each activation the block stores in bf16 by one
    # rounding, 2^-9 relative; both carry through the linear stages that follow at most
    # undiminished, so the bar of an output is the sum over its path (measured values sit at a
    # third to a half of it, the independent errors adding in quadrature):
    #   y      : gate|up, down                      2 contractions, roundings g|u, h, y
    #   dx     : down bwd, gate|up fwd, gate|up bwd  3 contractions, roundings g|u, dh, dg|du, dx1|dx2, sum
    #   dA, dB of gate, up : down bwd, gate|up fwd, own products   3 contractions, roundings g|u, dh, dg|du
    #   dA, dB of down     : gate|up fwd (through h), own products 2 contractions, roundings g|u, h
    r = 2.0 ** -9
    bars = dict(y=2 * TOL + 3 * r, dx=3 * TOL + 5 * r, dA_gate=3 * TOL + 3 * r, dB_gate=3 * TOL + 3 * r,
                dA_up=3 * TOL + 3 * r, dB_up=3 * TOL + 3 * r, dA_down=2 * TOL + 2 * r, dB_down=2 * TOL + 2 * r)
    # (the shared form rounds dx once instead of dx1, dx2 and their sum: the same bar covers it)
    for kind, errs in all_errs.items():
        assert all(errs[k] <= bars[k] for k in bars), (kind, errs, bars)
