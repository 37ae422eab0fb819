"""The library under HIP graph capture: forward (dense and small-token kernels) and backward are
captured once and replayed several times with new inputs written in place, with eager work and
device synchronisations between the replays; every replay must equal the eager call on the same
inputs bit for bit (the launches are deterministic), and the eager call is held to the oracle.

The small-token kernel is the delicate one: its cross-block flags carry a per-launch value that
a captured launch repeats on every replay, so the consumer clears each flag it has seen."""
import numpy as np
import pytest
import torch

import oracle
from paper_2309_14717_amd import synth
from helpers import TOL, layer_on_gpu, rel_err

pytestmark = pytest.mark.gpu


def fresh(like, seed, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(like.shape, generator=g) * scale).to(like.dtype).cuda()


# the decode kernel, the sixteen-token kernel (one and two groups of sixteen), and the decode kernel's several-token-group form
@pytest.mark.parametrize("tokens,bits", [(4, 4), (9, 4), (24, 4), (3, 2), (11, 3)])
def test_graph_replay_small_token_forward(gpu_api, tokens, bits):
    # 2 slabs x 16 parts: fifteen flags per slab are raised and consumed in every launch
    cfg = synth.LayerConfig("graph_st", tokens, 2048, 512, bits, 32, 8, 0.5, seed=31)
    L = layer_on_gpu(gpu_api, cfg)
    x = L["x"].clone()
    y = torch.empty((cfg.tokens, cfg.d_out), dtype=torch.float32, device="cuda")
    ws = torch.empty(gpu_api.workspace_bytes(L["desc"], cfg.tokens, gpu_api.OP_FORWARD), dtype=torch.uint8,
                     device="cuda")
    args = (L["desc"], x, L["packed"], L["g_alpha"], L["g_beta"])
    gpu_api.forward(*args, ws=ws, y=y)  # eager warm-up (also sets the kernel's LDS attribute)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        gpu_api.forward(*args, ws=ws, y=y)
    for rep in range(4):
        x.copy_(fresh(x, 100 + rep))
        y.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = y.clone()
        want = gpu_api.forward(*args)  # eager, own workspace and output
        torch.cuda.synchronize()
        assert torch.equal(got, want), f"replay {rep}"
        ref = oracle.forward(x.float().cpu().numpy().astype(np.float64), L["codes"], L["alpha"], L["beta"],
                             cfg.group)
        assert rel_err(want.cpu().numpy(), ref) <= 1e-5


@pytest.mark.parametrize("keep", [False, True], ids=["plain", "kept"])
def test_graph_replay_forward_backward(gpu_api, keep):
    """keep: the pair in which the forward leaves the pooled activations and the backward reads
    them instead of x (the buffer between the two is part of the captured graph's state)."""
    cfg = synth.LayerConfig("graph_fb", 200, 384, 520, 4, 32, 16, 0.5, seed=32)
    L = layer_on_gpu(gpu_api, cfg)
    d = L["desc"]
    x, dy = L["x"].clone(), L["dy"].clone()
    y = torch.empty((cfg.tokens, cfg.d_out), dtype=torch.float32, device="cuda")
    dx = torch.empty((cfg.tokens, cfg.d_in), dtype=torch.float32, device="cuda")
    dA, dB = torch.zeros_like(L["A"]), torch.zeros_like(L["B"])
    ws_f = torch.empty(gpu_api.workspace_bytes(d, cfg.tokens, gpu_api.OP_FORWARD), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(gpu_api.workspace_bytes(d, cfg.tokens, gpu_api.OP_BACKWARD), dtype=torch.uint8, device="cuda")
    w = (L["packed"], L["g_alpha"], L["g_beta"], L["A"], L["B"])

    kept = torch.empty(gpu_api.kept_bytes(d, cfg.tokens), dtype=torch.uint8, device="cuda")

    def both():
        if keep:
            gpu_api.forward_keep(d, x, *w, ws=ws_f, y=y, kept=kept)
            gpu_api.backward_kept(d, dy, kept, *w, dA=dA, dB=dB, ws=ws_b, dx=dx)
        else:
            gpu_api.forward(d, x, *w, ws=ws_f, y=y)
            gpu_api.backward(d, dy, x, *w, dA=dA, dB=dB, ws=ws_b, dx=dx)

    both()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        both()
    for rep in range(3):
        x.copy_(fresh(x, 200 + rep))
        dy.copy_(fresh(dy, 300 + rep))
        for t in (y, dx, dA, dB):
            t.fill_(float("nan"))
        kept.fill_(0xff)
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (y, dx, dA, dB)]
        ey = gpu_api.forward(d, x, *w)
        edx, edA, edB = gpu_api.backward(d, dy, x, *w)
        torch.cuda.synchronize()
        for name, g, e in zip(("y", "dx", "dA", "dB"), got, (ey, edx, edA, edB)):
            assert torch.equal(g, e), f"replay {rep}: {name}"
        x64 = x.float().cpu().numpy().astype(np.float64)
        dy64 = dy.float().cpu().numpy().astype(np.float64)
        ry = oracle.forward(x64, L["codes"], L["alpha"], L["beta"], cfg.group, L["np"]["A"], L["np"]["B"], cfg.s)
        rdx, rdA, rdB = oracle.backward(dy64, x64, L["codes"], L["alpha"], L["beta"], cfg.group,
                                        L["np"]["A"], L["np"]["B"], cfg.s)
        for name, e, r in zip(("y", "dx", "dA", "dB"), (ey, edx, edA, edB), (ry, rdx, rdA, rdB)):
            assert rel_err(e.cpu().numpy(), r) <= TOL, name


@pytest.mark.parametrize("tokens", [2, 64])
def test_graph_replay_deployed_forward(gpu_api, tokens):
    """The deployed layer under capture: the decode kernel on the stream (2 tokens: flags and
    partial sums in the workspace) and the dense kernel on the prepared factor words (64)."""
    cfg = synth.LayerConfig("graph_dep", tokens, 2048, 512, 4, 32, 8, 0.5, seed=33)
    L = layer_on_gpu(gpu_api, cfg)
    d = L["desc"]
    beta_m = gpu_api.merge(d, L["g_beta"], L["A"], L["B"])
    dep = gpu_api.deploy(d, L["packed"], L["g_alpha"], beta_m)
    x = L["x"].clone()
    y = torch.empty((tokens, cfg.d_out), dtype=torch.float32, device="cuda")
    ws = torch.empty(gpu_api.workspace_bytes(d, tokens, gpu_api.OP_FORWARD), dtype=torch.uint8, device="cuda")
    gpu_api.forward_deployed(d, x, dep, packed=L["packed"], ws=ws, y=y)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        gpu_api.forward_deployed(d, x, dep, packed=L["packed"], ws=ws, y=y)
    for rep in range(3):
        x.copy_(fresh(x, 400 + rep))
        y.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = y.clone()
        want = gpu_api.forward(d, x, L["packed"], L["g_alpha"], beta_m)   # eager, the plain entry point
        torch.cuda.synchronize()
        assert torch.equal(got, want), f"replay {rep}"
        ref = oracle.forward(x.float().cpu().numpy().astype(np.float64), L["codes"], L["alpha"],
                             beta_m.cpu().numpy(), cfg.group)
        assert rel_err(want.cpu().numpy(), ref) <= (1e-5 if tokens <= 4 else TOL)


def test_graph_replay_shared_layers(gpu_api):
    """Two linears sharing x as one wide layer, forward (keeping the pooled activations) and
    backward captured together; every replay equals the eager pair bit for bit, and the eager
    pair is held to the per-linear oracle."""
    T, d_in, widths, ranks, ss, g = 96, 512, (256, 160), (16, 8), (0.5, 0.25), 32
    parts = []
    for q, (w, r, s) in enumerate(zip(widths, ranks, ss)):
        cfg = synth.LayerConfig(f"gs{q}", T, d_in, w, 4, g, r, s, seed=70 + q)
        parts.append((cfg, synth.make_inputs(cfg)))
    W = np.concatenate([d["W"] for _, d in parts], axis=1)
    desc = gpu_api.make_desc(d_in, sum(widths), 4, g)
    to = lambda a, dt=torch.float32: torch.from_numpy(np.ascontiguousarray(a)).to(dt).cuda()
    packed, alpha, beta = gpu_api.quantize(desc, to(W))
    adapters = [(to(d["A"]), to(d["B"]), cfg.s) for cfg, d in parts]
    x = to(parts[0][1]["x"], torch.bfloat16)
    dy = to(np.concatenate([d["dy"] for _, d in parts], axis=1), torch.bfloat16)
    y = torch.empty((T, desc.d_out), dtype=torch.float32, device="cuda")
    dx = torch.empty((T, d_in), dtype=torch.float32, device="cuda")
    grads = [(torch.zeros_like(A), torch.zeros_like(B)) for A, B, _ in adapters]
    w = (packed, alpha, beta, adapters)
    _, kept = gpu_api.forward_shared(desc, x, *w, keep=True, y=y)
    lib, arr = gpu_api.load(), gpu_api._parts(desc, adapters, x.device)
    import ctypes
    ws_f = torch.empty(lib.qalora_shared_workspace_bytes(ctypes.byref(desc), T, gpu_api.OP_FORWARD, 2, arr),
                       dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(lib.qalora_shared_workspace_bytes(ctypes.byref(desc), T, gpu_api.OP_BACKWARD, 2, arr),
                       dtype=torch.uint8, device="cuda")

    def both():
        gpu_api.forward_shared(desc, x, *w, keep=True, ws=ws_f, y=y, kept=kept)
        gpu_api.backward_shared(desc, dy, None, kept, *w, grads=grads, ws=ws_b, dx=dx)

    both()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        both()
    for rep in range(3):
        x.copy_(fresh(x, 500 + rep))
        dy.copy_(fresh(dy, 600 + rep))
        for t in (y, dx, *[t for pair in grads for t in pair]):
            t.fill_(float("nan"))
        kept.fill_(0xff)
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (y, dx, *[t for pair in grads for t in pair])]
        ey = gpu_api.forward_shared(desc, x, *w)
        edx, eg = gpu_api.backward_shared(desc, dy, x, None, *w)
        torch.cuda.synchronize()
        for i, (g_, e_) in enumerate(zip(got, (ey, edx, *[t for pair in eg for t in pair]))):
            assert torch.equal(g_, e_), f"replay {rep}: output {i}"
    # the last eager pair against the oracle, linear by linear
    x64 = x.float().cpu().numpy().astype(np.float64)
    dy64 = dy.float().cpu().numpy().astype(np.float64)
    col, dx_ref = 0, 0.0
    for q, (cfg, d) in enumerate(parts):
        codes, al, be = oracle.quantize(d["W"], 4, g)
        ref = oracle.forward(x64, codes, al, be, g, d["A"], d["B"], cfg.s)
        assert rel_err(ey.cpu().numpy()[:, col:col + cfg.d_out], ref) <= TOL
        rdx, rdA, rdB = oracle.backward(dy64[:, col:col + cfg.d_out], x64, codes, al, be, g, d["A"], d["B"], cfg.s)
        dx_ref = dx_ref + rdx
        assert rel_err(eg[q][0].cpu().numpy(), rdA) <= TOL and rel_err(eg[q][1].cpu().numpy(), rdB) <= TOL
        col += cfg.d_out
    assert rel_err(edx.cpu().numpy(), dx_ref) <= TOL
