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
