"""GPU parity of the fused AdamW step (Sec. 4.1's recipe) against the fp64 oracle: the adapter
tensors of a decoder layer's seven linears, several steps with the state carried on the device,
the clip active and inactive, ragged sizes, gradients consumed in place."""
import numpy as np
import pytest
import torch

import oracle
from helpers import record, rel_err

pytestmark = pytest.mark.gpu


def layer_shapes(d=512, ff=1408, g=32, r=16):
    """A and B of q, k, v, o, gate, up, down at a reduced LLaMA-like width."""
    shapes = []
    for d_in, d_out in ((d, d),) * 4 + ((d, ff), (d, ff), (ff, d)):
        shapes += [(d_in // g, r), (r, d_out)]
    return shapes


@pytest.mark.parametrize("max_norm,wd,gscale", [(0.3, 0.0, 1.0), (0.3, 0.01, 1e-4), (0.0, 0.1, 1.0)])
def test_adamw_steps_match_oracle(gpu_api, max_norm, wd, gscale):
    rng = np.random.default_rng(11)
    shapes = layer_shapes() + [(5,), (4095,), (4097,), (4100,), (8192,)]  # ragged sizes around a block of 4096
    hp = gpu_api.AdamW(2e-3, 0.9, 0.999, 1e-8, wd, max_norm)
    # the hyper-parameters are inputs: the oracle gets the values the fp32 struct holds
    lr, b1, b2, eps, wd64, mn64 = (float(x) for x in (hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay,
                                                       hp.max_grad_norm))
    p_h = [rng.standard_normal(s).astype(np.float32) * 0.02 for s in shapes]
    m_h = [np.zeros(s, np.float32) for s in shapes]
    v_h = [np.zeros(s, np.float32) for s in shapes]
    p_d = [torch.from_numpy(x).cuda() for x in p_h]
    m_d = [torch.zeros_like(x) for x in p_d]
    v_d = [torch.zeros_like(x) for x in p_d]
    norm_d = torch.zeros(4, dtype=torch.float32, device="cuda")
    worst = dict(p=0.0, m=0.0, v=0.0)
    for step in range(1, 5):
        g_h = [(rng.standard_normal(s) * gscale).astype(np.float32) for s in shapes]
        g_d = [torch.from_numpy(x).cuda() for x in g_h]
        gpu_api.adamw_step(hp, step, p_d, g_d, m_d, v_d, zero_grads=(step % 2 == 0), grad_norm=norm_d)
        rp, rm, rv, rn = oracle.adamw_step(p_h, g_h, m_h, v_h, step, lr, b1, b2, eps, wd64, mn64)
        assert abs(float(norm_d[0]) - rn) <= 1e-6 * rn
        for i in range(len(shapes)):
            worst["p"] = max(worst["p"], rel_err(p_d[i].cpu().numpy(), rp[i]))
            worst["m"] = max(worst["m"], rel_err(m_d[i].cpu().numpy(), rm[i]))
            worst["v"] = max(worst["v"], rel_err(v_d[i].cpu().numpy(), rv[i]))
            if step % 2 == 0:
                assert not g_d[i].any()          # consumed: ready for an accumulating backward
            else:
                assert np.array_equal(g_d[i].cpu().numpy(), g_h[i])
        # the device state (fp32) is what both sides continue from
        p_h = [x.cpu().numpy() for x in p_d]
        m_h = [x.cpu().numpy() for x in m_d]
        v_h = [x.cpu().numpy() for x in v_d]
    record(f"adamw max_norm={max_norm} wd={wd} gscale={gscale}", **worst)
    assert max(worst.values()) <= 2e-6


def test_adamw_without_clip_needs_no_workspace_and_reruns_identically(gpu_api):
    rng = np.random.default_rng(12)
    shapes = layer_shapes()
    hp = gpu_api.AdamW(1e-3, 0.9, 0.95, 1e-8, 0.0, 0.0)
    runs = []
    for _ in range(2):
        r2 = np.random.default_rng(13)
        p = [torch.from_numpy(r2.standard_normal(s).astype(np.float32)).cuda() for s in shapes]
        g = [torch.from_numpy(r2.standard_normal(s).astype(np.float32)).cuda() for s in shapes]
        m = [torch.zeros_like(x) for x in p]
        v = [torch.zeros_like(x) for x in p]
        gpu_api.adamw_step(hp, 1, p, g, m, v, ws=torch.empty(16, dtype=torch.uint8, device="cuda"))
        runs.append([x.clone() for x in p])
    assert all(torch.equal(a, b) for a, b in zip(*runs))
    # with the clip (block sums, fixed order) reruns are bit-identical too
    hp2 = gpu_api.AdamW(1e-3, 0.9, 0.95, 1e-8, 0.0, 0.3)
    runs = []
    for _ in range(2):
        r2 = np.random.default_rng(14)
        p = [torch.from_numpy(r2.standard_normal(s).astype(np.float32)).cuda() for s in shapes]
        g = [torch.from_numpy(r2.standard_normal(s).astype(np.float32)).cuda() for s in shapes]
        m = [torch.zeros_like(x) for x in p]
        v = [torch.zeros_like(x) for x in p]
        gpu_api.adamw_step(hp2, 3, p, g, m, v)
        runs.append([x.clone() for x in p])
    assert all(torch.equal(a, b) for a, b in zip(*runs))
