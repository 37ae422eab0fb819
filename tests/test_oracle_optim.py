"""Pins of the oracle's optimiser step (Sec. 4.1's recipe: AdamW, a maximum gradient norm of
0.3, a constant learning rate) against things that are not the oracle: torch's own AdamW and
gradient clipping on the CPU over several steps, a step worked by hand, and the limits every
form of Adam has (first step moves each weight by about lr; a zero gradient leaves m, v to
decay and the weight to its decay alone)."""
import numpy as np
import torch

import oracle


def run_torch(params, grads_per_step, lr, betas, eps, wd, max_norm):
    ps = [torch.nn.Parameter(torch.tensor(p, dtype=torch.float64)) for p in params]
    opt = torch.optim.AdamW(ps, lr=lr, betas=betas, eps=eps, weight_decay=wd)
    norms = []
    for grads in grads_per_step:
        for p, g in zip(ps, grads):
            p.grad = torch.tensor(g, dtype=torch.float64)
        if max_norm > 0:
            norms.append(float(torch.nn.utils.clip_grad_norm_(ps, max_norm)))
        opt.step()
    st = [opt.state[p] for p in ps]
    return ([p.detach().numpy() for p in ps], [s["exp_avg"].numpy() for s in st],
            [s["exp_avg_sq"].numpy() for s in st], norms)


def test_against_library_adamw_over_several_steps():
    rng = np.random.default_rng(0)
    shapes = [(32, 8), (8, 96), (5,), (3, 7)]
    for max_norm, wd, gscale in ((0.3, 0.0, 1.0), (0.3, 0.01, 1e-3), (0.0, 0.1, 1.0)):
        params = [rng.standard_normal(s).astype(np.float32) * 0.02 for s in shapes]
        steps = [[(rng.standard_normal(s) * gscale).astype(np.float32) for s in shapes] for _ in range(5)]
        lr, betas, eps = 2e-3, (0.9, 0.95), 1e-8
        tp, tm, tv, tn = run_torch(params, steps, lr, betas, eps, wd, max_norm)
        p = [x.astype(np.float64) for x in params]
        m = [np.zeros(s) for s in shapes]
        v = [np.zeros(s) for s in shapes]
        norms = []
        for t, grads in enumerate(steps, start=1):
            # the oracle takes fp32 state; feed it values that fp32 holds exactly
            p32, m32, v32 = ([a.astype(np.float32) for a in xs] for xs in (p, m, v))
            p, m, v, n = oracle.adamw_step(p32, grads, m32, v32, t, lr, betas[0], betas[1], eps, wd, max_norm)
            norms.append(n)
        # state passes through fp32 between the oracle's steps, torch's stays in fp64
        for a, b in zip(p, tp):
            np.testing.assert_allclose(a, b, rtol=0, atol=5e-7 * max(1.0, np.abs(b).max()))
        for a, b in zip(m, tm):
            np.testing.assert_allclose(a, b, rtol=0, atol=1e-6 * np.abs(b).max())
        for a, b in zip(v, tv):
            np.testing.assert_allclose(a, b, rtol=0, atol=1e-6 * np.abs(b).max())
        if max_norm > 0:
            np.testing.assert_allclose(norms, tn, rtol=1e-12)


def test_one_step_by_hand():
    """p = 1, g = 2, clip inactive, step 1: m = 0.2, v = 0.004, m_hat = 2, v_hat = 4,
    p' = 1 (1 - lr wd) - lr * 2 / (2 + eps)."""
    lr, wd, eps = 0.1, 0.5, 1e-8
    p, m, v, n = oracle.adamw_step([np.array([1.0], np.float32)], [np.array([2.0], np.float32)],
                                   [np.zeros(1, np.float32)], [np.zeros(1, np.float32)], 1, lr, 0.9, 0.999,
                                   eps, wd, 0.0)
    assert n == 2.0
    np.testing.assert_allclose(m[0], [0.2], rtol=1e-15)
    np.testing.assert_allclose(v[0], [0.004], rtol=1e-12)
    np.testing.assert_allclose(p[0], [1.0 * (1 - lr * wd) - lr * 2.0 / (2.0 + eps)], rtol=1e-12)


def test_clip_rescales_all_tensors_by_one_factor():
    g = [np.array([3.0, 0.0], np.float32), np.array([[4.0]], np.float32)]  # joint norm 5
    assert oracle.grad_norm(g) == 5.0
    z = [np.zeros_like(x) for x in g]
    _, m, _, n = oracle.adamw_step(z, g, z, z, 1, 1e-3, 0.9, 0.999, 1e-8, 0.0, 0.3)
    clip = 0.3 / (5.0 + 1e-6)
    np.testing.assert_allclose(m[0], 0.1 * clip * g[0].astype(np.float64), rtol=1e-12)
    np.testing.assert_allclose(m[1], 0.1 * clip * g[1].astype(np.float64), rtol=1e-12)
    # below the maximum nothing is rescaled
    small = [x * np.float32(0.01) for x in g]
    _, m2, _, _ = oracle.adamw_step(z, small, z, z, 1, 1e-3, 0.9, 0.999, 1e-8, 0.0, 0.3)
    np.testing.assert_allclose(m2[0], 0.1 * small[0].astype(np.float64), rtol=1e-12)


def test_limits():
    rng = np.random.default_rng(3)
    p0 = rng.standard_normal(64).astype(np.float32)
    g = (rng.standard_normal(64) + 3.0).astype(np.float32)
    z = np.zeros(64, np.float32)
    # first step without decay: every weight moves by lr * sign(g) (to eps / |g|)
    p, _, _, _ = oracle.adamw_step([p0], [g], [z], [z], 1, 1e-2, 0.9, 0.999, 1e-8, 0.0, 0.0)
    np.testing.assert_allclose(p[0] - p0, -1e-2 * np.sign(g), rtol=1e-6)
    # zero gradient: moments decay by their betas, the weight by lr * wd and the old momentum only
    m0 = rng.standard_normal(64).astype(np.float32)
    v0 = np.abs(rng.standard_normal(64)).astype(np.float32)
    p, m, v, n = oracle.adamw_step([p0], [z], [m0], [v0], 7, 1e-2, 0.9, 0.999, 1e-8, 0.1, 0.3)
    assert n == 0.0
    np.testing.assert_allclose(m[0], 0.9 * m0.astype(np.float64), rtol=1e-15)
    np.testing.assert_allclose(v[0], 0.999 * v0.astype(np.float64), rtol=1e-15)
