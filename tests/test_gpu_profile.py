"""The measurement aid of the C ABI (what bench.py's roofline numbers come from): armed events
bracket exactly the dense contraction kernel, the armed kernel reports the clock it ran at, and
arming changes no result."""
import pytest
import torch

from paper_2309_14717_amd import synth
from helpers import layer_on_gpu

pytestmark = pytest.mark.gpu


def test_armed_events_and_clock_probe(gpu_api):
    cfg = synth.LayerConfig("prof", 512, 1024, 1024, 4, 32, 16, 0.5, seed=41)
    L = layer_on_gpu(gpu_api, cfg)
    w = (L["packed"], L["g_alpha"], L["g_beta"], L["A"], L["B"])
    y_plain = gpu_api.forward(L["desc"], L["x"], *w)
    dx_plain, dA_plain, dB_plain = gpu_api.backward(L["desc"], L["dy"], L["x"], *w)
    n = 3
    timers = [gpu_api.KernelTimer(d, n) for d in (0, 1)]
    for _ in range(n):
        for t in timers:
            t.arm()
        y = gpu_api.forward(L["desc"], L["x"], *w)
        dx, dA, dB = gpu_api.backward(L["desc"], L["dy"], L["x"], *w)
    torch.cuda.synchronize()
    assert torch.equal(y, y_plain) and torch.equal(dx, dx_plain)
    assert torch.equal(dA, dA_plain) and torch.equal(dB, dB_plain)
    for t in timers:
        ms = t.elapsed_ms()
        assert len(ms) == n and all(0.0 < v < 50.0 for v in ms)
        ghz = t.shader_clock_ghz()
        assert ghz is not None and 0.3 < ghz < 3.0   # a real clock, nominal 2.4 GHz
        t.close()


def test_arm_rejects_bad_direction(gpu_api):
    import ctypes
    lib = gpu_api.load()
    assert lib.qalora_profile_arm(2, None, None) == gpu_api.EINVAL
    assert lib.qalora_profile_arm_clock(-1, None) == gpu_api.EINVAL
    khz = ctypes.c_int()
    assert lib.qalora_profile_wall_clock_khz(ctypes.byref(khz)) == gpu_api.OK and khz.value > 0
