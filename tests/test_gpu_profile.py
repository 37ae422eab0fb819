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


def test_block_time_line(gpu_api):
    """Every block of the armed launch reports start <= end of its K loop <= end and an XCD id;
    blocks beyond the buffer's capacity are left alone; the result is unchanged."""
    cfg = synth.LayerConfig("prof", 512, 1024, 1024, 4, 32, 16, 0.5, seed=41)
    L = layer_on_gpu(gpu_api, cfg)
    w = (L["packed"], L["g_alpha"], L["g_beta"], L["A"], L["B"])
    y_plain = gpu_api.forward(L["desc"], L["x"], *w)
    t = gpu_api.KernelTimer(0, 1)
    t.arm()
    t.arm_blocks(capacity=4)      # the launch has 8 tiles of 256 x 256: four of them report
    y = gpu_api.forward(L["desc"], L["x"], *w)
    torch.cuda.synchronize()
    assert torch.equal(y, y_plain)
    c = t.block_times.cpu().numpy()
    assert (c[:, 0] > 0).all() and (c[:, 0] <= c[:, 1]).all() and (c[:, 1] <= c[:, 2]).all()
    assert ((c[:, 3] >= 0) & (c[:, 3] < 8)).all()
    tl = t.block_timeline()
    assert tl["blocks"] == 4 and tl["end_us_min_med_max"][2] < 1e4
    t.close()
    lib = gpu_api.load()
    assert lib.qalora_profile_arm_blocks(3, None, 0) == gpu_api.EINVAL
    assert lib.qalora_profile_arm_blocks(0, t.block_times.data_ptr(), 0) == gpu_api.EINVAL
    assert lib.qalora_profile_arm_blocks(0, None, 0) == gpu_api.OK
