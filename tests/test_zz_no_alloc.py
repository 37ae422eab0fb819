"""The entry point that allocates nothing (qalora_forward_noalloc): its output against
qalora_forward's -- same kernels, so bit for bit -- and against the oracle, on two calls in a
row that share the library's built-in scratch, the second with a smaller input."""
import numpy as np
import pytest
import torch

import oracle
from paper_2309_14717_amd import synth
from helpers import layer_on_gpu, record, rel_err

pytestmark = pytest.mark.gpu


def test_noalloc_matches_forward_twice(gpu_api):
    big = synth.LayerConfig("na_big", 16, 4096, 5128, 4, 32, 8, 0.5, seed=31)     # ragged last slab
    small = synth.LayerConfig("na_small", 3, 1024, 520, 4, 64, 8, 0.5, seed=32)
    for cfg in (big, small):  # the second call finds the first call's flags and partial sums
        L = layer_on_gpu(gpu_api, cfg)
        ref = oracle.forward(L["np"]["x"], L["codes"], L["alpha"], L["beta"], cfg.group)
        for odt in (torch.float32, torch.bfloat16):
            y_ws = gpu_api.forward(L["desc"], L["x"], L["packed"], L["g_alpha"], L["g_beta"], out_dtype=odt)
            y_na = gpu_api.forward_noalloc(L["desc"], L["x"], L["packed"], L["g_alpha"], L["g_beta"],
                                           out_dtype=odt)
            assert torch.equal(y_na, y_ws)
        err = rel_err(gpu_api.forward_noalloc(L["desc"], L["x"], L["packed"], L["g_alpha"],
                                              L["g_beta"]).cpu().numpy(), ref)
        record(f"noalloc {cfg.name} T={cfg.tokens}", y=err)
        assert err <= 1e-5


def test_noalloc_rejects_what_its_scratch_cannot_hold(gpu_api):
    cfg = synth.LayerConfig("na_rej", 17, 1024, 512, 4, 32, 8, 0.5, seed=33)
    L = layer_on_gpu(gpu_api, cfg)
    with pytest.raises(gpu_api.QaloraError) as e:
        gpu_api.forward_noalloc(L["desc"], L["x"], L["packed"], L["g_alpha"], L["g_beta"])
    assert e.value.status == gpu_api.EUNSUPPORTED
    # a shape outside the streaming kernels (group 16) is refused too, not routed elsewhere
    cfg = synth.LayerConfig("na_rej2", 4, 1024, 512, 4, 16, 8, 0.5, seed=34)
    L = layer_on_gpu(gpu_api, cfg)
    with pytest.raises(gpu_api.QaloraError) as e:
        gpu_api.forward_noalloc(L["desc"], L["x"], L["packed"], L["g_alpha"], L["g_beta"])
    assert e.value.status == gpu_api.EUNSUPPORTED
