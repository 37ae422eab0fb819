"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol
the header declares, sizes are consistent, and argument errors are reported before any launch."""
import ctypes
import os
import re

import pytest

from paper_2309_14717_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(api.LIB_PATH):
        from paper_2309_14717_amd import build
        build.build()
    return api.load()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "qalora.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qalora_[a-z0-9_]+)\s*\(", text)))


def test_exports_every_declared_symbol(lib):
    names = declared_functions()
    assert set(names) == set(api.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings(lib):
    for st in (0, -1, -2, -3, -4, -5):
        assert api.status_string(st).startswith("QALORA_")
    assert "unknown" in api.status_string(-99)


def test_desc_validation(lib):
    ok = api.make_desc(4096, 4096, 4, 32, 64, 0.25)
    assert api.check_desc(ok) == api.OK
    assert api.check_desc(api.make_desc(4096, 4096, 5, 32)) == api.EINVAL       # bits
    assert api.check_desc(api.make_desc(4096, 4096, 4, 0)) == api.EINVAL        # group
    assert api.check_desc(api.make_desc(4100, 4096, 4, 32)) == api.EINVAL       # L must divide D_in
    assert api.check_desc(api.make_desc(4096, 4096, 4, 32, -1)) == api.EINVAL   # rank
    assert api.check_desc(api.make_desc(0, 4096, 4, 32)) == api.EINVAL
    assert api.check_desc(api.make_desc(36, 64, 4, 4)) == api.EUNSUPPORTED      # group % 8
    assert api.check_desc(api.make_desc(64, 64, 3, 16)) == api.EUNSUPPORTED     # INT3 wants g % 32
    assert api.check_desc(api.make_desc(64, 60, 4, 32)) == api.EUNSUPPORTED     # d_out % 8
    assert api.check_desc(api.make_desc(64, 64, 4, 32, 512)) == api.EUNSUPPORTED
    assert lib.qalora_check_desc(None) == api.EINVAL


def test_packed_and_workspace_sizes(lib):
    for bits, per_weight_bits in ((4, 4), (3, 3), (2, 2)):
        d = api.make_desc(4096, 11008, bits, 128, 64, 0.25)
        assert api.packed_bytes(d) == 4096 * 11008 * per_weight_bits // 8
    d = api.make_desc(4096, 4096, 4, 32, 64, 0.25)
    assert api.workspace_bytes(d, 4096, api.OP_QUANTIZE) == 0
    assert api.workspace_bytes(d, 4096, api.OP_MERGE) == 0
    f = api.workspace_bytes(d, 4096, api.OP_FORWARD)
    b = api.workspace_bytes(d, 4096, api.OP_BACKWARD)
    # forward: the fp16 copy of x and one factor word per (group, column); backward: more
    assert f >= 4096 * 4096 * 2 + 128 * 4096 * 4 and b > f
    assert api.workspace_bytes(d, 4096, 99) == 0
    d0 = api.make_desc(4096, 4096, 4, 32, 0, 0.0)
    # the adapter is folded into the factor words, so the forward needs the same room without one
    assert api.workspace_bytes(d0, 4096, api.OP_FORWARD) == f
    assert 4096 * 8 <= api.workspace_bytes(d0, 4096, api.OP_BACKWARD) < b
    assert api.packed_bytes(api.make_desc(4096, 4096, 7, 32)) == 0


def test_argument_errors_are_caught_before_launch(lib):
    """Fake (never dereferenced) pointer values: every call below must return on the host."""
    d = api.make_desc(1024, 1024, 4, 32, 16, 2.0)
    P = ctypes.c_void_p
    good, odd = 0x10000, 0x10004
    ref = ctypes.byref(d)
    assert lib.qalora_forward(ref, 64, P(good), P(good), P(good), P(good), None, None, None, 0, None, 0, None) == api.EINVAL
    assert lib.qalora_forward(ref, 0, P(good), P(good), P(good), P(good), None, None, P(good), 0, None, 0, None) == api.EINVAL
    assert lib.qalora_forward(ref, 64, P(good), P(good), P(good), P(good), P(good), None, P(good), 0, None, 0, None) == api.EINVAL
    assert lib.qalora_forward(ref, 64, P(good), P(good), P(good), P(good), None, None, P(good), 7, None, 0, None) == api.EINVAL
    assert lib.qalora_forward(ref, 64, P(odd), P(good), P(good), P(good), None, None, P(good), 0, None, 0, None) == api.EALIGN
    assert lib.qalora_forward(ref, 64, P(good), P(good), P(good), P(good), None, None, P(good), 0, None, 0, None) == api.EWORKSPACE
    assert lib.qalora_forward(ref, 64, P(good), P(good), P(good), P(good), P(good), P(good), P(good), 0, None, 0, None) == api.EWORKSPACE
    assert lib.qalora_forward(ref, 64, P(good), P(good), P(good), P(good), P(good), P(good), P(good), 0, P(good), 64, None) == api.EWORKSPACE
    assert lib.qalora_backward(ref, 64, None, P(good), P(good), P(good), P(good), None, None, P(good), 0, None, None, 0, None, 0, None) == api.EINVAL
    assert lib.qalora_backward(ref, 64, P(good), P(good), P(good), P(good), P(good), P(good), P(good), P(good), 0, None, P(good), 0, P(good), 1 << 40, None) == api.EINVAL
    assert lib.qalora_backward(ref, 64, P(good), P(good), P(good), P(good), P(good), P(good), P(good), P(good), 0, P(good), P(good), 2, P(good), 1 << 40, None) == api.EINVAL
    assert lib.qalora_backward(ref, 64, P(good), P(good), P(good), P(good), P(good), P(good), P(good), P(good), 0, P(good), P(good), 0, P(good), 16, None) == api.EWORKSPACE
    assert lib.qalora_backward(ref, 64, P(good), P(good), P(good), P(odd), P(good), None, None, P(good), 0, None, None, 0, None, 0, None) == api.EALIGN
    assert lib.qalora_quantize(ref, None, P(good), P(good), P(good), None, 0, None) == api.EINVAL
    assert lib.qalora_quantize(ref, P(good), P(good), P(odd), P(good), None, 0, None) == api.EALIGN
    assert lib.qalora_merge(ref, P(good), None, P(good), P(good), None) == api.EINVAL
    assert lib.qalora_beta_from_zero_point(ref, P(good), None, P(good), None) == api.EINVAL
    assert lib.qalora_beta_from_zero_point(ref, P(good), P(odd), P(good), None) == api.EALIGN
    assert lib.qalora_zero_point_from_beta(ref, None, P(good), P(good), None) == api.EINVAL
    assert lib.qalora_zero_point_from_beta(ref, P(good), P(good), P(odd), None) == api.EALIGN
    assert lib.qalora_pack_factors16(ref, P(good), None, P(good), None) == api.EINVAL
    assert lib.qalora_pack_factors16(ref, P(good), P(good), P(odd), None) == api.EALIGN
    assert lib.qalora_forward_factors16(ref, 0, P(good), P(good), P(good), P(good), 0, P(good), 1 << 30, None) == api.EINVAL
    assert lib.qalora_forward_factors16(ref, 4, P(good), P(good), None, P(good), 0, P(good), 1 << 30, None) == api.EINVAL
    assert lib.qalora_forward_factors16(ref, 4, P(good), P(good), P(good), P(good), 7, P(good), 1 << 30, None) == api.EINVAL
    assert lib.qalora_forward_factors16(ref, 4, P(odd), P(good), P(good), P(good), 0, P(good), 1 << 30, None) == api.EALIGN
    assert lib.qalora_forward_factors16(ref, 4, P(good), P(good), P(good), P(good), 0, P(good), 16, None) == api.EWORKSPACE
    assert lib.qalora_forward_factors16(ref, 400, P(good), P(good), P(good), P(good), 0, None, 0, None) == api.EWORKSPACE
    # the matrix path of the 16-bit-factor forward needs room for the expanded factors on top
    fwd = lib.qalora_workspace_bytes(ref, 400, api.OP_FORWARD)
    assert lib.qalora_workspace_bytes(ref, 400, api.OP_FORWARD_FACTORS16) >= 2 * (1024 // 32) * 1024 * 4
    assert lib.qalora_workspace_bytes(ref, 4, api.OP_FORWARD_FACTORS16) > 0 and fwd > 0
    # the kept-activation pair: the buffer is required, and only an adapter has anything to keep
    assert lib.qalora_kept_bytes(ref, 64) >= 64 * 32 * 4 + 64 * 16 * 4
    assert lib.qalora_kept_bytes(ref, 0) == 0
    assert lib.qalora_kept_bytes(ctypes.byref(api.make_desc(1024, 1024, 4, 32, 0, 0.0)), 64) == 0
    assert lib.qalora_forward_keep(ref, 64, P(good), P(good), P(good), P(good), P(good), P(good), P(good), 0, None, P(good), 1 << 30, None) == api.EINVAL
    assert lib.qalora_forward_keep(ref, 64, P(good), P(good), P(good), P(good), None, None, P(good), 0, P(good), P(good), 1 << 30, None) == api.EINVAL
    assert lib.qalora_forward_keep(ref, 64, P(good), P(good), P(good), P(good), P(good), P(good), P(good), 0, P(odd), P(good), 1 << 30, None) == api.EALIGN
    assert lib.qalora_forward_keep(ref, 64, P(good), P(good), P(good), P(good), P(good), P(good), P(good), 0, P(good), P(good), 16, None) == api.EWORKSPACE
    assert lib.qalora_backward_kept(ref, 64, P(good), None, P(good), P(good), P(good), P(good), P(good), P(good), 0, P(good), P(good), 0, P(good), 1 << 40, None) == api.EINVAL
    assert lib.qalora_backward_kept(ref, 64, P(good), P(good), P(good), P(good), P(good), None, None, P(good), 0, None, None, 0, P(good), 1 << 40, None) == api.EINVAL
    assert lib.qalora_backward_kept(ref, 64, P(good), P(odd), P(good), P(good), P(good), P(good), P(good), P(good), 0, P(good), P(good), 0, P(good), 1 << 40, None) == api.EALIGN
    assert lib.qalora_backward_kept(ref, 64, P(good), P(good), P(good), P(good), P(good), P(good), P(good), P(good), 0, P(good), P(good), 0, P(good), 16, None) == api.EWORKSPACE
    assert lib.qalora_unpack(ref, None, P(good), None) == api.EINVAL
    assert lib.qalora_pack(ref, P(good), P(odd), None) == api.EALIGN
    bad = api.make_desc(1024, 1004, 4, 32, 16, 2.0)
    assert lib.qalora_forward(ctypes.byref(bad), 64, P(good), P(good), P(good), P(good), None, None, P(good), 0, None, 0, None) == api.EUNSUPPORTED
    # operands beyond the kernels' 32-bit byte offsets are refused, not wrapped around
    huge = api.make_desc(65536, 65536, 4, 32, 0, 0.0)
    big_ws = 1 << 44
    assert lib.qalora_forward(ctypes.byref(huge), 1 << 16, P(good), P(good), P(good), P(good), None, None, P(good), 0, P(good), big_ws, None) == api.EUNSUPPORTED
    assert lib.qalora_backward(ctypes.byref(huge), 1 << 16, P(good), P(good), P(good), P(good), P(good), None, None, P(good), 0, None, None, 0, P(good), big_ws, None) == api.EUNSUPPORTED


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(api, "_lib", None)
    monkeypatch.setattr(api, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        api.load()


def test_adamw_argument_errors(lib):
    """The fused optimiser step checks its tensor table on the host (fake pointers, no launch)."""
    P = ctypes.c_void_p
    hp = api.AdamW(2e-5, 0.9, 0.999, 1e-8, 0.0, 0.3)
    good, odd = 0x10000, 0x10004
    arr = lambda v, n=2: (ctypes.c_void_p * n)(*([v] * n))
    numel = (ctypes.c_size_t * 2)(4096, 1000)
    assert lib.qalora_adamw_workspace_bytes(2, numel) >= 2 * 4
    assert lib.qalora_adamw_workspace_bytes(0, numel) == 0
    assert lib.qalora_adamw_workspace_bytes(33, numel) == 0
    call = lambda **kw: lib.qalora_adamw_step(
        kw.get("hp", ctypes.byref(hp)), kw.get("step", 1), kw.get("n", 2), kw.get("p", arr(good)), arr(good),
        kw.get("m", arr(good)), arr(good), kw.get("numel", numel), 0, None, kw.get("ws", P(good)),
        kw.get("ws_bytes", 1 << 20), None)
    assert call(hp=None) == api.EINVAL
    assert call(step=0) == api.EINVAL
    assert call(n=0) == api.EINVAL
    assert call(n=33) == api.EINVAL
    assert call(p=arr(None)) == api.EINVAL
    assert call(m=arr(odd)) == api.EALIGN
    assert call(numel=(ctypes.c_size_t * 2)(4096, 0)) == api.EINVAL
    assert call(ws=None, ws_bytes=0) == api.EWORKSPACE   # clipping needs the block sums
    assert call(ws_bytes=4) == api.EWORKSPACE
    bad = api.AdamW(2e-5, 1.0, 0.999, 1e-8, 0.0, 0.3)
    assert call(hp=ctypes.byref(bad)) == api.EINVAL
