"""Thin Python binding of the C-ABI library (include/qalora.h).

Argument marshalling only: every step of the layer runs in the HIP kernels behind the
C ABI.  PyTorch supplies device memory and the stream.  There is no fallback: if the
shared library has not been built, or a call returns an error status, this raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqalora_hip.so")

OK, EINVAL, EALIGN, EWORKSPACE, EUNSUPPORTED, EHIP = 0, -1, -2, -3, -4, -5
F32, BF16 = 0, 1
OP_QUANTIZE, OP_FORWARD, OP_BACKWARD, OP_MERGE, OP_FORWARD_FACTORS16, OP_QUANTIZE_COMPENSATED = 0, 1, 2, 3, 4, 5

EXPORTS = (
    "qalora_status_string", "qalora_check_desc", "qalora_packed_bytes", "qalora_workspace_bytes",
    "qalora_quantize", "qalora_unpack", "qalora_pack", "qalora_forward", "qalora_backward",
    "qalora_merge", "qalora_profile_arm", "qalora_profile_event_create",
    "qalora_profile_event_elapsed_ms", "qalora_profile_event_destroy", "qalora_profile_copy",
    "qalora_swiglu_forward", "qalora_swiglu_backward",
    "qalora_profile_arm_clock", "qalora_profile_arm_blocks", "qalora_profile_wall_clock_khz",
    "qalora_beta_from_zero_point", "qalora_zero_point_from_beta",
    "qalora_pack_factors16", "qalora_forward_factors16",
    "qalora_adamw_workspace_bytes", "qalora_adamw_step",
    "qalora_kept_bytes", "qalora_forward_keep", "qalora_backward_kept",
    "qalora_forward_noalloc", "qalora_profile_mfma_probe",
    "qalora_deployed_bytes", "qalora_deploy", "qalora_forward_deployed",
    "qalora_shared_kept_bytes", "qalora_shared_workspace_bytes", "qalora_forward_shared",
    "qalora_quantize_compensated",
    "qalora_backward_shared", "qalora_swiglu_forward_wide", "qalora_swiglu_backward_wide",
)


class Desc(ctypes.Structure):
    """Mirror of ``qalora_desc``."""
    _fields_ = [("d_in", ctypes.c_int32), ("d_out", ctypes.c_int32), ("bits", ctypes.c_int32),
                ("group", ctypes.c_int32), ("rank", ctypes.c_int32), ("s", ctypes.c_float)]


class QaloraError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)}")


_lib = None


def load() -> ctypes.CDLL:
    """Load the in-tree shared library; fail loudly when it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} not found: build the HIP library first "
            "(python -m paper_2309_14717_amd.build); there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    vp, cp, i, sz = ctypes.c_void_p, ctypes.POINTER(Desc), ctypes.c_int, ctypes.c_size_t
    lib.qalora_status_string.restype = ctypes.c_char_p
    lib.qalora_status_string.argtypes = [i]
    lib.qalora_check_desc.argtypes = [cp]
    lib.qalora_packed_bytes.restype = sz
    lib.qalora_packed_bytes.argtypes = [cp]
    lib.qalora_workspace_bytes.restype = sz
    lib.qalora_workspace_bytes.argtypes = [cp, i, i]
    lib.qalora_quantize.argtypes = [cp, vp, vp, vp, vp, vp, sz, vp]
    lib.qalora_quantize_compensated.argtypes = [cp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.qalora_unpack.argtypes = [cp, vp, vp, vp]
    lib.qalora_pack.argtypes = [cp, vp, vp, vp]
    lib.qalora_forward.argtypes = [cp, i, vp, vp, vp, vp, vp, vp, vp, i, vp, sz, vp]
    lib.qalora_backward.argtypes = [cp, i, vp, vp, vp, vp, vp, vp, vp, vp, i, vp, vp, i, vp, sz, vp]
    lib.qalora_merge.argtypes = [cp, vp, vp, vp, vp, vp]
    lib.qalora_shared_kept_bytes.restype = sz
    lib.qalora_shared_kept_bytes.argtypes = [cp, i, i, vp]
    lib.qalora_shared_workspace_bytes.restype = sz
    lib.qalora_shared_workspace_bytes.argtypes = [cp, i, i, i, vp]
    lib.qalora_forward_shared.argtypes = [cp, i, vp, vp, vp, vp, i, vp, vp, i, vp, vp, sz, vp]
    lib.qalora_backward_shared.argtypes = [cp, i, vp, vp, vp, vp, vp, vp, i, vp, vp, i, i, vp, sz, vp]
    lib.qalora_swiglu_forward_wide.argtypes = [vp, vp, sz, sz, vp]
    lib.qalora_swiglu_backward_wide.argtypes = [vp, vp, vp, sz, sz, vp]
    lib.qalora_deployed_bytes.restype = sz
    lib.qalora_deployed_bytes.argtypes = [cp]
    lib.qalora_deploy.argtypes = [cp, vp, vp, vp, vp, vp]
    lib.qalora_forward_deployed.argtypes = [cp, i, vp, vp, vp, vp, i, vp, sz, vp]
    lib.qalora_profile_mfma_probe.argtypes = [i, i, i, i, i, vp, vp, vp]
    lib.qalora_forward_noalloc.argtypes = [cp, i, vp, vp, vp, vp, vp, i, vp]
    lib.qalora_kept_bytes.restype = sz
    lib.qalora_kept_bytes.argtypes = [cp, i]
    lib.qalora_forward_keep.argtypes = [cp, i, vp, vp, vp, vp, vp, vp, vp, i, vp, vp, sz, vp]
    lib.qalora_backward_kept.argtypes = [cp, i, vp, vp, vp, vp, vp, vp, vp, vp, i, vp, vp, i, vp, sz, vp]
    lib.qalora_profile_arm.argtypes = [i, vp, vp]
    lib.qalora_profile_event_create.argtypes = [ctypes.POINTER(vp)]
    lib.qalora_profile_event_elapsed_ms.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_float)]
    lib.qalora_profile_event_destroy.argtypes = [vp]
    lib.qalora_profile_copy.argtypes = [vp, vp, sz, vp]
    lib.qalora_swiglu_forward.argtypes = [vp, vp, vp, sz, vp]
    lib.qalora_profile_arm_clock.argtypes = [ctypes.c_int, vp]
    lib.qalora_profile_arm_blocks.argtypes = [ctypes.c_int, vp, ctypes.c_int]
    lib.qalora_profile_wall_clock_khz.argtypes = [ctypes.POINTER(ctypes.c_int)]
    lib.qalora_swiglu_backward.argtypes = [vp, vp, vp, vp, vp, sz, vp]
    lib.qalora_pack_factors16.argtypes = [cp, vp, vp, vp, vp]
    lib.qalora_forward_factors16.argtypes = [cp, i, vp, vp, vp, vp, i, vp, sz, vp]
    lib.qalora_adamw_workspace_bytes.restype = sz
    lib.qalora_adamw_workspace_bytes.argtypes = [i, vp]
    lib.qalora_adamw_step.argtypes = [vp, i, i, vp, vp, vp, vp, vp, i, vp, vp, sz, vp]
    lib.qalora_beta_from_zero_point.argtypes = [cp, vp, vp, vp, vp]
    lib.qalora_zero_point_from_beta.argtypes = [cp, vp, vp, vp, vp]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().qalora_status_string(int(status)).decode()


def make_desc(d_in, d_out, bits=4, group=32, rank=0, s=0.0) -> Desc:
    return Desc(int(d_in), int(d_out), int(bits), int(group), int(rank), float(s))


def check_desc(desc: Desc) -> int:
    return int(load().qalora_check_desc(ctypes.byref(desc)))


def packed_bytes(desc: Desc) -> int:
    return int(load().qalora_packed_bytes(ctypes.byref(desc)))


def workspace_bytes(desc: Desc, tokens: int, op: int) -> int:
    return int(load().qalora_workspace_bytes(ctypes.byref(desc), int(tokens), int(op)))


def _p(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc, where):
    if rc != OK:
        raise QaloraError(int(rc), where)


def _workspace(desc, tokens, op, ws, device="cuda"):
    # a caller-provided workspace is passed through as it is (the library checks its size)
    if ws is None:
        ws = torch.empty(max(workspace_bytes(desc, tokens, op), 16), dtype=torch.uint8, device=device)
    else:
        _need(ws, "ws", device=device)
    return ws, ws.numel() * ws.element_size()


def _need(t, name, dtype=None, shape=None, nbytes=None, device=None, optional=False):
    """The C ABI sees raw pointers only: a tensor of the wrong size, type or device would become
    an out-of-bounds device access there, so every operand is checked here first."""
    if t is None:
        if optional:
            return
        raise ValueError(f"{name}: missing")
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise ValueError(f"{name}: must be a device tensor")
    if device is not None and t.device != torch.device(device):
        raise ValueError(f"{name}: on {t.device}, expected {device}")
    if not t.is_contiguous():
        raise ValueError(f"{name}: must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name}: dtype {t.dtype}, expected {dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: shape {tuple(t.shape)}, expected {tuple(shape)}")
    if nbytes is not None and t.numel() * t.element_size() < nbytes:
        raise ValueError(f"{name}: {t.numel() * t.element_size()} bytes, needs at least {nbytes}")


def _need_layer(desc, x, in_features, packed, alpha, beta, A, B, x_name="x"):
    """Checks shared by every forward / backward entry; returns (tokens, device)."""
    _need(x, x_name, torch.bfloat16)
    dev = x.device
    if check_desc(desc) != OK:  # the library rejects the call with its own status
        return x.shape[0], dev
    if x.dim() != 2 or x.shape[1] != in_features:
        raise ValueError(f"{x_name}: shape {tuple(x.shape)}, expected [tokens, {in_features}]")
    L = desc.d_in // max(desc.group, 1)
    _need(packed, "packed", nbytes=packed_bytes(desc), device=dev)
    _need(alpha, "alpha", torch.float32, (L, desc.d_out), device=dev)
    if beta is not None:
        _need(beta, "beta", torch.float32, (L, desc.d_out), device=dev)
    if (A is None) != (B is None):
        raise ValueError("A and B must be given together")
    if A is not None:
        _need(A, "A", torch.float32, (L, desc.rank), device=dev)
        _need(B, "B", torch.float32, (desc.rank, desc.d_out), device=dev)
    return x.shape[0], dev


def _need_factor_pair(desc, alpha, other, other_name):
    _need(alpha, "alpha", torch.float32)
    shape = (desc.d_in // desc.group, desc.d_out) if check_desc(desc) == OK else tuple(alpha.shape)
    _need(alpha, "alpha", shape=shape)
    _need(other, other_name, torch.float32, shape, device=alpha.device)


def _need_out(t, name, rows, cols, dev):
    _need(t, name, shape=(rows, cols), device=dev)
    if t.dtype not in (torch.float32, torch.bfloat16):
        raise ValueError(f"{name}: dtype {t.dtype}, expected float32 or bfloat16")


def quantize(desc: Desc, W: torch.Tensor):
    """W fp32 [d_in, d_out] (device) -> (packed uint8, alpha fp32 [L, d_out], beta fp32 [L, d_out])."""
    _need(W, "W", torch.float32)
    if check_desc(desc) == OK:
        _need(W, "W", shape=(desc.d_in, desc.d_out))
    L = desc.d_in // max(desc.group, 1)
    packed = torch.empty(packed_bytes(desc), dtype=torch.uint8, device=W.device)
    alpha = torch.empty((L, desc.d_out), dtype=torch.float32, device=W.device)
    beta = torch.empty_like(alpha)
    rc = load().qalora_quantize(ctypes.byref(desc), _p(W), _p(packed), _p(alpha), _p(beta), None, 0,
                                _stream())
    _check(rc, "qalora_quantize")
    return packed, alpha, beta


def quantize_compensated(desc: Desc, W: torch.Tensor, hinv_chol: torch.Tensor):
    """Error-compensated code selection under an inverse-Hessian Cholesky factor U [d_in, d_in]
    (upper triangular, H^-1 = U^T U).  Returns (packed, alpha, beta) like quantize()."""
    _need(W, "W", torch.float32)
    if check_desc(desc) == OK:
        _need(W, "W", shape=(desc.d_in, desc.d_out))
        _need(hinv_chol, "hinv_chol", torch.float32, (desc.d_in, desc.d_in), device=W.device)
    L = desc.d_in // max(desc.group, 1)
    packed = torch.empty(packed_bytes(desc), dtype=torch.uint8, device=W.device)
    alpha = torch.empty((L, desc.d_out), dtype=torch.float32, device=W.device)
    beta = torch.empty_like(alpha)
    ws = torch.empty(max(workspace_bytes(desc, 1, OP_QUANTIZE_COMPENSATED), 16), dtype=torch.uint8, device=W.device)
    rc = load().qalora_quantize_compensated(ctypes.byref(desc), _p(W), _p(hinv_chol), _p(packed), _p(alpha),
                                            _p(beta), _p(ws), ws.numel(), _stream())
    _check(rc, "qalora_quantize_compensated")
    return packed, alpha, beta


def unpack(desc: Desc, packed: torch.Tensor) -> torch.Tensor:
    _need(packed, "packed", nbytes=packed_bytes(desc))
    codes = torch.empty((desc.d_in, desc.d_out), dtype=torch.uint8, device=packed.device)
    _check(load().qalora_unpack(ctypes.byref(desc), _p(packed), _p(codes), _stream()), "qalora_unpack")
    return codes


def pack(desc: Desc, codes: torch.Tensor) -> torch.Tensor:
    _need(codes, "codes", torch.uint8)
    if check_desc(desc) == OK:
        _need(codes, "codes", shape=(desc.d_in, desc.d_out))
    packed = torch.empty(packed_bytes(desc), dtype=torch.uint8, device=codes.device)
    _check(load().qalora_pack(ctypes.byref(desc), _p(codes), _p(packed), _stream()), "qalora_pack")
    return packed


def forward(desc: Desc, x, packed, alpha, beta, A=None, B=None, out_dtype=torch.float32, ws=None,
            y=None):
    """y = x W~ + s (pool(x) A) B.  x bf16 [T, d_in]; returns y [T, d_out]."""
    T, dev = _need_layer(desc, x, desc.d_in, packed, alpha, beta, A, B)
    if y is None:
        y = torch.empty((T, desc.d_out), dtype=out_dtype, device=dev)
    _need_out(y, "y", T, desc.d_out, dev)
    ws, ws_bytes = _workspace(desc, T, OP_FORWARD, ws, dev)
    rc = load().qalora_forward(ctypes.byref(desc), T, _p(x), _p(packed), _p(alpha), _p(beta), _p(A),
                               _p(B), _p(y), BF16 if y.dtype == torch.bfloat16 else F32, _p(ws),
                               ws_bytes, _stream())
    _check(rc, "qalora_forward")
    return y


def forward_noalloc(desc: Desc, x, packed, alpha, beta, out_dtype=torch.float32, y=None):
    """Adapter-free few-token forward on the library's built-in scratch (no workspace)."""
    T, dev = _need_layer(desc, x, desc.d_in, packed, alpha, beta, None, None)
    if y is None:
        y = torch.empty((T, desc.d_out), dtype=out_dtype, device=dev)
    _need_out(y, "y", T, desc.d_out, dev)
    rc = load().qalora_forward_noalloc(ctypes.byref(desc), T, _p(x), _p(packed), _p(alpha), _p(beta), _p(y),
                                       BF16 if y.dtype == torch.bfloat16 else F32, _stream())
    _check(rc, "qalora_forward_noalloc")
    return y


class Part(ctypes.Structure):
    """Mirror of ``qalora_part``."""
    _fields_ = [("d_out", ctypes.c_int32), ("rank", ctypes.c_int32), ("s", ctypes.c_float),
                ("A", ctypes.c_void_p), ("B", ctypes.c_void_p), ("dA", ctypes.c_void_p), ("dB", ctypes.c_void_p)]


def _parts(desc, adapters, dev, grads=None):
    """adapters: list of (A [L, rank], B [rank, d_out_p], s); grads: list of (dA, dB) or None."""
    L = desc.d_in // max(desc.group, 1)
    arr = (Part * len(adapters))()
    for q, (A, B, s) in enumerate(adapters):
        _need(A, f"A[{q}]", torch.float32, device=dev)
        _need(B, f"B[{q}]", torch.float32, device=dev)
        if A.dim() != 2 or B.dim() != 2 or A.shape[0] != L or A.shape[1] != B.shape[0]:
            raise ValueError(f"part {q}: A {tuple(A.shape)}, B {tuple(B.shape)}, expected [{L}, r] and [r, d_out]")
        arr[q].d_out, arr[q].rank, arr[q].s = int(B.shape[1]), int(A.shape[1]), float(s)
        arr[q].A, arr[q].B = A.data_ptr(), B.data_ptr()
        if grads is not None:
            dA, dB = grads[q]
            _need(dA, f"dA[{q}]", torch.float32, tuple(A.shape), device=dev)
            _need(dB, f"dB[{q}]", torch.float32, tuple(B.shape), device=dev)
            arr[q].dA, arr[q].dB = dA.data_ptr(), dB.data_ptr()
    if sum(int(B.shape[1]) for _, B, _ in adapters) != desc.d_out:
        raise ValueError("the parts' widths must add up to d_out")
    return arr


def forward_shared(desc: Desc, x, packed, alpha, beta, adapters, keep=False, out_dtype=torch.float32,
                   ws=None, y=None, kept=None):
    """Linears that share x as one wide layer (see qalora_forward_shared).  ``adapters`` is a
    list of (A, B, s), one per part in column order.  Returns y, or (y, kept) with ``keep``."""
    T, dev = _need_layer(desc, x, desc.d_in, packed, alpha, beta, None, None)
    arr = _parts(desc, adapters, dev)
    n = len(adapters)
    if y is None:
        y = torch.empty((T, desc.d_out), dtype=out_dtype, device=dev)
    _need_out(y, "y", T, desc.d_out, dev)
    if keep:
        kb = int(load().qalora_shared_kept_bytes(ctypes.byref(desc), T, n, arr))
        if kept is None:
            kept = torch.empty(max(kb, 16), dtype=torch.uint8, device=dev)
        _need(kept, "kept", nbytes=kb, device=dev)
    if ws is None:
        ws = torch.empty(max(int(load().qalora_shared_workspace_bytes(ctypes.byref(desc), T, OP_FORWARD, n, arr)), 16),
                         dtype=torch.uint8, device=dev)
    _need(ws, "ws", device=dev)
    rc = load().qalora_forward_shared(ctypes.byref(desc), T, _p(x), _p(packed), _p(alpha), _p(beta), n, arr,
                                      _p(y), BF16 if y.dtype == torch.bfloat16 else F32,
                                      _p(kept) if keep else None, _p(ws), ws.numel() * ws.element_size(), _stream())
    _check(rc, "qalora_forward_shared")
    return (y, kept) if keep else y


def backward_shared(desc: Desc, dy, x, kept, packed, alpha, beta, adapters, want_dx=True,
                    dx_dtype=torch.float32, grads=None, accumulate=False, ws=None, dx=None):
    """Backward of forward_shared: one dx over all parts, (dA, dB) per part.  Pass ``kept`` (from
    forward_shared(keep=True)) or ``x``.  Returns (dx, [(dA, dB), ...])."""
    T, dev = _need_layer(desc, dy, desc.d_out, packed, alpha, beta, None, None, x_name="dy")
    if kept is None:
        _need(x, "x", torch.bfloat16, (T, desc.d_in), device=dev)
    if grads is None:
        grads = [(torch.zeros_like(A), torch.zeros_like(B)) for A, B, _ in adapters]
    arr = _parts(desc, adapters, dev, grads)
    n = len(adapters)
    if kept is not None:
        _need(kept, "kept", nbytes=int(load().qalora_shared_kept_bytes(ctypes.byref(desc), T, n, arr)), device=dev)
    if want_dx and dx is None:
        dx = torch.empty((T, desc.d_in), dtype=dx_dtype, device=dev)
    if dx is not None:
        _need_out(dx, "dx", T, desc.d_in, dev)
    if ws is None:
        ws = torch.empty(max(int(load().qalora_shared_workspace_bytes(ctypes.byref(desc), T, OP_BACKWARD, n, arr)), 16),
                         dtype=torch.uint8, device=dev)
    _need(ws, "ws", device=dev)
    dxd = BF16 if (dx is not None and dx.dtype == torch.bfloat16) else F32
    rc = load().qalora_backward_shared(ctypes.byref(desc), T, _p(dy), _p(x) if kept is None else None, _p(kept),
                                       _p(packed), _p(alpha), _p(beta), n, arr, _p(dx), dxd,
                                       1 if accumulate else 0, _p(ws), ws.numel() * ws.element_size(), _stream())
    _check(rc, "qalora_backward_shared")
    return dx, grads


def deploy(desc: Desc, packed, alpha, beta):
    """One-time repack of a (merged) 4-bit layer into the decode kernel's stream."""
    n = int(load().qalora_deployed_bytes(ctypes.byref(desc)))
    if n == 0:
        raise QaloraError(EUNSUPPORTED, "qalora_deployed_bytes")
    L = desc.d_in // desc.group
    _need(packed, "packed", nbytes=packed_bytes(desc))
    _need(alpha, "alpha", torch.float32, (L, desc.d_out), device=packed.device)
    _need(beta, "beta", torch.float32, (L, desc.d_out), device=packed.device)
    out = torch.empty(n, dtype=torch.uint8, device=packed.device)
    _check(load().qalora_deploy(ctypes.byref(desc), _p(packed), _p(alpha), _p(beta), _p(out), _stream()),
           "qalora_deploy")
    return out


def forward_deployed(desc: Desc, x, deployed, packed=None, out_dtype=torch.float32, ws=None, y=None):
    """Adapter-free forward of a deployed layer: the decode stream up to four tokens, beyond that
    the dense kernel on ``packed`` (then required) with the prepared factor words."""
    _need(x, "x", torch.bfloat16)
    T, dev = x.shape[0], x.device
    if check_desc(desc) == OK:
        _need(x, "x", shape=(T, desc.d_in))
        _need(deployed, "deployed", nbytes=int(load().qalora_deployed_bytes(ctypes.byref(desc))), device=dev)
        if T > 4:
            _need(packed, "packed", nbytes=packed_bytes(desc), device=dev)
    if y is None:
        y = torch.empty((T, desc.d_out), dtype=out_dtype, device=dev)
    _need_out(y, "y", T, desc.d_out, dev)
    ws, ws_bytes = _workspace(desc, T, OP_FORWARD, ws, dev)
    rc = load().qalora_forward_deployed(ctypes.byref(desc), T, _p(x), _p(packed), _p(deployed), _p(y),
                                        BF16 if y.dtype == torch.bfloat16 else F32, _p(ws), ws_bytes, _stream())
    _check(rc, "qalora_forward_deployed")
    return y


WS_STATUS_OFFSET = 2048


def streaming_status(ws) -> int:
    """The status word the few-token kernels set in a forward workspace when a bounded wait ran
    out (0 = never, provided the caller zeroed it first).  Synchronises."""
    _need(ws, "ws", nbytes=WS_STATUS_OFFSET + 8)
    return int(ws.view(torch.uint8)[WS_STATUS_OFFSET:WS_STATUS_OFFSET + 8].cpu().view(torch.int64).item())


def pack_factors16(desc: Desc, alpha, beta, out=None):
    """One int32 word per (group, column): fp16(alpha) | fp16(beta) << 16."""
    L = desc.d_in // max(desc.group, 1)
    _need(alpha, "alpha", torch.float32, (L, desc.d_out))
    _need(beta, "beta", torch.float32, (L, desc.d_out), device=alpha.device)
    if out is None:
        out = torch.empty(alpha.shape, dtype=torch.int32, device=alpha.device)
    _need(out, "out", nbytes=4 * L * desc.d_out, device=alpha.device)
    _check(load().qalora_pack_factors16(ctypes.byref(desc), _p(alpha), _p(beta), _p(out), _stream()),
           "qalora_pack_factors16")
    return out


def forward_factors16(desc: Desc, x, packed, factors16, out_dtype=torch.float32, ws=None, y=None):
    """Adapter-free y = x W~ with the factors stored in 16 bits (see pack_factors16)."""
    _need(x, "x", torch.bfloat16)
    T, dev = x.shape[0], x.device
    if check_desc(desc) == OK:
        _need(x, "x", shape=(T, desc.d_in))
        _need(packed, "packed", nbytes=packed_bytes(desc), device=dev)
        _need(factors16, "factors16", nbytes=4 * (desc.d_in // desc.group) * desc.d_out, device=dev)
    if y is None:
        y = torch.empty((T, desc.d_out), dtype=out_dtype, device=dev)
    _need_out(y, "y", T, desc.d_out, dev)
    ws, ws_bytes = _workspace(desc, T, OP_FORWARD_FACTORS16, ws, dev)
    rc = load().qalora_forward_factors16(ctypes.byref(desc), T, _p(x), _p(packed), _p(factors16), _p(y),
                                         BF16 if y.dtype == torch.bfloat16 else F32, _p(ws), ws_bytes,
                                         _stream())
    _check(rc, "qalora_forward_factors16")
    return y


def backward(desc: Desc, dy, x, packed, alpha, beta, A=None, B=None, want_dx=True,
             dx_dtype=torch.float32, dA=None, dB=None, accumulate=False, ws=None, dx=None):
    """Returns (dx, dA, dB).  dy bf16 [T, d_out], x bf16 [T, d_in]."""
    T, dev = _need_layer(desc, dy, desc.d_out, packed, alpha, beta, A, B, x_name="dy")
    if A is not None or x is not None:
        _need(x, "x", torch.bfloat16, (T, desc.d_in), device=dev)
    if want_dx and dx is None:
        dx = torch.empty((T, desc.d_in), dtype=dx_dtype, device=dev)
    if dx is not None:
        _need_out(dx, "dx", T, desc.d_in, dev)
    if A is not None:
        if dA is None:
            dA = torch.zeros_like(A)
        if dB is None:
            dB = torch.zeros_like(B)
        _need(dA, "dA", torch.float32, tuple(A.shape), device=dev)
        _need(dB, "dB", torch.float32, tuple(B.shape), device=dev)
    ws, ws_bytes = _workspace(desc, T, OP_BACKWARD, ws, dev)
    dxd = BF16 if (dx is not None and dx.dtype == torch.bfloat16) else F32
    rc = load().qalora_backward(ctypes.byref(desc), T, _p(dy), _p(x), _p(packed), _p(alpha),
                                _p(beta), _p(A), _p(B), _p(dx), dxd, _p(dA), _p(dB),
                                1 if accumulate else 0, _p(ws), ws_bytes, _stream())
    _check(rc, "qalora_backward")
    return dx, dA, dB


def kept_bytes(desc: Desc, tokens: int) -> int:
    return int(load().qalora_kept_bytes(ctypes.byref(desc), tokens))


def forward_keep(desc: Desc, x, packed, alpha, beta, A, B, out_dtype=torch.float32, ws=None, y=None,
                 kept=None):
    """forward() that also leaves the pooled activations the backward needs.  Returns (y, kept)."""
    T, dev = _need_layer(desc, x, desc.d_in, packed, alpha, beta, A, B)
    if y is None:
        y = torch.empty((T, desc.d_out), dtype=out_dtype, device=dev)
    _need_out(y, "y", T, desc.d_out, dev)
    if kept is None:
        kept = torch.empty(max(kept_bytes(desc, T), 16), dtype=torch.uint8, device=dev)
    _need(kept, "kept", nbytes=kept_bytes(desc, T), device=dev)
    ws, ws_bytes = _workspace(desc, T, OP_FORWARD, ws, dev)
    rc = load().qalora_forward_keep(ctypes.byref(desc), T, _p(x), _p(packed), _p(alpha), _p(beta), _p(A),
                                    _p(B), _p(y), BF16 if y.dtype == torch.bfloat16 else F32, _p(kept),
                                    _p(ws), ws_bytes, _stream())
    _check(rc, "qalora_forward_keep")
    return y, kept


def backward_kept(desc: Desc, dy, kept, packed, alpha, beta, A, B, want_dx=True,
                  dx_dtype=torch.float32, dA=None, dB=None, accumulate=False, ws=None, dx=None):
    """backward() from what forward_keep() left instead of x.  Returns (dx, dA, dB)."""
    T, dev = _need_layer(desc, dy, desc.d_out, packed, alpha, beta, A, B, x_name="dy")
    _need(kept, "kept", nbytes=kept_bytes(desc, T), device=dev)
    if want_dx and dx is None:
        dx = torch.empty((T, desc.d_in), dtype=dx_dtype, device=dev)
    if dx is not None:
        _need_out(dx, "dx", T, desc.d_in, dev)
    if dA is None:
        dA = torch.zeros_like(A)
    if dB is None:
        dB = torch.zeros_like(B)
    _need(dA, "dA", torch.float32, tuple(A.shape), device=dev)
    _need(dB, "dB", torch.float32, tuple(B.shape), device=dev)
    ws, ws_bytes = _workspace(desc, T, OP_BACKWARD, ws, dev)
    dxd = BF16 if (dx is not None and dx.dtype == torch.bfloat16) else F32
    rc = load().qalora_backward_kept(ctypes.byref(desc), T, _p(dy), _p(kept), _p(packed), _p(alpha),
                                     _p(beta), _p(A), _p(B), _p(dx), dxd, _p(dA), _p(dB),
                                     1 if accumulate else 0, _p(ws), ws_bytes, _stream())
    _check(rc, "qalora_backward_kept")
    return dx, dA, dB


def merge(desc: Desc, beta, A, B, out=None):
    """beta' = beta + (s/g) A B; ``out`` may be ``beta`` itself."""
    _need(beta, "beta", torch.float32)
    if check_desc(desc) == OK:
        L = desc.d_in // desc.group
        _need(beta, "beta", shape=(L, desc.d_out))
        _need(A, "A", torch.float32, (L, desc.rank), device=beta.device)
        _need(B, "B", torch.float32, (desc.rank, desc.d_out), device=beta.device)
    if out is None:
        out = torch.empty_like(beta)
    _need(out, "out", torch.float32, tuple(beta.shape), device=beta.device)
    _check(load().qalora_merge(ctypes.byref(desc), _p(beta), _p(A), _p(B), _p(out), _stream()),
           "qalora_merge")
    return out


def beta_from_zero_point(desc: Desc, alpha, z, out=None):
    """beta = -(alpha z): import a zero point (code units) as the zero factor of Eq. 1."""
    _need_factor_pair(desc, alpha, z, "z")
    if out is None:
        out = torch.empty_like(alpha)
    _need(out, "out", torch.float32, tuple(alpha.shape), device=alpha.device)
    _check(load().qalora_beta_from_zero_point(ctypes.byref(desc), _p(alpha), _p(z), _p(out), _stream()),
           "qalora_beta_from_zero_point")
    return out


def zero_point_from_beta(desc: Desc, alpha, beta, out=None):
    """z = -(beta / alpha): export the zero factor as a zero point in code units."""
    _need_factor_pair(desc, alpha, beta, "beta")
    if out is None:
        out = torch.empty_like(alpha)
    _need(out, "out", torch.float32, tuple(alpha.shape), device=alpha.device)
    _check(load().qalora_zero_point_from_beta(ctypes.byref(desc), _p(alpha), _p(beta), _p(out), _stream()),
           "qalora_zero_point_from_beta")
    return out


class AdamW(ctypes.Structure):
    """Mirror of ``qalora_adamw``."""
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("weight_decay", ctypes.c_float), ("max_grad_norm", ctypes.c_float)]


def adamw_step(hp: AdamW, step: int, params, grads, exp_avg, exp_avg_sq, zero_grads=False, grad_norm=None,
               ws=None):
    """One fused AdamW step with a joint gradient-norm clip over lists of fp32 device tensors
    (updated in place).  ``grad_norm``: optional one-element fp32 device tensor for the norm."""
    n = len(params)
    for ts, nm in ((params, "params"), (grads, "grads"), (exp_avg, "exp_avg"), (exp_avg_sq, "exp_avg_sq")):
        if len(ts) != n:
            raise ValueError(f"{nm}: {len(ts)} tensors, expected {n}")
        for t, p0 in zip(ts, params):
            _need(t, nm, torch.float32, tuple(p0.shape), device=params[0].device)
    _need(grad_norm, "grad_norm", torch.float32, nbytes=4, optional=True)
    ptrs = [(ctypes.c_void_p * n)(*[t.data_ptr() for t in ts]) for ts in (params, grads, exp_avg, exp_avg_sq)]
    numel = (ctypes.c_size_t * n)(*[t.numel() for t in params])
    if ws is None:
        ws = torch.empty(max(load().qalora_adamw_workspace_bytes(n, numel), 16), dtype=torch.uint8, device="cuda")
    rc = load().qalora_adamw_step(ctypes.byref(hp), int(step), n, ptrs[0], ptrs[1], ptrs[2], ptrs[3], numel,
                                  1 if zero_grads else 0, _p(grad_norm), _p(ws), ws.numel(), _stream())
    _check(rc, "qalora_adamw_step")


def profile_copy(dst: torch.Tensor, src: torch.Tensor):
    """Plain copy kernel of known size (yardstick for the HBM traffic counters)."""
    _need(src, "src")
    n = src.numel() * src.element_size()
    _need(dst, "dst", nbytes=n, device=src.device)
    _check(load().qalora_profile_copy(_p(dst), _p(src), n, _stream()), "qalora_profile_copy")


def mfma_probe(shape: int, lds_reads: bool, valu_per_mfma: int, iters: int = 500, blocks: int = 256):
    """Issue-rate probe of the matrix cores (measurement aid).  Returns (cycles per matrix
    instruction per SIMD, shader clock in GHz, TFLOP/s) over all blocks of the launch."""
    sink = torch.empty(blocks * 512, dtype=torch.float32, device="cuda")
    counts = torch.zeros((blocks, 2), dtype=torch.int64, device="cuda")
    for _ in range(2):  # the second launch runs at the clock the mix settles to
        _check(load().qalora_profile_mfma_probe(int(shape), 1 if lds_reads else 0, int(valu_per_mfma), int(iters),
                                                int(blocks), _p(sink), _p(counts), _stream()), "qalora_profile_mfma_probe")
        torch.cuda.synchronize()
    khz = ctypes.c_int()
    _check(load().qalora_profile_wall_clock_khz(ctypes.byref(khz)), "wall_clock_khz")
    c = counts.cpu().double()
    cycles, ticks = c[:, 0].mean().item(), c[:, 1].mean().item()
    per_simd = iters * 64.0  # matrix instructions per SIMD: 32 per K step per wavefront, 2 wavefronts (or 64, 1)
    seconds = ticks / (khz.value * 1e3)
    flops = blocks * 4 * per_simd * 2.0 * 32 * 32 * 16
    return cycles / per_simd, cycles / ticks * khz.value * 1e3 / 1e9, flops / seconds / 1e12


def swiglu_forward(gate, up, out=None):
    """Harness glue: h = silu(gate) * up, bf16 tensors of equal shape."""
    _need(gate, "gate", torch.bfloat16)
    _need(up, "up", torch.bfloat16, tuple(gate.shape), device=gate.device)
    if out is None:
        out = torch.empty_like(gate)
    _need(out, "out", torch.bfloat16, tuple(gate.shape), device=gate.device)
    _check(load().qalora_swiglu_forward(_p(gate), _p(up), _p(out), gate.numel(), _stream()),
           "qalora_swiglu_forward")
    return out


def swiglu_backward(dh, gate, up, dgate=None, dup=None):
    """Harness glue: gradients of h = silu(gate) * up with respect to gate and up (bf16)."""
    _need(gate, "gate", torch.bfloat16)
    _need(up, "up", torch.bfloat16, tuple(gate.shape), device=gate.device)
    _need(dh, "dh", torch.bfloat16, tuple(gate.shape), device=gate.device)
    if dgate is None:
        dgate = torch.empty_like(gate)
    if dup is None:
        dup = torch.empty_like(up)
    _need(dgate, "dgate", torch.bfloat16, tuple(gate.shape), device=gate.device)
    _need(dup, "dup", torch.bfloat16, tuple(gate.shape), device=gate.device)
    _check(load().qalora_swiglu_backward(_p(dh), _p(gate), _p(up), _p(dgate), _p(dup), gate.numel(),
                                         _stream()), "qalora_swiglu_backward")
    return dgate, dup


def swiglu_forward_strided(gu, cols, out=None):
    """Harness glue on gu = [gate | up] ([rows, 2 cols] bf16): h = silu(gate) * up."""
    _need(gu, "gu", torch.bfloat16)
    rows = gu.shape[0]
    _need(gu, "gu", shape=(rows, 2 * cols))
    if out is None:
        out = torch.empty((rows, cols), dtype=torch.bfloat16, device=gu.device)
    _need(out, "out", torch.bfloat16, (rows, cols), device=gu.device)
    _check(load().qalora_swiglu_forward_wide(_p(gu), _p(out), rows, cols, _stream()), "qalora_swiglu_forward_wide")
    return out


def swiglu_backward_strided(dh, gu, cols, out=None):
    """Harness glue: dgu = [dgate | dup] of h = silu(gate) * up on gu = [gate | up]."""
    _need(gu, "gu", torch.bfloat16)
    rows = gu.shape[0]
    _need(gu, "gu", shape=(rows, 2 * cols))
    _need(dh, "dh", torch.bfloat16, (rows, cols), device=gu.device)
    if out is None:
        out = torch.empty_like(gu)
    _need(out, "out", torch.bfloat16, (rows, 2 * cols), device=gu.device)
    _check(load().qalora_swiglu_backward_wide(_p(dh), _p(gu), _p(out), rows, cols, _stream()),
           "qalora_swiglu_backward_wide")
    return out


class KernelTimer:
    """HIP-event pairs recorded by the library around its dense-contraction kernel
    (measurement aid of the C ABI); ``direction`` 0 = forward kernel, 1 = backward kernel."""

    def __init__(self, direction: int, n: int):
        self.direction = direction
        self.pairs = []
        for _ in range(n):
            a, b = ctypes.c_void_p(), ctypes.c_void_p()
            _check(load().qalora_profile_event_create(ctypes.byref(a)), "event_create")
            _check(load().qalora_profile_event_create(ctypes.byref(b)), "event_create")
            self.pairs.append((a, b))
        self.used = 0
        # per launch: shader cycles and wall-clock ticks at the first block's start and end
        self.counts = torch.zeros((n, 4), dtype=torch.int64, device="cuda")

    def arm(self):
        a, b = self.pairs[self.used]
        _check(load().qalora_profile_arm(self.direction, a, b), "profile_arm")
        _check(load().qalora_profile_arm_clock(self.direction, _p(self.counts[self.used])),
               "profile_arm_clock")
        self.used += 1

    def arm_blocks(self, capacity=4096):
        """Call right after arm(): the armed kernel's blocks also report their time line."""
        self.block_times = torch.zeros((capacity, 4), dtype=torch.int64, device="cuda")
        _check(load().qalora_profile_arm_blocks(self.direction, _p(self.block_times), capacity),
               "profile_arm_blocks")

    def block_timeline(self):
        """Summary of the last arm_blocks() launch, in microseconds from the first block's start."""
        khz = ctypes.c_int()
        _check(load().qalora_profile_wall_clock_khz(ctypes.byref(khz)), "wall_clock_khz")
        c = self.block_times.cpu().numpy()
        c = c[c[:, 0] > 0]
        if len(c) == 0:
            return None
        import numpy as np
        us = lambda v: (v - c[:, 0].min()) / khz.value * 1e3
        st, kend, en, xcd = us(c[:, 0]), us(c[:, 1]), us(c[:, 2]), c[:, 3]
        q = lambda v: [round(float(x), 1) for x in (v.min(), np.median(v), v.max())]
        return {"blocks": int(len(c)), "start_us_min_med_max": q(st), "k_loop_end_us_min_med_max": q(kend),
                "end_us_min_med_max": q(en), "epilogue_us_median": round(float(np.median(en - kend)), 1),
                "end_us_median_by_xcd": {int(x): round(float(np.median(en[xcd == x])), 1) for x in sorted(set(xcd.tolist()))}}

    def shader_clock_ghz(self):
        """Average shader clock over the life of the armed kernels' first blocks (None when the
        armed kernel was one that does not report)."""
        khz = ctypes.c_int()
        _check(load().qalora_profile_wall_clock_khz(ctypes.byref(khz)), "wall_clock_khz")
        c = self.counts[: self.used].cpu().double()
        cycles, ticks = c[:, 2] - c[:, 0], c[:, 3] - c[:, 1]
        ok = ticks > 0
        if not bool(ok.any()):
            return None
        return float((cycles[ok] / ticks[ok]).mean()) * khz.value * 1e3 / 1e9

    def block_cycles(self):
        """Mean shader cycles the armed kernels' first blocks lived for (None if not reported)."""
        c = self.counts[: self.used].cpu().double()
        cycles = c[:, 2] - c[:, 0]
        ok = (c[:, 3] - c[:, 1]) > 0
        return float(cycles[ok].mean()) if bool(ok.any()) else None

    def elapsed_ms(self):
        out = []
        for a, b in self.pairs[: self.used]:
            ms = ctypes.c_float()
            _check(load().qalora_profile_event_elapsed_ms(a, b, ctypes.byref(ms)), "event_elapsed")
            out.append(ms.value)
        return out

    def close(self):
        for a, b in self.pairs:
            load().qalora_profile_event_destroy(a)
            load().qalora_profile_event_destroy(b)
        self.pairs = []
