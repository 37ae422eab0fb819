"""CPU oracle for the QA-LoRA adapted linear layer -- TEST INFRASTRUCTURE ONLY.

Thin ctypes/numpy marshalling over ``qalora_oracle.c`` (plain C, fp64).  Only the
tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import this
package; the GPU library never does, and this package never imports the GPU
library.  Every function cites the passage of the paper it follows in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qalora_oracle.c")
_LIB = os.path.join(_HERE, "libqalora_oracle.so")
_lib = None

CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared", "-fPIC"]


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (seconds).  Rebuilds when the source is newer."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        try:
            build()
        except (OSError, subprocess.CalledProcessError):
            if not os.path.exists(_LIB):
                raise
        _lib = ctypes.CDLL(_LIB)
        _lib.qo_adapter_params.restype = ctypes.c_longlong
        _lib.qo_lora_params.restype = ctypes.c_longlong
        _lib.qo_quant_factor_pairs.restype = ctypes.c_longlong
        _lib.qo_sum_squares.restype = ctypes.c_double
    return _lib


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(_load().qo_num_threads())


def quantize(W, bits: int, group: int):
    """Group-wise min-max quantization (Eq. 1 per group, Sec. 3.3).

    Returns (codes uint8 [D_in, D_out], alpha fp32 [L, D_out], beta fp32 [L, D_out]).
    """
    W = _f32(W)
    d_in, d_out = W.shape
    L = d_in // group
    codes = np.empty((d_in, d_out), np.uint8)
    alpha = np.empty((L, d_out), np.float32)
    beta = np.empty((L, d_out), np.float32)
    rc = _load().qo_quantize(_ptr(W), d_in, d_out, bits, group, _ptr(codes), _ptr(alpha), _ptr(beta))
    if rc != 0:
        raise ValueError("oracle.quantize: bad arguments")
    return codes, alpha, beta


def quantize_compensated(W, U, bits: int, group: int, block: int = 128):
    """Error-compensated code selection (the post-training quantizer's role, Sec. 4.1 /
    App. B.1): rows quantized in order, each row's error spread over the later rows through
    U, the upper Cholesky factor of the inverse input Hessian (H^-1 = U^T U); lazy updates per
    ``block`` rows.  Same outputs as ``quantize``."""
    W, U = _f32(W), _f32(U)
    d_in, d_out = W.shape
    if U.shape != (d_in, d_in):
        raise ValueError("oracle.quantize_compensated: U must be [d_in, d_in]")
    L = d_in // group
    codes = np.empty((d_in, d_out), np.uint8)
    alpha = np.empty((L, d_out), np.float32)
    beta = np.empty((L, d_out), np.float32)
    rc = _load().qo_quantize_compensated(_ptr(W), d_in, d_out, bits, group, _ptr(U), block, _ptr(codes),
                                         _ptr(alpha), _ptr(beta))
    if rc != 0:
        raise ValueError("oracle.quantize_compensated: bad arguments")
    return codes, alpha, beta


def dequantize(codes, alpha, beta, group: int):
    """W~ = alpha * codes + beta per group (Eq. 1), fp64."""
    codes = np.ascontiguousarray(codes, np.uint8)
    alpha, beta = _f32(alpha), _f32(beta)
    d_in, d_out = codes.shape
    Wt = np.empty((d_in, d_out), np.float64)
    _load().qo_dequantize(_ptr(codes), _ptr(alpha), _ptr(beta), d_in, d_out, group, _ptr(Wt))
    return Wt


def pool(x, group: int):
    """Group average of the input (Sec. 3.3 / App. B.2 with the 1/g), fp64 [T, L]."""
    x = _f32(x)
    T, d_in = x.shape
    P = np.empty((T, d_in // group), np.float64)
    _load().qo_pool(_ptr(x), T, d_in, group, _ptr(P))
    return P


def forward(x, codes, alpha, beta, group: int, A=None, B=None, s: float = 0.0,
            round_wt_bf16: bool = False):
    """y = x W~ + s (pool(x) A) B (Alg. 1 forward), fp64 [T, D_out].

    ``A is None``: no adapter (post-merge inference).  ``round_wt_bf16`` selects the
    declared-precision mode (W~ rounded to bf16 before use); the default is the
    paper's definition.
    """
    x = _f32(x)
    codes = np.ascontiguousarray(codes, np.uint8)
    alpha, beta = _f32(alpha), _f32(beta)
    T, d_in = x.shape
    d_out = codes.shape[1]
    r = 0
    if A is not None:
        A, B = _f32(A), _f32(B)
        r = A.shape[1]
    y = np.empty((T, d_out), np.float64)
    _load().qo_forward(_ptr(x), T, _ptr(codes), _ptr(alpha), _ptr(beta), d_in, d_out, group,
                       _ptr(A), _ptr(B), r, ctypes.c_double(float(s)), int(round_wt_bf16), _ptr(y))
    return y


def backward(dy, x, codes, alpha, beta, group: int, A=None, B=None, s: float = 0.0,
             round_wt_bf16: bool = False, want_dx: bool = True, want_dAdB: bool = True):
    """(dx, dA, dB) of the forward above with W~ frozen (derived from Alg. 1), fp64."""
    dy, x = _f32(dy), _f32(x)
    codes = np.ascontiguousarray(codes, np.uint8)
    alpha, beta = _f32(alpha), _f32(beta)
    T, d_in = x.shape
    d_out = codes.shape[1]
    r = 0
    dA = dB = None
    if A is not None:
        A, B = _f32(A), _f32(B)
        r = A.shape[1]
        if want_dAdB:
            dA = np.empty(A.shape, np.float64)
            dB = np.empty(B.shape, np.float64)
    dx = np.empty((T, d_in), np.float64) if want_dx else None
    _load().qo_backward(_ptr(dy), _ptr(x), T, _ptr(codes), _ptr(alpha), _ptr(beta), d_in, d_out,
                        group, _ptr(A), _ptr(B), r, ctypes.c_double(float(s)), int(round_wt_bf16),
                        _ptr(dx), _ptr(dA), _ptr(dB))
    return dx, dA, dB


def merge(beta, A, B, group: int, s: float):
    """beta' = beta + (s/g) A B (Alg. 1 merge / App. B.3 in Eq. 1's convention), fp32."""
    beta, A, B = _f32(beta), _f32(A), _f32(B)
    L, d_out = beta.shape
    out = np.empty_like(beta)
    _load().qo_merge(_ptr(beta), _ptr(A), _ptr(B), L, d_out, A.shape[1], group,
                     ctypes.c_double(float(s)), _ptr(out))
    return out


def forward_zp_sum(x, codes, alpha, z, group: int, A=None, B=None, s_sum: float = 0.0):
    """The paper's literal form: W~ = alpha (codes - z), SUM pooling (Alg. 1, App. B)."""
    x = _f32(x)
    codes = np.ascontiguousarray(codes, np.uint8)
    alpha = _f32(alpha)
    z = np.ascontiguousarray(z, np.float64)
    T, d_in = x.shape
    d_out = codes.shape[1]
    r = 0
    if A is not None:
        A, B = _f32(A), _f32(B)
        r = A.shape[1]
    y = np.empty((T, d_out), np.float64)
    _load().qo_forward_zp_sum(_ptr(x), T, _ptr(codes), _ptr(alpha), _ptr(z), d_in, d_out, group,
                              _ptr(A), _ptr(B), r, ctypes.c_double(float(s_sum)), _ptr(y))
    return y


def merge_zp_sum(z, alpha, A, B, s_sum: float):
    """z' = z - s_sum (A B) / alpha (Alg. 1 merge_with_quantization, App. B.3)."""
    z = np.ascontiguousarray(z, np.float64)
    alpha, A, B = _f32(alpha), _f32(A), _f32(B)
    L, d_out = z.shape
    out = np.empty_like(z)
    _load().qo_merge_zp_sum(_ptr(z), _ptr(alpha), _ptr(A), _ptr(B), L, d_out, A.shape[1],
                            ctypes.c_double(float(s_sum)), _ptr(out))
    return out


def beta_from_zero_point(alpha, z):
    """beta = -alpha z: the zero factor of Eq. 1 that names the same weights as the zero
    point z of App. B.1 / Alg. 1 (fp64)."""
    alpha = _f32(alpha)
    z = np.ascontiguousarray(z, np.float64)
    out = np.empty(alpha.shape, np.float64)
    _load().qo_beta_from_zero_point(_ptr(alpha), _ptr(z), ctypes.c_size_t(alpha.size), _ptr(out))
    return out


def zero_point_from_beta(alpha, beta):
    """z = -beta / alpha (fp64): Eq. 1's zero factor as a zero point in code units."""
    alpha, beta = _f32(alpha), _f32(beta)
    out = np.empty(alpha.shape, np.float64)
    _load().qo_zero_point_from_beta(_ptr(alpha), _ptr(beta), ctypes.c_size_t(alpha.size), _ptr(out))
    return out


def grad_norm(grads) -> float:
    """Joint L2 norm of all gradient tensors (fp64)."""
    lib = _load()
    total = 0.0
    for g in grads:
        g = _f32(g)
        total += float(lib.qo_sum_squares(_ptr(g), ctypes.c_size_t(g.size)))
    return float(np.sqrt(total))


def adamw_step(params, grads, exp_avg, exp_avg_sq, step: int, lr: float, beta1: float = 0.9,
               beta2: float = 0.999, eps: float = 1e-8, weight_decay: float = 0.0,
               max_grad_norm: float = 0.0):
    """One AdamW step on a list of tensors with a joint gradient-norm clip (Sec. 4.1's recipe;
    max_grad_norm <= 0: no clip).  The clip factor is min(1, max / (norm + 1e-6)), the form the
    usual training loops apply.  Returns (params, exp_avg, exp_avg_sq) as fp64 lists and the norm."""
    lib = _load()
    norm = grad_norm(grads)
    clip = min(1.0, max_grad_norm / (norm + 1e-6)) if max_grad_norm > 0 else 1.0
    outs = ([], [], [])
    for p, g, m, v in zip(params, grads, exp_avg, exp_avg_sq):
        p, g, m, v = _f32(p), _f32(g), _f32(m), _f32(v)
        po, mo, vo = (np.empty(p.shape, np.float64) for _ in range(3))
        lib.qo_adamw_update(_ptr(p), _ptr(g), _ptr(m), _ptr(v), ctypes.c_size_t(p.size),
                            ctypes.c_double(clip), ctypes.c_double(lr), ctypes.c_double(beta1),
                            ctypes.c_double(beta2), ctypes.c_double(eps), ctypes.c_double(weight_decay),
                            int(step), _ptr(po), _ptr(mo), _ptr(vo))
        for o, t in zip(outs, (po, mo, vo)):
            o.append(t)
    return outs[0], outs[1], outs[2], norm


def adapter_params(d_in: int, d_out: int, group: int, rank: int) -> int:
    return int(_load().qo_adapter_params(d_in, d_out, group, rank))


def lora_params(d_in: int, d_out: int, rank: int) -> int:
    return int(_load().qo_lora_params(d_in, d_out, rank))


def quant_factor_pairs(d_in: int, d_out: int, group: int) -> int:
    return int(_load().qo_quant_factor_pairs(d_in, d_out, group))
