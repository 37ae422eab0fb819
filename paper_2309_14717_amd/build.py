"""Compile the HIP sources into the in-tree C-ABI shared library for gfx950.

Run as ``python -m paper_2309_14717_amd.build``.  hipcc cross-compiles without a GPU.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libqalora_hip.so")
SOURCES = ["api.hip", "quantize.hip", "gemm_dq.hip", "adapter.hip", "smallt.hip", "smallt4.hip", "smallt4_f16.hip",
           "glue.hip", "optim.hip", "probe.hip", "compensate.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


# Kernels that must compile with zero scratch memory: those whose waits on outstanding memory
# operations are counted by hand (a register spill would add scratch traffic to the same
# counter), and the adapter-gradient kernel, whose staging arrays once ended up in scratch
# unnoticed (a local array the compiler does not promote to registers costs a round trip to
# memory per element).
NO_SCRATCH = {"gemm_dq.hip": "gemm_dq_kernel", "smallt.hip": "smallt_kernel", "smallt4.hip": "smallt4_kernel", "smallt4_f16.hip": "smallt4_kernel",
              "adapter.hip": ("adapter_grads_kernel", "front_kernel", "front_wide_kernel")}


def _as_tuple(v):
    return v if isinstance(v, tuple) else (v,)


def _check_no_scratch(src: str, remarks: str) -> None:
    """Parse -Rpass-analysis=kernel-resource-usage remarks; fail on any scratch use."""
    name, bad = None, []
    for line in remarks.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].split()[0]
        elif "ScratchSize [bytes/lane]:" in line and name and any(k in name for k in _as_tuple(NO_SCRATCH[src])):
            if int(line.split("ScratchSize [bytes/lane]:")[1].split()[0]) != 0:
                bad.append(name)
    if bad:
        raise RuntimeError(f"{src}: kernels that must not use scratch memory do: {bad}")


def _compile(src: str, extra) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    if src in NO_SCRATCH:
        cmd.insert(1, "-Rpass-analysis=kernel-resource-usage")
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if res.returncode != 0:
            sys.stderr.write(res.stdout)
            raise subprocess.CalledProcessError(res.returncode, cmd)
        _check_no_scratch(src, res.stdout)
    else:
        subprocess.check_call(cmd)
    return obj


def build(verbose: bool = False, extra_flags=(), variant: str = "") -> str:
    """Build the library.  `variant` names a measurement build (say, with -DQALORA_ABLATE=n in
    `extra_flags`): it goes to libqalora_hip.<variant>.so with objects of its own, so the
    library the tests and the product load is never replaced by it."""
    global OBJ
    lib = LIB if not variant else LIB[:-3] + "." + variant + ".so"
    obj_dir = OBJ if not variant else OBJ + "_" + variant
    os.makedirs(obj_dir, exist_ok=True)
    saved, OBJ = OBJ, obj_dir
    try:
        with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
            objs = list(ex.map(lambda s: _compile(s, list(extra_flags)), SOURCES))
    finally:
        OBJ = saved
    tmp = lib + ".tmp%d" % os.getpid()
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
    os.replace(tmp, lib)
    if verbose:
        print("built", lib)
    return lib


if __name__ == "__main__":
    # python -m paper_2309_14717_amd.build [--variant NAME] [compiler flags ...]
    args = sys.argv[1:]
    name = ""
    if len(args) >= 2 and args[0] == "--variant":
        name, args = args[1], args[2:]
    build(verbose=True, extra_flags=args, variant=name)
