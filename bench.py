#!/usr/bin/env python3
"""Benchmark of the QA-LoRA adapted linear layer on one MI355X.

Workloads (``--workload``), all on seeded synthetic tensors already resident in HBM:

  c2 (default)  one adapted forward (y = x W~ + s (pool(x) A) B) plus one backward (dx, dA, dB) of
                the LLaMA-7B attention-projection layer.  "extras" also reports quantize, merge,
                the post-merge forward and the small-token (memory-bound) table of the c5 shapes.
  c3            the SwiGLU MLP block of one LLaMA-7B decoder layer: gate/up/down adapted linears,
                forward and backward (dx, dA, dB of all three); the elementwise glue is torch.
  c4            one layer of the LLaMA-13B low-bit sweep at --bits / --group.
  probe         measurement aids only (no layer): what the matrix cores sustain under the
                instruction mixes of the contraction kernel (qalora_profile_mfma_probe) and the
                rate of the vendor library's plain fp16 / bf16 product on the same box.
  c5            post-merge inference at --tokens (1, 4, 16 or 256): one forward of the
                8192x22016 layer plus one of the 22016x8192 layer, rotating over eight weight
                sets (> 1 GB) so that nothing is served from the last-level cache.

A "step" is one pass of the workload.  Quantization of W is setup and is not timed.
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_TFLOPS = 2500.0   # MI355X dense bf16 / fp16 matrix peak
NOMINAL_CLOCK_GHZ = 2.4      # the clock the published peaks assume
PEAK_HBM_GBS = 8000.0
METRIC = "QA-LoRA linear fwd+bwd TFLOP/s & % of MFMA/HBM roofline, LLaMA-7B shapes"


def layer_flops(cfg, adapter=True):
    """Algorithmic flops of one forward and one backward (two dense contractions, no dW product,
    plus the adapter products); unpack / dequant / pooling count zero."""
    T, di, do, r, L = cfg.tokens, cfg.d_in, cfg.d_out, cfg.rank, cfg.groups
    main = 2.0 * T * di * do
    if not adapter:
        return dict(fwd=main, bwd=main, fwd_kernel=main, bwd_kernel=main)
    fwd_adapter = 2.0 * T * L * r + 2.0 * T * r * do
    bwd_adapter = 2 * (2.0 * T * r * do) + 2 * (2.0 * T * L * r)
    return dict(fwd=main + fwd_adapter, bwd=main + bwd_adapter,
                fwd_kernel=main + 2.0 * T * r * do,          # x W~ + (sU) B
                bwd_kernel=main + 2.0 * T * L * r)           # dy W~^T + dU A^T (unpooled)


def forward_bytes(cfg, tokens, out_bytes=2, factor_bytes=4):
    """Algorithmic HBM bytes of one adapter-free forward: every operand once."""
    codes = cfg.d_in * cfg.d_out * cfg.bits // 8
    factors = 2 * cfg.groups * cfg.d_out * factor_bytes
    return codes + factors + tokens * cfg.d_in * 2 + tokens * cfg.d_out * out_bytes


def read_traffic(name, key="traffic_bytes_per_launch"):
    """HBM bytes per launch of the dominant kernel.  Hardware counters cannot be read from inside
    this process, so the figure is the one of the committed rocprofv3 --pmc summary of the same
    workload, and `traffic_source` in the output says so."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        for line in open(path):
            if line.startswith(key + ":"):
                return float(line.split(":", 1)[1].split()[0])
    except OSError:
        pass
    return None


def traffic_fields(name, key="traffic_bytes_per_launch"):
    t = read_traffic(name, key) if name else None
    return {"traffic": t,
            "traffic_source": (f"profiles/{name} (committed rocprofv3 --pmc run of this workload, not "
                               "measured in this run)") if t is not None else None}


class Layer:
    """One quantized layer on the device, with adapters and preallocated outputs / workspace."""

    keep = True   # training steps: the forward keeps pool(x) and U for the backward (--no-keep: re-read x)

    def __init__(self, api, torch, cfg, odt, gen=None, want_bwd=True, merged=False):
        self.api, self.cfg = api, cfg
        from paper_2309_14717_amd import synth
        dev = "cuda"
        self.desc = api.make_desc(cfg.d_in, cfg.d_out, cfg.bits, cfg.group, cfg.rank, cfg.s)
        if gen is None:   # host generator: the arrays the parity tests and the oracle use
            d = synth.make_inputs(cfg)
            self.host = d
            W = torch.from_numpy(d["W"]).to(dev)
            self.x = torch.from_numpy(d["x"]).to(dev).to(torch.bfloat16)
            self.dy = torch.from_numpy(d["dy"]).to(dev).to(torch.bfloat16) if want_bwd else None
            self.A = torch.from_numpy(d["A"]).to(dev)
            self.B = torch.from_numpy(d["B"]).to(dev)
        else:             # device generator: extra weight sets of the same distribution
            self.host = None
            W = torch.randn((cfg.d_in, cfg.d_out), generator=gen, device=dev) * cfg.w_std
            self.x = torch.randn((cfg.tokens, cfg.d_in), generator=gen, device=dev).to(torch.bfloat16)
            self.dy = None
            self.A = torch.randn((cfg.groups, cfg.rank), generator=gen, device=dev) * cfg.ab_std
            self.B = torch.randn((cfg.rank, cfg.d_out), generator=gen, device=dev) * cfg.ab_std
        self.W = W
        self.packed, self.alpha, self.beta = api.quantize(self.desc, W)
        self.beta_m = api.merge(self.desc, self.beta, self.A, self.B) if merged else None
        self.fac16 = None
        self.dep = None   # deployment stream of the merged layer (decode layout)
        T = cfg.tokens
        self.y = torch.empty((T, cfg.d_out), dtype=odt, device=dev)
        self.ws_f = torch.empty(max(16, api.workspace_bytes(self.desc, T, api.OP_FORWARD)), dtype=torch.uint8, device=dev)
        if want_bwd:
            self.dx = torch.empty((T, cfg.d_in), dtype=odt, device=dev)
            self.dA, self.dB = torch.zeros_like(self.A), torch.zeros_like(self.B)
            self.ws_b = torch.empty(api.workspace_bytes(self.desc, T, api.OP_BACKWARD), dtype=torch.uint8, device=dev)
            self.kept = torch.empty(max(16, api.kept_bytes(self.desc, T)), dtype=torch.uint8, device=dev)

    def drop_w(self):
        self.W = None

    def forward(self, x=None):
        a = self.api
        if self.keep and self.dy is not None:
            return a.forward_keep(self.desc, self.x if x is None else x, self.packed, self.alpha, self.beta,
                                  self.A, self.B, ws=self.ws_f, y=self.y, kept=self.kept)[0]
        return a.forward(self.desc, self.x if x is None else x, self.packed, self.alpha, self.beta,
                         self.A, self.B, ws=self.ws_f, y=self.y)

    def forward_merged(self, x=None, y=None, ws=None):
        a = self.api
        xx = self.x if x is None else x
        if self.dep is not None and (xx.shape[0] <= 4 or xx.shape[0] > 32):
            # the static merged layer as deployed: decode stream, or prepared factor words
            return a.forward_deployed(self.desc, xx, self.dep, packed=self.packed,
                                      ws=self.ws_f if ws is None else ws, y=self.y if y is None else y)
        if self.fac16 is not None:  # factors of the merged layer stored as fp16 pairs
            return a.forward_factors16(self.desc, self.x if x is None else x, self.packed, self.fac16,
                                       ws=self.ws_f if ws is None else ws, y=self.y if y is None else y)
        return a.forward(self.desc, self.x if x is None else x, self.packed, self.alpha, self.beta_m,
                         ws=self.ws_f if ws is None else ws, y=self.y if y is None else y)

    def backward(self, dy=None, x=None):
        a = self.api
        if self.keep:   # x is not read: the matching forward() left what is needed in self.kept
            return a.backward_kept(self.desc, self.dy if dy is None else dy, self.kept, self.packed,
                                   self.alpha, self.beta, self.A, self.B, dA=self.dA, dB=self.dB,
                                   ws=self.ws_b, dx=self.dx)
        return a.backward(self.desc, self.dy if dy is None else dy, self.x if x is None else x,
                          self.packed, self.alpha, self.beta, self.A, self.B, dA=self.dA, dB=self.dB,
                          ws=self.ws_b, dx=self.dx)


class MlpBlock:
    """The SwiGLU MLP block of one LLaMA-7B decoder layer (workload c3): three adapted linears
    chained through bf16 activations, y = down(silu(gate(x)) * up(x)), and its backward."""

    def __init__(self, api, torch, synth, odt):
        self.api = api
        self.gate = Layer(api, torch, synth.CONFIGS["c3_gate"], odt)
        self.gate.drop_w()
        self.up = Layer(api, torch, synth.CONFIGS["c3_up"], odt)
        self.up.drop_w()
        self.down = Layer(api, torch, synth.CONFIGS["c3_down"], odt)
        self.down.drop_w()
        self.x, self.dy = self.gate.x, self.down.dy
        self.h = torch.empty_like(self.gate.y)
        self.dg, self.du = torch.empty_like(self.gate.y), torch.empty_like(self.gate.y)

    def step(self):
        api, gate, up, down, x = self.api, self.gate, self.up, self.down, self.x
        g = gate.forward(x)
        u = up.forward(x)
        api.swiglu_forward(g, u, out=self.h)
        down.forward(self.h)
        dh, _, _ = down.backward(self.dy, self.h)
        api.swiglu_backward(dh, g, u, dgate=self.dg, dup=self.du)
        dx1, _, _ = gate.backward(self.dg, x)
        dx2, _, _ = up.backward(self.du, x)
        return dx1.add_(dx2)


class MlpBlockShared(MlpBlock):
    """The same block with gate and up evaluated as one 4096 x 22016 layer (they share x): one
    front pass and one dense launch forward, and dx of both as one contraction over K = 22016."""

    def __init__(self, api, torch, synth, odt):
        self.api = api
        cg, cu = synth.CONFIGS["c3_gate"], synth.CONFIGS["c3_up"]
        g, u = synth.make_inputs(cg), synth.make_inputs(cu)
        dev = "cuda"
        W = torch.from_numpy(np.concatenate([g["W"], u["W"]], axis=1)).to(dev)
        self.desc = api.make_desc(cg.d_in, cg.d_out + cu.d_out, cg.bits, cg.group)
        self.packed, self.alpha, self.beta = api.quantize(self.desc, W)
        del W
        self.adapters = [(torch.from_numpy(d["A"]).to(dev), torch.from_numpy(d["B"]).to(dev), c.s)
                         for c, d in ((cg, g), (cu, u))]
        self.grads = [(torch.zeros_like(A), torch.zeros_like(B)) for A, B, _ in self.adapters]
        self.gate_cfg, self.up_cfg = cg, cu
        self.down = Layer(api, torch, synth.CONFIGS["c3_down"], odt)
        self.down.drop_w()
        self.x = torch.from_numpy(g["x"]).to(dev).to(torch.bfloat16)
        self.dy = self.down.dy
        T = cg.tokens
        self.gu = torch.empty((T, self.desc.d_out), dtype=odt, device=dev)      # [gate | up]
        self.dgu = torch.empty_like(self.gu)
        self.h = torch.empty((T, cg.d_out), dtype=odt, device=dev)
        self.dx = torch.empty((T, cg.d_in), dtype=odt, device=dev)
        lib, arr = api.load(), api._parts(self.desc, self.adapters, self.x.device)
        import ctypes
        self.kept = torch.empty(lib.qalora_shared_kept_bytes(ctypes.byref(self.desc), T, 2, arr), dtype=torch.uint8, device=dev)
        self.ws_f = torch.empty(lib.qalora_shared_workspace_bytes(ctypes.byref(self.desc), T, api.OP_FORWARD, 2, arr),
                                dtype=torch.uint8, device=dev)
        self.ws_b = torch.empty(lib.qalora_shared_workspace_bytes(ctypes.byref(self.desc), T, api.OP_BACKWARD, 2, arr),
                                dtype=torch.uint8, device=dev)

    def step(self):
        api, down, n = self.api, self.down, self.gate_cfg.d_out
        w = (self.packed, self.alpha, self.beta, self.adapters)
        api.forward_shared(self.desc, self.x, *w, keep=True, ws=self.ws_f, y=self.gu, kept=self.kept)
        api.swiglu_forward_strided(self.gu, n, out=self.h)
        down.forward(self.h)
        dh, _, _ = down.backward(self.dy, self.h)
        api.swiglu_backward_strided(dh, self.gu, n, out=self.dgu)
        dx, _ = api.backward_shared(self.desc, self.dgu, None, self.kept, *w, grads=self.grads, ws=self.ws_b, dx=self.dx)
        return dx


def timed(torch, fn, n=20, warm=2):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    s.record()
    for _ in range(n):
        fn()
    e.record()
    torch.cuda.synchronize()
    return s.elapsed_time(e) / n


def capture(torch, fns):
    """One HIP graph holding a call of each fn in order (each has run eagerly before: the first
    use of a kernel sets its LDS attribute, which is not stream work)."""
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for fn in fns:
            fn()
    return g


def timed_graph(torch, fns, n):
    """Average time of one call over n calls that cycle through `fns`, launched as graph replays:
    launches of 25 us kernels from Python are otherwise bound by the host (two argument-checked
    ctypes calls take longer than the kernels they start on a slow host core), which is not what
    a serving loop does either."""
    for fn in fns:
        fn()
    torch.cuda.synchronize()
    full = capture(torch, fns)
    rem = capture(torch, fns[: n % len(fns)]) if n % len(fns) else None
    for _ in range(2):
        full.replay()
    torch.cuda.synchronize()
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    s.record()
    for _ in range(n // len(fns)):
        full.replay()
    if rem is not None:
        rem.replay()
    e.record()
    torch.cuda.synchronize()
    return s.elapsed_time(e) / n


KERNEL_STATS = {}  # direction -> median / min / count of the armed kernel durations of the last run


SETTLE = {}  # extra untimed warm-up the last run_steps needed before its step time was steady


def settle(torch, step, chunk=10, tol=0.015, max_chunks=40):
    """Untimed warm-up beyond --warmup: run chunks of `chunk` steps until two consecutive chunks
    agree to `tol` (the chip's power management takes a while to reach the clock it then holds
    under this load; a short run would otherwise time the transient)."""
    prev, calm, n = None, 0, 0
    for _ in range(max_chunks):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(chunk):
            step()
        torch.cuda.synchronize()
        t = time.perf_counter() - t0
        n += chunk
        calm = calm + 1 if (prev is not None and abs(t - prev) <= tol * prev) else 0
        prev = t
        if calm >= 2:
            break
    return n


BLOCK_TIMELINE = {}
ARM_EVERY = [None]   # --arm-every


def run_steps(torch, api, step, steps, warmup, directions=(0, 1), arm_every=None):
    """Warm up, then time exactly `steps` steps; per-direction kernel times from events armed
    around the dense kernel on every `arm_every`-th step of the timed region (an armed launch
    costs the stream a few microseconds of event handling, which would otherwise weigh on
    `value` -- by 10 % for the 30 us kernels of the small-token workload).  Short runs arm every
    second step so that the kernel figure still rests on ten samples or more."""
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    if arm_every is None:
        arm_every = 2 if steps <= 50 else 4
    # (the timers are made before the settling steps, so that nothing but the synchronisation
    # lies between the last settling step and the timed region)
    timers = {d: api.KernelTimer(d, (steps + arm_every - 1) // arm_every) for d in directions}
    SETTLE["steps"] = settle(torch, step)
    t0 = time.perf_counter()
    for i in range(steps):
        if i % arm_every == 0:
            for t in timers.values():
                t.arm()
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kms = {d: float(np.mean(t.elapsed_ms())) for d, t in timers.items()}
    for d, t in timers.items():  # median and minimum of the same samples, for the record
        ms = np.asarray(t.elapsed_ms())
        KERNEL_STATS[d] = {"median_ms": round(float(np.median(ms)), 5), "min_ms": round(float(ms.min()), 5),
                           "samples": int(ms.size), "block_cycles": t.block_cycles()}
    clk = {d: t.shader_clock_ghz() for d, t in timers.items()}
    for t in timers.values():
        t.close()
    # outside the timed region: one more step whose armed kernels lay their blocks out on a time line
    extra = {d: api.KernelTimer(d, 1) for d in directions}
    for t in extra.values():
        t.arm()
        t.arm_blocks()
    step()
    torch.cuda.synchronize()
    for d, t in extra.items():
        BLOCK_TIMELINE[d] = t.block_timeline()
        t.close()
    return (t1 - t0) * 1e3 / steps, kms, clk


def clock_fields(clk_ghz, achieved_tflops):
    """The published matrix-core peak assumes the nominal clock; under load the chip runs the
    kernel slower.  Report the clock the kernel's first block measured for itself and the
    fraction of the peak scaled to that clock (context: `frac` stays against the published peak)."""
    if not clk_ghz:
        return {}
    return {"shader_clock_ghz": round(clk_ghz, 3),
            "frac_at_measured_clock": round(achieved_tflops / (PEAK_MFMA_TFLOPS * clk_ghz / NOMINAL_CLOCK_GHZ), 4)}


def small_token_sets(torch, api, synth, name, n_sets, odt, bits=4, deployed=False):
    """`n_sets` merged layers of one c5 shape (distinct weights, same distribution); with
    `deployed` each also holds its deployment stream (the static merged model repacked once)."""
    cfg = synth.CONFIGS[name].scaled(tokens=256, bits=bits)
    gen = torch.Generator(device="cuda").manual_seed(1000 + cfg.seed)
    sets = []
    for i in range(n_sets):
        L = Layer(api, torch, cfg, odt, gen=gen if i else None, want_bwd=False, merged=True)
        L.drop_w()
        if deployed and bits == 4:
            L.dep = api.deploy(L.desc, L.packed, L.alpha, L.beta_m)
        sets.append(L)
    return cfg, sets


def small_token_table(torch, api, synth, odt, n_sets=8, tokens=(1, 4, 16, 256), iters=128):
    rows = []
    for name in ("c5_up", "c5_down"):
        cfg, sets = small_token_sets(torch, api, synth, name, n_sets, odt, deployed=True)
        for T in tokens:
            x = sets[0].x[:T].contiguous()
            y = torch.empty((T, cfg.d_out), dtype=odt, device="cuda")
            ws = torch.empty(api.workspace_bytes(sets[0].desc, T, api.OP_FORWARD), dtype=torch.uint8, device="cuda")
            # four rotations of the weight sets per graph: the seam between two replays costs a few
            # microseconds, which 8 launches of 25 us would carry visibly
            ms = timed_graph(torch, [(lambda L=L: L.forward_merged(x=x, y=y, ws=ws)) for L in sets] * 4, iters)
            by = forward_bytes(cfg, T, y.element_size())
            fl = 2.0 * T * cfg.d_in * cfg.d_out
            rows.append({"shape": f"{cfg.d_in}x{cfg.d_out}", "tokens": T,
                         "layout": ("deployment stream" if T <= 4 else
                                    ("packed codes + deployed factor words" if T > 32 else "training layout")), "us": round(ms * 1e3, 2),
                         "GB/s": round(by / ms / 1e6, 1), "frac_hbm": round(by / ms / 1e6 / PEAK_HBM_GBS, 4),
                         "TFLOP/s": round(fl / ms / 1e9, 2)})
        del sets
        torch.cuda.empty_cache()
    return rows


def adamw_layer_timing(torch, api, d=4096, ff=11008, g=32, r=64):
    """The fused optimiser step over the adapters of one LLaMA-7B decoder layer (seven linears,
    fourteen tensors; AdamW with the 0.3 norm clip of the paper's recipe).  Algorithmic bytes:
    the gradient once for the norm, then p, g, m, v read and p, m, v written = 32 B/parameter."""
    shapes = []
    for d_in, d_out in ((d, d),) * 4 + ((d, ff), (d, ff), (ff, d)):
        shapes += [(d_in // g, r), (r, d_out)]
    gen = torch.Generator(device="cuda").manual_seed(5)
    p = [torch.randn(s, device="cuda", generator=gen) * 0.02 for s in shapes]
    gr = [torch.randn(s, device="cuda", generator=gen) for s in shapes]
    m = [torch.zeros_like(x) for x in p]
    v = [torch.zeros_like(x) for x in p]
    hp = api.AdamW(2e-5, 0.9, 0.999, 1e-8, 0.0, 0.3)
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    # (replayed as a graph: the two launches take 20 us, less than their launch from Python; the
    # step number, a kernel argument, then stays at 2, which changes no timing)
    api.adamw_step(hp, 1, p, gr, m, v, ws=ws)
    ms = timed_graph(torch, [lambda: api.adamw_step(hp, 2, p, gr, m, v, ws=ws)] * 5, 50)
    n = sum(x.numel() for x in p)
    return {"parameters": n, "tensors": len(p), "us": round(ms * 1e3, 2), "GB/s": round(32.0 * n / ms / 1e6, 1),
            "frac_hbm": round(32.0 * n / ms / 1e6 / PEAK_HBM_GBS, 4)}


def probe_report(torch, api):
    """Ceilings of the dense contraction on this machine: issue interval, clock and rate of the
    matrix instruction alone, with the operand reads from LDS, and with n vector instructions
    behind each one (all 256 compute units busy, and 16 of them for comparison); and the vendor
    library's plain product (torch.matmul) at two sizes."""
    rows = []
    for blocks in (16, 256):
        for shape, lds, nv in ((0, 0, 0), (0, 1, 0), (0, 1, 1), (0, 1, 2), (0, 1, 3), (0, 1, 4), (0, 1, 6), (0, 1, 8),
                               (0, 1, 102), (0, 1, 104),   # 2 / 4 per MFMA, issued as one burst per K-16 slice
                               (1, 0, 0), (1, 1, 0), (1, 1, 2), (1, 1, 4), (1, 1, 6), (1, 1, 8),
                               (2, 0, 0), (2, 1, 0), (2, 1, 2), (2, 1, 4)):
            cyc, ghz, tf = api.mfma_probe(shape, bool(lds), nv, iters=2000, blocks=blocks)
            rows.append({"blocks": blocks, "wavefronts_x_tiles": ("8 x (4x2)", "4 x (4x4)", "8 x (4x2) AGPR acc")[shape],
                         "lds_fragment_reads": bool(lds), "valu_per_mfma": nv % 100,
                         "valu_issued": "burst per slice" if nv >= 100 else "behind each MFMA",
                         "cycles_per_mfma_per_simd": round(cyc, 2), "shader_clock_ghz": round(ghz, 3),
                         "TFLOP/s": round(tf, 1), "frac_of_peak": round(tf / PEAK_MFMA_TFLOPS, 4)})
    vendor = []
    for n in (4096, 8192):
        for dt, name in ((torch.float16, "f16"), (torch.bfloat16, "bf16")):
            a = torch.randn((n, n), device="cuda").to(dt)
            b = torch.randn((n, n), device="cuda").to(dt)
            c = torch.empty((n, n), device="cuda", dtype=dt)
            ms = timed(torch, lambda: torch.matmul(a, b, out=c), n=50, warm=10)
            tf = 2.0 * n ** 3 / ms / 1e9
            vendor.append({"n": n, "dtype": name, "ms": round(ms, 4), "TFLOP/s": round(tf, 1),
                           "frac_of_peak": round(tf / PEAK_MFMA_TFLOPS, 4)})
            del a, b, c
    return {"workload": "probe: matrix-core issue probes and the vendor library's plain product",
            "mfma_probe": rows, "vendor_gemm": vendor}


def two_stream_backward(torch, api, synth):
    """Can the adapter-gradient kernels hide under the dx contraction?  The backward of the c2
    layer as two calls -- dx only (adapter-free: front pass and contraction) and gradients only
    (front pass, dU product, gradient kernels, reduction) -- one after the other on one stream,
    and at the same time on two streams of equal priority."""
    cfg = synth.CONFIGS["c2"]
    L = Layer(api, torch, cfg, torch.bfloat16)
    L.drop_w()
    d = L.desc
    ws2 = torch.empty_like(L.ws_b)
    dA2, dB2 = torch.zeros_like(L.A), torch.zeros_like(L.B)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()

    def dx_only():
        api.backward(d, L.dy, None, L.packed, L.alpha, L.beta, None, None, ws=L.ws_b, dx=L.dx)

    def grads_only():
        api.backward(d, L.dy, L.x, L.packed, L.alpha, L.beta, L.A, L.B, want_dx=False, dA=dA2, dB=dB2, ws=ws2)

    def one_stream():
        dx_only()
        grads_only()

    def two_streams():
        with torch.cuda.stream(s2):
            grads_only()
        with torch.cuda.stream(s1):
            dx_only()

    def wall(fn, n=60):
        for _ in range(20):
            fn()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return round((time.perf_counter() - t) / n * 1e6, 1)

    return {"dx_only_us": wall(dx_only), "gradients_only_us": wall(grads_only),
            "both_on_one_stream_us": wall(one_stream), "both_on_two_streams_us": wall(two_streams)}


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_oracle_baseline(fn_flops_pairs, label):
    """Time the oracle (as it stands) on the host: list of (callable, flops)."""
    import oracle
    tc = time.perf_counter()
    flops = 0.0
    for fn, fl in fn_flops_pairs:
        fn()
        flops += fl
    dt = time.perf_counter() - tc
    return {"value": round(flops / dt / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle", "sample": f"{label}, fp64, {dt:.1f} s", "cpu_model": cpu_model()}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4", "c5", "probe"])
    ap.add_argument("--bits", type=int, default=4, help="c4, c5: code width (c5 is defined at 4)")
    ap.add_argument("--group", type=int, default=32, help="c4: group size")
    ap.add_argument("--tokens", type=int, default=16, help="c5: tokens per call")
    ap.add_argument("--factors16", action="store_true",
                    help="c5: alpha, beta of the merged layers stored as fp16 pairs (the configuration itself has fp32)")
    ap.add_argument("--shared", action="store_true",
                    help="c3: gate and up as one wide layer (they share x): qalora_forward_shared / backward_shared")
    ap.add_argument("--no-deployed", action="store_true",
                    help="c5, up to four tokens: read the training layout instead of the deployment stream")
    ap.add_argument("--out-dtype", default="bf16", choices=["bf16", "f32"])
    ap.add_argument("--no-keep", action="store_true",
                    help="backward re-reads x instead of the pooled activations the forward kept")
    ap.add_argument("--library", default=None,
                    help="measure another build of the library (e.g. an ablation variant made by "
                         "`python -m paper_2309_14717_amd.build --variant NAME -DQALORA_ABLATE=n`); "
                         "the output carries its name")
    ap.add_argument("--arm-every", type=int, default=None,
                    help="arm the kernel-timing events on every n-th timed step (default: 2 for runs of "
                         "up to 50 steps, else 4; 0: never, then the roofline has no kernel time)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=4096)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch the library's plain copy kernel (256 MiB, 4 times): the "
                         "yardstick for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the layer shards by tokens with one "
              "all-reduce of dA/dB per step; no multi-GPU path is built). Use --gpus 1.",
              file=sys.stderr)
        sys.exit(2)
    Layer.keep = not args.no_keep
    ARM_EVERY[0] = args.arm_every

    import torch
    from paper_2309_14717_amd import api, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.library:   # a measurement build; the binding itself has no such switch
        if not os.path.exists(args.library):
            sys.exit(f"bench.py: {args.library} not found")
        api.LIB_PATH = os.path.abspath(args.library)
    api.load()
    odt = torch.bfloat16 if args.out_dtype == "bf16" else torch.float32
    extras, cpu_baseline = {}, None
    if args.calibrate_copy:
        src = torch.ones(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(4):
            api.profile_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    if args.workload == "probe":
        rep = probe_report(torch, api)
        rep["two_stream_backward_c2"] = two_stream_backward(torch, api, synth)
        print(json.dumps(rep))
        return

    if args.workload in ("c1", "c2", "c4"):
        cfg = synth.CONFIGS[args.workload]
        if args.workload == "c4":
            cfg = cfg.scaled(bits=args.bits, group=args.group)
        L = Layer(api, torch, cfg, odt)

        def step():
            L.forward()
            L.backward()

        ms_per_step, kms, clk = run_steps(torch, api, step, args.steps, args.warmup, arm_every=ARM_EVERY[0])
        fl = layer_flops(cfg)
        total_flops = fl["fwd"] + fl["bwd"]
        kf, kb = kms[0], kms[1]
        dom = ("fwd", kf, fl["fwd_kernel"]) if kf >= kb else ("bwd", kb, fl["bwd_kernel"])
        achieved = dom[2] / (dom[1] * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": f"gemm_dq_kernel<{cfg.bits},{dom[0]}>",
                    "achieved": round(achieved, 2), "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(achieved / PEAK_MFMA_TFLOPS, 4), "avg_kernel_ms": round(dom[1], 4),
                    "fwd_kernel_ms": round(kf, 4), "bwd_kernel_ms": round(kb, 4),
                    **traffic_fields(f"gemm_dq_{args.workload}_pmc.txt")}
        roofline.update(clock_fields(clk[0 if dom[0] == "fwd" else 1], achieved))
        st = KERNEL_STATS.get(0 if dom[0] == "fwd" else 1)
        if st:
            roofline.update({"kernel_ms_median": st["median_ms"], "kernel_ms_min": st["min_ms"],
                             "kernel_samples": st["samples"],
                             "first_block_shader_cycles": st["block_cycles"]})
        if BLOCK_TIMELINE.get(0 if dom[0] == "fwd" else 1):
            roofline["block_timeline"] = BLOCK_TIMELINE[0 if dom[0] == "fwd" else 1]
        workload = (f"{cfg.name}: QA-LoRA linear fwd+bwd, T={cfg.tokens}, {cfg.d_in}x{cfg.d_out}, "
                    f"INT{cfg.bits} g={cfg.group}, rank {cfg.rank}, s={cfg.s}, x/dy bf16, outputs {args.out_dtype}")
        if not args.no_extras:
            beta_m = torch.empty_like(L.beta)
            L.beta_m = beta_m
            merge_ms = timed(torch, lambda: api.merge(L.desc, L.beta, L.A, L.B, out=beta_m))
            extras = {
                "fwd_ms": round(timed(torch, L.forward), 4),
                "bwd_ms": round(timed(torch, L.backward), 4),
                "quantize_ms": round(timed(torch, lambda: api.quantize(L.desc, L.W), 5), 4),
                "merge_ms": round(merge_ms, 4),
                "merge_GB/s": round(2 * L.beta.numel() * 4 / merge_ms / 1e6, 1),
                "post_merge_fwd_ms": round(timed(torch, L.forward_merged), 4),
            }
            if args.workload == "c2":
                # error-compensated code selection of the same layer under a seeded synthetic
                # Hessian (factorised by the framework: the library takes the factor)
                gen = torch.Generator(device="cuda").manual_seed(77)
                X = torch.randn((2 * cfg.d_in, cfg.d_in), generator=gen, device="cuda", dtype=torch.float64)
                H = X.T @ X / X.shape[0]
                H += 0.01 * torch.diag(H).mean() * torch.eye(cfg.d_in, device="cuda", dtype=torch.float64)
                U = torch.linalg.cholesky(torch.linalg.inv(H), upper=True).float().contiguous()
                del X, H
                extras["quantize_compensated_ms"] = round(
                    timed(torch, lambda: api.quantize_compensated(L.desc, L.W, U), 3, 1), 3)
                del U
                L.drop_w()
                extras["adamw_step_decoder_layer"] = adamw_layer_timing(torch, api)
                extras["small_token_post_merge_forward"] = small_token_table(torch, api, synth, odt)
        if not args.no_cpu_baseline:
            import oracle
            d = L.host
            n = min(args.cpu_sample_tokens, cfg.tokens)
            codes = api.unpack(L.desc, L.packed).cpu().numpy()
            al, be = L.alpha.cpu().numpy(), L.beta.cpu().numpy()
            cpu_baseline = cpu_oracle_baseline(
                [(lambda: oracle.forward(d["x"][:n], codes, al, be, cfg.group, d["A"], d["B"], cfg.s), fl["fwd"] * n / cfg.tokens),
                 (lambda: oracle.backward(d["dy"][:n], d["x"][:n], codes, al, be, cfg.group, d["A"], d["B"], cfg.s),
                  fl["bwd"] * n / cfg.tokens)],
                f"forward+backward of the first {n} of {cfg.tokens} tokens of the same layer")

    elif args.workload == "c3":
        if odt != torch.bfloat16:
            sys.exit("bench.py: workload c3 chains layers through bf16 activations; use --out-dtype bf16")
        blk = (MlpBlockShared if args.shared else MlpBlock)(api, torch, synth, odt)
        down, step = blk.down, blk.step

        ms_per_step, kms, clk = run_steps(torch, api, step, args.steps, args.warmup, arm_every=ARM_EVERY[0])
        fls = [layer_flops(c) for c in (synth.CONFIGS["c3_gate"], synth.CONFIGS["c3_up"], synth.CONFIGS["c3_down"])]
        total_flops = sum(f["fwd"] + f["bwd"] for f in fls)
        # armed events catch the first contraction of each direction: gate forward, down backward
        kf, kb = kms[0], kms[1]
        # (shared: the first forward contraction is the wide gate|up layer, twice the flops)
        cands = [("fwd 4096x22016", kf, fls[0]["fwd_kernel"] + fls[1]["fwd_kernel"]) if args.shared
                 else ("fwd 4096x11008", kf, fls[0]["fwd_kernel"]), ("bwd 11008x4096", kb, fls[2]["bwd_kernel"])]
        dom = max(cands, key=lambda c: c[1])
        achieved = dom[2] / (dom[1] * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": f"gemm_dq_kernel<4,{dom[0]}>", "achieved": round(achieved, 2),
                    "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_MFMA_TFLOPS, 4),
                    "avg_kernel_ms": round(dom[1], 4), "gate_fwd_kernel_ms": round(kf, 4),
                    "down_bwd_kernel_ms": round(kb, 4),
                    **(traffic_fields("gemm_dq_c3_shared_pmc.txt", "traffic_bytes_per_launch_fwd_wide")
                       if dom[0] == "fwd 4096x22016" else
                       traffic_fields("gemm_dq_c3_pmc.txt", "traffic_bytes_per_launch_" + dom[0][:3]))}
        roofline.update(clock_fields(clk[0 if dom[0].startswith("fwd") else 1], achieved))
        workload = ("c3: LLaMA-7B SwiGLU MLP block fwd+bwd, T=4096, gate/up 4096x11008 + down 11008x4096, "
                    f"INT4 g=32, rank 64, s=0.25, bf16 activations, outputs {args.out_dtype}; SwiGLU glue fused (one kernel each way)")
        cfg = synth.CONFIGS["c3_gate"]
        if args.shared:
            workload = workload.replace("c3:", "c3 (gate and up as one wide layer sharing x):")
        if not args.no_cpu_baseline:
            import oracle
            d = synth.make_inputs(cfg)
            n = min(256, cfg.tokens)
            codes, al, be = oracle.quantize(d["W"], cfg.bits, cfg.group)
            cpu_baseline = cpu_oracle_baseline(
                [(lambda: oracle.forward(d["x"][:n], codes, al, be, cfg.group, d["A"], d["B"], cfg.s),
                  fls[0]["fwd"] * n / cfg.tokens),
                 (lambda: oracle.backward(d["dy"][:n], d["x"][:n], codes, al, be, cfg.group, d["A"], d["B"], cfg.s),
                  fls[0]["bwd"] * n / cfg.tokens)],
                f"forward+backward of the gate projection on the first {n} of {cfg.tokens} tokens")

    else:  # c5
        T = args.tokens
        n_sets = 8
        dep = not args.no_deployed and not args.factors16
        cfg_u, ups = small_token_sets(torch, api, synth, "c5_up", n_sets, odt, args.bits, deployed=dep)
        cfg_d, downs = small_token_sets(torch, api, synth, "c5_down", n_sets, odt, args.bits, deployed=dep)
        fb = 2 if args.factors16 else 4
        if args.factors16:
            for Lr in ups + downs:
                Lr.fac16 = api.pack_factors16(Lr.desc, Lr.alpha, Lr.beta_m)
        xu, xd = ups[0].x[:T].contiguous(), downs[0].x[:T].contiguous()
        yu = torch.empty((T, cfg_u.d_out), dtype=odt, device="cuda")
        yd = torch.empty((T, cfg_d.d_out), dtype=odt, device="cuda")
        op = api.OP_FORWARD_FACTORS16 if args.factors16 else api.OP_FORWARD
        ws_u = torch.empty(api.workspace_bytes(ups[0].desc, T, op), dtype=torch.uint8, device="cuda")
        ws_d = torch.empty(api.workspace_bytes(downs[0].desc, T, op), dtype=torch.uint8, device="cuda")
        counter = [0]

        def step():
            i = counter[0] % n_sets
            counter[0] += 1
            ups[i].forward_merged(x=xu, y=yu, ws=ws_u)      # arms catch this kernel (first forward of the step)
            downs[i].forward_merged(x=xd, y=yd, ws=ws_d)

        streaming = T <= (32 if args.bits == 4 else 16)
        if streaming:
            # graph replays of whole rotations (see timed_graph); then a few eager steps with armed
            # events for the event-bracketed figure
            def one(i):
                def f():
                    ups[i].forward_merged(x=xu, y=yu, ws=ws_u)
                    downs[i].forward_merged(x=xd, y=yd, ws=ws_d)
                return f
            for _ in range(max(args.warmup, n_sets)):
                step()
            torch.cuda.synchronize()
            full = capture(torch, [one(i) for i in range(n_sets)])
            rem = capture(torch, [one(i) for i in range(args.steps % n_sets)]) if args.steps % n_sets else None
            SETTLE["steps"] = n_sets * settle(torch, full.replay)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps // n_sets):
                full.replay()
            if rem is not None:
                rem.replay()
            torch.cuda.synchronize()
            ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
            _, kms, clk = run_steps(torch, api, step, 14, 0, directions=(0,), arm_every=7)
        else:
            ms_per_step, kms, clk = run_steps(torch, api, step, args.steps, max(args.warmup, n_sets), directions=(0,), arm_every=7)
        total_flops = 2.0 * T * (cfg_u.d_in * cfg_u.d_out + cfg_d.d_in * cfg_d.d_out)
        by_u = forward_bytes(cfg_u, T, yu.element_size(), fb)
        by_step = by_u + forward_bytes(cfg_d, T, yd.element_size(), fb)
        k = kms[0]
        if streaming:  # the streaming kernels' range
            # A step is two launches of the streaming kernel with (to 0.1 %) the same algorithmic
            # bytes, back to back on one stream, so the average launch duration over the timed
            # region is half the step.  (An event pair around a single 30 us launch reads 3-5 us
            # high -- launch and marker latency that back-to-back launches overlap -- and is
            # reported beside it.)
            k_avg = ms_per_step / 2.0
            ach = by_step / 2.0 / k_avg / 1e6
            kname = "smallt4_kernel" if (T <= 4 or args.bits != 4) else "smallt_kernel"
            roofline = {"bound": "hbm", "kernel": f"{kname} (8192x22016 and 22016x8192 alternating)",
                        "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": round(ach / PEAK_HBM_GBS, 4), "avg_kernel_ms": round(k_avg, 5),
                        "event_bracketed_ms_8192x22016": round(k, 5),
                        **traffic_fields(("smallt4_c5_pmc.txt" if T <= 4 else "smallt_c5_pmc.txt")
                                         if (args.bits == 4 and not args.factors16 and T <= 16) else None)}
        else:
            ach = 2.0 * T * cfg_u.d_in * cfg_u.d_out / (k * 1e-3) / 1e12
            roofline = {"bound": "mfma", "kernel": f"gemm_dq_kernel<{args.bits},fwd> (8192x22016)", "achieved": round(ach, 2),
                        "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": round(ach / PEAK_MFMA_TFLOPS, 4),
                        "avg_kernel_ms": round(k, 5), "hbm_GB/s": round(by_u / k / 1e6, 1), "traffic": None,
                        "traffic_source": None}
            roofline.update(clock_fields(clk[0], ach))
        extras = {"GB/s_whole_step": round(by_step / ms_per_step / 1e6, 1),
                  "frac_hbm_whole_step": round(by_step / ms_per_step / 1e6 / PEAK_HBM_GBS, 4),
                  "bytes_per_step": by_step, "weight_sets": n_sets}
        workload = (f"c5: post-merge forward, T={T}, 8192x22016 then 22016x8192, INT{args.bits} g=32, merged beta, "
                    f"x bf16, outputs {args.out_dtype}, {n_sets} weight sets rotated"
                    + (", alpha and beta stored as fp16 pairs" if args.factors16 else "")
                    + (", deployed (qalora_deploy)" if (dep and (T <= 4 or T > 32) and args.bits == 4) else ""))
        cfg = cfg_u
        if not args.no_cpu_baseline:
            import oracle
            L0 = ups[0]
            n = min(T, 16)
            codes = api.unpack(L0.desc, L0.packed).cpu().numpy()
            al, be = L0.alpha.cpu().numpy(), L0.beta_m.cpu().numpy()
            xh = L0.x[:n].float().cpu().numpy()
            cpu_baseline = cpu_oracle_baseline(
                [(lambda: oracle.forward(xh, codes, al, be, cfg.group), 2.0 * n * cfg.d_in * cfg.d_out)],
                f"post-merge forward of the 8192x22016 layer on {n} tokens")

    value = total_flops / (ms_per_step * 1e-3) / 1e12
    out = {
        "metric": METRIC, "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "warmup_settle_steps": SETTLE.get("steps", 0), "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f16" if args.workload != "c5" or args.tokens > (32 if args.bits == 4 else 16) else "bf16",
        "data": "synthetic",
        "config": {"workload": workload, "flops_per_step": total_flops,
                   "frac_of_mfma_peak": round(value / PEAK_MFMA_TFLOPS, 4),
                   "backward_reads": ("n/a" if args.workload == "c5" else
                                      ("pooled activations kept by the forward" if Layer.keep else "x"))},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "extras": extras,
    }
    if args.library:
        out["config"]["library"] = os.path.basename(args.library) + " (a measurement build: results may be wrong on purpose)"
    print(json.dumps(out))


if __name__ == "__main__":
    main()
