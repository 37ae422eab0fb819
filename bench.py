#!/usr/bin/env python3
"""Benchmark of the QA-LoRA adapted linear layer on one MI355X.

One "step" = one adapted forward (y = x W~ + s (pool(x) A) B) plus one backward
(dx, dA, dB) of a single linear layer through the C-ABI library, on seeded synthetic
tensors already resident in HBM.  Quantization of W is setup and is not timed; merge and
the post-merge forward are reported separately in "extras".

Prints ONE JSON line (see README for the fields).
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
PEAK_HBM_GBS = 8000.0


def layer_flops(cfg):
    """Algorithmic flops of one forward + backward (two dense contractions, no dW product,
    plus the adapter products); unpack / dequant / pooling count zero."""
    T, di, do, r, L = cfg.tokens, cfg.d_in, cfg.d_out, cfg.rank, cfg.groups
    main = 2.0 * T * di * do
    fwd_adapter = 2.0 * T * L * r + 2.0 * T * r * do
    bwd_adapter = 2 * (2.0 * T * r * do) + 2 * (2.0 * T * L * r)
    return dict(fwd=main + fwd_adapter, bwd=main + bwd_adapter,
                fwd_kernel=main + 2.0 * T * r * do,          # x W~ + (sU) B
                bwd_kernel=main + 2.0 * T * L * r)           # dy W~^T + dU A^T (unpooled)


def read_traffic(workload):
    """HBM bytes per launch of the dominant kernel, from the committed rocprofv3 --pmc summary."""
    path = os.path.join(ROOT, "profiles", f"gemm_dq_{workload}_pmc.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c2")
    ap.add_argument("--out-dtype", default="bf16", choices=["bf16", "f32"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=4096)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the layer shards by tokens with one "
              "all-reduce of dA/dB per step; no multi-GPU path is built). Use --gpus 1.",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2309_14717_amd import api, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    api.load()
    cfg = synth.CONFIGS[args.workload]
    d = synth.make_inputs(cfg)
    dev = "cuda"
    W = torch.from_numpy(d["W"]).to(dev)
    x = torch.from_numpy(d["x"]).to(dev).to(torch.bfloat16)
    dy = torch.from_numpy(d["dy"]).to(dev).to(torch.bfloat16)
    A = torch.from_numpy(d["A"]).to(dev)
    B = torch.from_numpy(d["B"]).to(dev)
    desc = api.make_desc(cfg.d_in, cfg.d_out, cfg.bits, cfg.group, cfg.rank, cfg.s)

    tq = time.perf_counter()
    packed, alpha, beta = api.quantize(desc, W)
    torch.cuda.synchronize()
    quantize_ms_cold = (time.perf_counter() - tq) * 1e3

    odt = torch.bfloat16 if args.out_dtype == "bf16" else torch.float32
    y = torch.empty((cfg.tokens, cfg.d_out), dtype=odt, device=dev)
    dx = torch.empty((cfg.tokens, cfg.d_in), dtype=odt, device=dev)
    dA, dB = torch.zeros_like(A), torch.zeros_like(B)
    ws_f = torch.empty(api.workspace_bytes(desc, cfg.tokens, api.OP_FORWARD), dtype=torch.uint8, device=dev)
    ws_b = torch.empty(api.workspace_bytes(desc, cfg.tokens, api.OP_BACKWARD), dtype=torch.uint8, device=dev)

    def step():
        api.forward(desc, x, packed, alpha, beta, A, B, ws=ws_f, y=y)
        api.backward(desc, dy, x, packed, alpha, beta, A, B, dA=dA, dB=dB, ws=ws_b, dx=dx)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- timed region: exactly `steps` steps, kernel events armed inside the library ----
    kt_f = api.KernelTimer(0, args.steps)
    kt_b = api.KernelTimer(1, args.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        kt_f.arm()
        kt_b.arm()
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    kf = float(np.mean(kt_f.elapsed_ms()))
    kb = float(np.mean(kt_b.elapsed_ms()))
    kt_f.close()
    kt_b.close()

    fl = layer_flops(cfg)
    total_flops = fl["fwd"] + fl["bwd"]
    value = total_flops / (ms_per_step * 1e-3) / 1e12

    dom = ("fwd", kf, fl["fwd_kernel"]) if kf >= kb else ("bwd", kb, fl["bwd_kernel"])
    achieved = dom[2] / (dom[1] * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": f"gemm_dq_kernel<{cfg.bits},{dom[0]}>",
                "achieved": round(achieved, 2), "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / PEAK_MFMA_TFLOPS, 4),
                "avg_kernel_ms": round(dom[1], 4),
                "fwd_kernel_ms": round(kf, 4), "bwd_kernel_ms": round(kb, 4),
                "traffic": read_traffic(args.workload)}

    # ---- extras: the rows of the path that are not per-step (untimed toward `value`) ----
    def timed(fn, n=20):
        fn()
        torch.cuda.synchronize()
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s.record()
        for _ in range(n):
            fn()
        e.record()
        torch.cuda.synchronize()
        return s.elapsed_time(e) / n

    beta_m = torch.empty_like(beta)
    extras = {
        "fwd_ms": round(timed(lambda: api.forward(desc, x, packed, alpha, beta, A, B, ws=ws_f, y=y)), 4),
        "bwd_ms": round(timed(lambda: api.backward(desc, dy, x, packed, alpha, beta, A, B, dA=dA, dB=dB, ws=ws_b, dx=dx)), 4),
        "quantize_ms": round(timed(lambda: api.quantize(desc, W), 5), 4),
        "merge_ms": round(timed(lambda: api.merge(desc, beta, A, B, out=beta_m)), 4),
        "post_merge_fwd_ms": round(timed(lambda: api.forward(desc, x, packed, alpha, beta_m, ws=ws_f, y=y)), 4),
    }

    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        n = min(args.cpu_sample_tokens, cfg.tokens)
        codes = api.unpack(desc, packed).cpu().numpy()
        al, be = alpha.cpu().numpy(), beta.cpu().numpy()
        tc = time.perf_counter()
        oracle.forward(d["x"][:n], codes, al, be, cfg.group, d["A"], d["B"], cfg.s)
        oracle.backward(d["dy"][:n], d["x"][:n], codes, al, be, cfg.group, d["A"], d["B"], cfg.s)
        dt = time.perf_counter() - tc
        cpu_baseline = {"value": round(total_flops * (n / cfg.tokens) / dt / 1e12, 6), "unit": "TFLOP/s",
                        "cores": oracle.num_threads(), "kind": "oracle",
                        "sample": f"forward+backward of the first {n} of {cfg.tokens} tokens of the "
                                  f"same layer, fp64, {dt:.1f} s"}

    out = {
        "metric": "QA-LoRA linear fwd+bwd TFLOP/s & % of MFMA/HBM roofline, LLaMA-7B shapes",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: QA-LoRA linear fwd+bwd, T={cfg.tokens}, "
                               f"{cfg.d_in}x{cfg.d_out}, INT{cfg.bits} g={cfg.group}, rank {cfg.rank}, "
                               f"s={cfg.s}, x/dy bf16, outputs {args.out_dtype}",
                   "flops_per_step": total_flops, "frac_of_mfma_peak": round(value / PEAK_MFMA_TFLOPS, 4)},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "extras": extras,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
