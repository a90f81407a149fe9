#!/usr/bin/env python3
"""Benchmark of the ATOMO encode/decode hot path on one MI355X.

A "step" is one pass of the whole path over one synthetic ResNet-18 layer-set gradient (21 fp32
matrices, 11,164,352 elements, rank-8 geometric signal + N(0, 1e-3^2) noise): Spectral-ATOMO
encode with budget s = 3 per layer (SVD -> Algorithm 1 -> Philox Bernoulli -> pack), then decode
of the 21 messages to dense gradients.  Inputs are resident in HBM before the timed region.

Prints ONE JSON line.  `value` = gradient elements encoded+decoded per second.
`roofline` prices the dominant kernel (by GPU time) against its bound; the per-kernel GPU times
come from HIP events recorded around every launch, in a second pass over the same K steps right
after the timed pass (the events cost a few microseconds per launch, so they stay out of `value`).
`cpu_baseline` is the fp64 oracle, as it stands, timed on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3        # MI355X published dense fp32 matrix peak
PEAK_FP32_VALU_TFLOPS = 78.6         # 256 CUs x 4 SIMD x 16 lanes x 2 flop x 2.4 GHz (packed fp32 off)
PEAK_HBM_GBS = 8000.0


def algorithmic_flops(shapes, sweeps):
    """Contraction flops of blocked one-sided Jacobi on real data, no padding:
    per sweep and matrix, Gram 4 M r^2, row update 4 M r^2, accumulation of the rotations 4 r^3."""
    gram = upd = 0.0
    for (m, n), sw in zip(shapes, sweeps):
        r, M = min(m, n), max(m, n)
        gram += sw * 4.0 * M * r * r
        upd += sw * (4.0 * M * r * r + 4.0 * r ** 3)
    return gram, upd


def eig_flops(shapes, sweeps, inner_sweeps=2):
    """Vector-ALU flops of the 64x64 two-sided Jacobi solves (2016 rotations per inner sweep, each
    touching 2 rows + 2 columns of the Gram matrix and 2 columns of the accumulator: 3 * 64 * 6 flops)
    plus the Newton-Schulz step (2 products of 64^3)."""
    total = 0.0
    for (m, n), sw in zip(shapes, sweeps):
        r = min(m, n)
        nb = -(-r // 32)
        nb2 = nb + (nb & 1)
        visits = sw * (nb2 - 1) * (nb2 // 2)
        total += visits * (inner_sweeps * 2016 * 3 * 64 * 6 + 2 * 2 * 64 ** 3)
    return total


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (the design note in DESIGN.md says "
              "how it would shard); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1806_04090_amd import binding, inputs

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    ctx = binding.Context(0)
    S, SEED = 3.0, 0
    shapes = list(inputs.RESNET18_SHAPES)
    host = inputs.resnet18_layer_set(0)
    mats = [torch.from_numpy(g).cuda() for g in host]
    n_elem = sum(g.size for g in host)
    msgs = [binding.alloc_svd_message(m, n, binding.default_capacity(S, min(m, n)), "cuda") for m, n in shapes]
    outs = [torch.empty(m, n, dtype=torch.float32, device="cuda") for m, n in shapes]
    groups = [[m] for m in msgs]

    def step():
        binding.atomo_encode_svd(ctx, mats, S, SEED, 0, msgs=msgs)
        binding.atomo_decode_svd_batch(ctx, groups, 1.0, outs=outs)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    status, max_sweeps = ctx.status()
    if status != 0:
        print(f"warm-up reported status {status}", file=sys.stderr)
        sys.exit(1)
    sweeps = ctx.svd_sweeps(len(mats))

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps

    # second pass, same K steps, with HIP events around every kernel launch
    ctx.profile_enable(True)
    prof = {}
    tp0 = time.perf_counter()
    for _ in range(args.steps):
        step()
        for name, (ms, cnt) in ctx.profile_read().items():
            a, b = prof.get(name, (0.0, 0))
            prof[name] = (a + ms, b + cnt)
    torch.cuda.synchronize()
    ms_per_step_profiled = (time.perf_counter() - tp0) * 1e3 / args.steps
    ctx.profile_enable(False)

    gram_fl, upd_fl = algorithmic_flops(shapes, sweeps)
    per_step_ms = {k: v[0] / args.steps for k, v in prof.items() if v[1]}
    launches = {k: v[1] / args.steps for k, v in prof.items() if v[1]}
    dominant = max(per_step_ms, key=per_step_ms.get)
    work = {
        "svd_gram": ("mfma", gram_fl, PEAK_FP32_MFMA_TFLOPS, "TFLOP/s"),
        "svd_update": ("mfma", upd_fl, PEAK_FP32_MFMA_TFLOPS, "TFLOP/s"),
        "svd_eig": ("alu", eig_flops(shapes, sweeps), PEAK_FP32_VALU_TFLOPS, "TFLOP/s"),
        "decode_svd": ("hbm", 4.0 * n_elem, PEAK_HBM_GBS, "GB/s"),
    }
    bound, amount, peak, unit = work.get(dominant, ("alu", 0.0, PEAK_FP32_VALU_TFLOPS, "TFLOP/s"))
    dom_ms = per_step_ms[dominant]
    achieved = amount / (dom_ms * 1e-3) / (1e12 if unit == "TFLOP/s" else 1e9)
    roofline = {
        "kernel": dominant, "bound": bound, "achieved": round(achieved, 3), "peak": peak, "unit": unit,
        "frac": round(achieved / peak, 5), "traffic": None,
        "avg_launch_us": round(dom_ms * 1e3 / launches[dominant], 2), "launches_per_step": launches[dominant],
        "per_step_ms_by_kernel": {k: round(v, 4) for k, v in sorted(per_step_ms.items())},
        "ms_per_step_with_events": round(ms_per_step_profiled, 4),
        "jacobi_sweeps_per_layer": sweeps,
        "encode_contraction": {
            "flops_per_step": gram_fl + upd_fl,
            "tflops_over_mfma_kernels": round((gram_fl + upd_fl) / ((per_step_ms.get("svd_gram", 0) +
                                              per_step_ms.get("svd_update", 0)) * 1e-3) / 1e12, 3),
            "tflops_over_whole_encode": round((gram_fl + upd_fl) / (sum(v for k, v in per_step_ms.items()
                                              if k.startswith("svd_")) * 1e-3) / 1e12, 3),
        },
    }

    cpu = None
    if not args.no_cpu_baseline and os.environ.get("ATOMO_BENCH_SKIP_CPU") != "1":
        cpu = cpu_baseline(host, S, SEED)

    line = {
        "metric": "gradient elements encoded+decoded/sec (SVD-ATOMO, ResNet-18 set)",
        "value": n_elem * args.steps / elapsed, "unit": "elements/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "resnet18_layer_set_svd_s3: 21 fp32 matrices (CIFAR-10 sizing), 11,164,352 elements, "
                               "rank-8 signal 0.5^k + N(0,1e-3^2), budget s=3 per layer, encode + decode",
                   "elements_per_step": n_elem, "budget_s": S, "philox_seed": SEED},
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))


def cpu_baseline(host_mats, s, seed):
    """The oracle (fp64, plain C, as it stands) on the same workload: one encode + decode of the whole
    21-layer set, host threads over layers (largest layers first so the threads stay busy)."""
    from concurrent.futures import ThreadPoolExecutor

    import oracle

    sample = sorted(enumerate(host_mats), key=lambda item: -item[1].size * min(item[1].shape))
    cores = min(len(sample), max(1, min(16, os.cpu_count() or 1)))

    def one(item):
        j, g = item
        enc = oracle.encode_svd(g, s, seed, j)
        oracle.decode_svd([enc], g.shape[0], g.shape[1])
        return g.size

    oracle.svd(np.eye(2))                      # load the library outside the timed region
    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=cores) as pool:
        n_elem = sum(pool.map(one, sample))
    dt = time.perf_counter() - t0
    return {"value": n_elem / dt, "unit": "elements/s", "cores": cores, "kind": "oracle",
            "sample": f"one full step (all 21 layers, {n_elem} elements), encode + decode, {dt:.1f} s wall on "
                      f"{cores} threads"}


if __name__ == "__main__":
    main()
