#!/usr/bin/env python3
"""Benchmark of the ATOMO encode/decode hot path on one MI355X.

A "step" is one pass of the whole path over one synthetic ResNet-18 layer-set gradient (21 fp32
matrices, 11,164,352 elements, rank-8 geometric signal + N(0, 1e-3^2) noise): Spectral-ATOMO
encode with budget s = 3 per layer (SVD -> Algorithm 1 -> Philox Bernoulli -> pack), then decode
of the 21 messages to dense gradients.  Inputs are resident in HBM before the timed region.

Prints ONE JSON line.  `value` = gradient elements encoded+decoded per second.
`roofline` prices the encode as a whole: contraction flops the algorithm executes on real data (no
padding, measured sweep counts) over the GPU time of one encode, taken inside the timed region from two HIP
events per step (one before the encode, one after it, on the stream the library launches on), against the
fp32 matrix-core peak.  `roofline.by_kernel_event_pass` breaks the step down by kernel class from a second pass
over the same K steps with events around every launch (slower than the timed pass: the events cost a few
microseconds per launch and the two streams of the encoder overlap; for detail, not for `achieved`).
`cpu_baseline` is the fp64 oracle, as it stands, timed on this machine's host cores.

`--leg NAME` runs one part alone, for profiling: `headline` (the timed steps and nothing else; prints the same
JSON line with the other legs null), or one of `entrywise`, `aggregate`, `section6`, `single`, `batch64` (prints
that leg's object only).
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
PEAK_FP32_VALU_TFLOPS = 157.3        # published vector fp32 peak (packed); 78.6 for the unpacked code built here
PEAK_HBM_GBS = 8000.0


def layer_geometry(m, n):
    """(r, M, Gram-space?) of one layer as the library schedules it: 32-row blocks, an even number of
    them, and from sixteen blocks up the sweeps run on the r x r Gram matrix instead of the data."""
    r, M = min(m, n), max(m, n)
    nb = -(-r // 32)
    nb2 = nb + (nb & 1)
    return r, M, nb2 >= 16


def block_rows(r):
    """Real rows in each 32-row block of a layer with r vectors, the zero block of an odd count included."""
    nb = -(-r // 32)
    rows = [min(32, r - 32 * b) for b in range(nb)]
    return rows + [0] * (nb & 1)


ROTATION_UNITS = 1.0 + 2.0 * 17.0 / 32.0   # vectors of 64 that one rotation of a Jacobi step updates, see executed_work


def executed_work(shapes, sweeps, refreshes, pair_visits, jacobi_steps, row_update_tiles, n_elem, kept_atoms):
    """Arithmetic and bytes the algorithm executes on real data (no padding) per step, by kernel class.

    Thin layers (r <= 32) are streaming passes over the data (svd_thin), priced by their bytes.
    A sweep visits every pair (i, j) of the layer's 32-row blocks once, n_i + n_j real rows per pair.
    Data-space layers (32 < r <= 480), one launch of svd_rowgram per tick (svd_update): the row update, 2 x 64 x 64 x 64
    per 64 x 64 tile of [A | T] that was rotated, counted on the device (pairs found converged are left alone), and
    the Gram matrices of the next tick's pairs, three of the four quadrants each: 2 M (n_i^2 + n_i n_j + n_j^2) per
    visit.  The Gram matrices of the first tick are a launch of their own (svd_gram).  Layers of 225 rows and more
    also form all of A A^T  M r (r + 64) at each check of the whole matrix near the end (the refreshes they
    report; svd_refresh).
    Gram-space layers, per refresh (svd_refresh): upper-triangular tiles of A A^T  M r (r + 64), and (every
    refresh but the first) A <- T A and T <- T T_old, 2 r^2 (M + r); per tick of a sweep, inside the svd_eig
    launches: C <- D^T C D  256 r^2 and Tgs <- D^T Tgs  128 r^2 (D block-diagonal in 64 x 64 blocks), and per pair
    problem the 32x32 block between its two row blocks, which it brings up to date itself (two chained products; the
    two diagonal blocks come from the pair problems of the tick before).
    64 x 64 eigen-solves: 32 rotations per Jacobi step (63 steps when every index pair is rotated, 32 when only
    the pairs that couple the two blocks are), each ROTATION_UNITS x 64 x 6 flops on the vector ALU: 64 x 6 for the
    columns of the accumulator, and for the rows and the columns of the symmetric block 2 x 64 x 6 x 17/32, because the
    register-resident steps update 17 of its 32 block diagonals (one triangle) and mirror the rest.  (The 31 steps of a
    full round that go through LDS update the whole block, 3 x 64 x 6: they are priced like the others, an under-count.)
    Plus a Newton-Schulz step of two 64^3 products per solve.  The
    svd_eig class is priced as a whole (vector-ALU rotations + the MFMA work its launches carry) against the
    157.3 TFLOP/s that is both the fp32 vector and the fp32 matrix peak.
    """
    gram = gram_first = refresh = twosided = catchup = thin_bytes = 0.0
    for (m, n), sw, rf in zip(shapes, sweeps, refreshes):
        r, M, gs = layer_geometry(m, n)
        if r <= 32:
            # thin layers: largest-entry pass, first Gram pass, one read + write per rotation, gather of the kept atoms
            thin_bytes += 4.0 * M * r * (3 + 2 * sw)
            continue
        rows = block_rows(r)
        nb2 = len(rows)
        if gs:
            visits = sw * (nb2 - 1) * (nb2 // 2)
            refresh += rf * M * r * (r + 64.0) + max(rf - 1, 0) * 2.0 * r * r * (M + r)
            twosided += sw * (nb2 - 1) * 384.0 * r * r
            # every pair problem but the first after a refresh forms its block from three 32x32 products
            catchup += max(visits - rf * (nb2 // 2), 0) * 2.0 * (32 * 64 * 64 + 32 * 64 * 32)
        else:
            quadrants = lambda i, j: 2.0 * M * (rows[i] ** 2 + rows[i] * rows[j] + rows[j] ** 2)
            first = [(nb2 - 1, 0)] + [(k, nb2 - 1 - k) for k in range(1, nb2 // 2)]    # the pairs of round 0
            gram_first += sum(quadrants(i, j) for i, j in first)
            gram += sw * sum(quadrants(i, j) for i in range(nb2) for j in range(i + 1, nb2)) - sum(quadrants(i, j) for i, j in first)
            refresh += rf * M * r * (r + 64.0)
    upd = row_update_tiles * 2.0 * 64 ** 3 + gram
    eig = jacobi_steps * 32 * ROTATION_UNITS * 64 * 6 + pair_visits * 2 * 2 * 64 ** 3 + twosided + catchup
    decode_bytes = 4.0 * n_elem + sum(4.0 * k * (m + n + 1) for (m, n), k in zip(shapes, kept_atoms))
    return {
        "svd_gram": ("mfma", gram_first, PEAK_FP32_MFMA_TFLOPS, "TFLOP/s"),
        "svd_update": ("mfma", upd, PEAK_FP32_MFMA_TFLOPS, "TFLOP/s"),
        "svd_refresh": ("mfma", refresh, PEAK_FP32_MFMA_TFLOPS, "TFLOP/s"),
        "svd_eig": ("alu", eig, PEAK_FP32_VALU_TFLOPS, "TFLOP/s"),
        "svd_prepare": ("hbm", 12.0 * n_elem, PEAK_HBM_GBS, "GB/s"),
        "svd_finalize": ("hbm", 4.0 * n_elem, PEAK_HBM_GBS, "GB/s"),
        "svd_thin": ("hbm", thin_bytes, PEAK_HBM_GBS, "GB/s"),
        "decode_svd": ("hbm", decode_bytes, PEAK_HBM_GBS, "GB/s"),
    }


def profiled_traffic_bytes(kernel):
    """HBM-side bytes of row `kernel` for this workload, from the committed rocprofv3 --pmc summary (FETCH_SIZE +
    WRITE_SIZE, each scaled by what the counter reads for a plain copy of known size; section "ResNet-18 steps
    only" of profiles/resnet18_svd_encode_hbm_traffic.md; the row "encode" is the sum over all launches of one
    encode).  bench.py cannot run the profiler on itself; None if the summary is not there."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "resnet18_svd_encode_hbm_traffic.md")
    try:
        text = open(path).read()
    except OSError:
        return None
    marker = text.find("## ResNet-18 steps only")
    if marker < 0:
        return None
    for row in text[marker:].splitlines():
        cells = [c.strip() for c in row.split("|")]
        if len(cells) >= 5 and cells[1] == kernel:
            try:
                return (float(cells[3]) + float(cells[4])) * 1024.0 * 1024.0
            except ValueError:
                return None
    return None


def dense_equivalent_flops(shapes, sweeps):
    """The contraction count of textbook blocked one-sided Jacobi on the data, sweeps x (8 M r^2 + 4 r^3) per layer:
    what the same number of sweeps would cost without the Gram-space reformulation.  These flops are not executed
    by the library; the figure is context only and enters no roofline fraction."""
    return sum(sw * (8.0 * max(m, n) * min(m, n) ** 2 + 4.0 * min(m, n) ** 3) for (m, n), sw in zip(shapes, sweeps))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-entrywise", action="store_true", help="skip the entry-wise and 16-worker decode legs")
    ap.add_argument("--no-adaptive", action="store_true",
                    help="enqueue the launches of all max_sweeps sweeps in every step (atomo_svd_options.adaptive = 0)")
    ap.add_argument("--leg", choices=["headline", "entrywise", "aggregate", "section6", "single", "batch64"], default=None,
                    help="run this part alone (for a profiler): `headline` prints the usual line without the other "
                         "legs, the others print their own object only")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run five plain device copies of 1 GiB, the known-size reference that scales the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this library has no multi-GPU path (layers are independent units and the "
              "Philox stream of (worker, layer) makes any assignment reproduce the same masks); run with --gpus 1",
              file=sys.stderr)
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
    if args.leg and args.leg != "headline":
        if args.leg == "entrywise":
            result = entrywise_leg(ctx, torch, binding, inputs)
        elif args.leg == "aggregate":
            result = aggregate_decode_leg(ctx, torch, binding, inputs, shapes, S, SEED)
        elif args.leg == "section6":
            result = section6_leg(ctx, torch, binding, inputs, S, SEED)
        elif args.leg == "single":
            result = single_layer_leg(ctx, torch, binding, inputs)
        else:
            result = batch64_leg(ctx, torch, binding, inputs, not args.no_cpu_baseline)
        if args.calibration_copy:
            calibration_copy(torch)
        print(json.dumps({"leg": args.leg, "result": result}))
        return
    headline_only = args.leg == "headline" or args.no_entrywise
    host = inputs.resnet18_layer_set(0)
    mats = [torch.from_numpy(g).cuda() for g in host]
    n_elem = sum(g.size for g in host)
    msgs = [binding.alloc_svd_message(m, n, binding.default_capacity(S, min(m, n)), "cuda") for m, n in shapes]
    outs = [torch.empty(m, n, dtype=torch.float32, device="cuda") for m, n in shapes]
    groups = [[m] for m in msgs]

    # a training loop encodes the same layer set step after step: `adaptive = 1` lets the library enqueue the sweeps
    # that the steps before needed plus one, instead of the launches of all 16 allowed sweeps (most of which find
    # nothing to do); a step that fell short would be reported by the status read after the timed region
    ADAPTIVE = 0 if args.no_adaptive else 1

    def step():
        binding.atomo_encode_svd(ctx, mats, S, SEED, 0, msgs=msgs, adaptive=ADAPTIVE)
        binding.atomo_decode_svd_batch(ctx, groups, 1.0, outs=outs)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    status, max_sweeps = ctx.status()
    if status != 0:
        print(f"warm-up reported status {status}", file=sys.stderr)
        sys.exit(1)
    sweeps = ctx.svd_sweeps(len(mats))
    refreshes = ctx.svd_refreshes(len(mats))
    kept_atoms = [int(m.count.item()) for m in msgs]

    # two HIP events per step on the launching stream (the encoder's internal stream is forked from and joined
    # back into it): GPU time of the encode alone, measured inside the timed region
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        ev[i][0].record()
        binding.atomo_encode_svd(ctx, mats, S, SEED, 0, msgs=msgs, adaptive=ADAPTIVE)
        ev[i][1].record()
        binding.atomo_decode_svd_batch(ctx, groups, 1.0, outs=outs)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    encode_ms = sum(a.elapsed_time(b) for a, b in ev) / args.steps
    status, _ = ctx.status()
    if status != 0:
        print(f"timed steps reported status {status}", file=sys.stderr)
        sys.exit(1)

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
    ctx.status()
    step()                                      # one step between two status reads: counters of exactly one step
    ctx.status()
    pair_visits, jacobi_steps, row_update_tiles = ctx.last_counters()

    per_step_ms = {k: v[0] / args.steps for k, v in prof.items() if v[1]}
    launches = {k: v[1] / args.steps for k, v in prof.items() if v[1]}
    work = executed_work(shapes, sweeps, refreshes, pair_visits, jacobi_steps, row_update_tiles, n_elem, kept_atoms)
    rotations = jacobi_steps * 32 * ROTATION_UNITS * 64 * 6
    # contraction flops executed on the matrix cores in one encode (the vector-ALU rotations are reported beside them)
    contraction = sum(work[k][1] for k in ("svd_gram", "svd_update", "svd_refresh")) + work["svd_eig"][1] - rotations
    by_kernel = {}
    for k, v in sorted(per_step_ms.items()):
        kb, ka, kp, ku = work[k]
        rate = ka / (v * 1e-3) / (1e12 if ku == "TFLOP/s" else 1e9)
        by_kernel[k] = {"ms": round(v, 4), "scopes": launches[k], "bound": kb, "achieved": round(rate, 3), "unit": ku,
                        "frac": round(rate / kp, 5)}
    achieved = contraction / (encode_ms * 1e-3) / 1e12
    dense_equivalent = dense_equivalent_flops(shapes, sweeps)
    roofline = {
        "kernel": "atomo_encode_svd (all launches of one encode of the 21-layer set)",
        "bound": "mfma", "achieved": round(achieved, 3), "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
        "frac": round(achieved / PEAK_FP32_MFMA_TFLOPS, 5),
        "encode_gpu_ms": round(encode_ms, 4),
        "executed_contraction_flops_per_encode": contraction,
        "vector_alu_rotation_flops_per_encode": rotations,
        "traffic": profiled_traffic_bytes("encode"),
        "traffic_unit": "HBM-side bytes per encode, all launches (rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE, scaled by a plain "
                        "copy of known size; read from the committed summary in profiles/, not measured by this run)",
        "jacobi_sweeps_per_layer": sweeps,
        "gram_refreshes_per_layer": refreshes,
        "eigen_solves_per_step": pair_visits, "jacobi_steps_per_step": jacobi_steps,
        "row_update_tiles_per_step": row_update_tiles,
        "by_kernel_event_pass": by_kernel,
        "ms_per_step_event_pass": round(ms_per_step_profiled, 4),
        # what the same sweep counts would cost as textbook blocked one-sided Jacobi on the data,
        # sweeps x (8 M r^2 + 4 r^3): flops this library does NOT execute (it sweeps on the r x r Gram matrix)
        "dense_equivalent_not_executed": {
            "flops_same_sweeps": dense_equivalent,
            "tflops_over_encode": round(dense_equivalent / (encode_ms * 1e-3) / 1e12, 3),
        },
    }
    entrywise = None if headline_only else entrywise_leg(ctx, torch, binding, inputs)
    aggregate = None if headline_only else aggregate_decode_leg(ctx, torch, binding, inputs, shapes, S, SEED)
    section6 = None if headline_only else section6_leg(ctx, torch, binding, inputs, S, SEED)
    single = None if args.leg == "headline" else single_layer_leg(ctx, torch, binding, inputs)
    batch64 = None if headline_only else batch64_leg(ctx, torch, binding, inputs, not args.no_cpu_baseline)
    # What a plain device-to-device copy reaches on this GPU (1 GiB, so nothing is served from a cache): context for
    # the HBM fractions above, which are all taken against the published 8 TB/s.
    copy_gbs = None
    if not headline_only:
        src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        copy_gbs = round(5 * 2.0 * src.numel() * 4 / (time.perf_counter() - t0) / 1e9, 1)
        del src, dst
    if args.calibration_copy:
        calibration_copy(torch)

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
                   "elements_per_step": n_elem, "budget_s": S, "philox_seed": SEED,
                   "svd_options": {"max_sweeps": 16, "adaptive": ADAPTIVE}},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "entrywise": entrywise,
        "decode_average_16_workers": aggregate,
        "section6_reshape": section6,
        "single_conv_layer_64x576": single,
        "batch_of_64_matrices_512x4608": batch64,
        "plain_copy_read_plus_write_gbs": copy_gbs,
        "fp32_mfma_loop_tflops": None if args.leg == "headline" else round(ctx.measure_mfma_fp32(), 1),
    }
    print(json.dumps(line))


def calibration_copy(torch):
    """Five plain device-to-device copies of 1 GiB: the transfer of known size against which the FETCH_SIZE and
    WRITE_SIZE counters of a rocprofv3 --pmc run of this script are scaled."""
    src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(5):
        dst.copy_(src)
    torch.cuda.synchronize()


def aggregate_decode_leg(ctx, torch, binding, inputs, shapes, s, seed, workers=16, reps=20):
    """Parameter-server side of the 16-worker configuration, outside the timed steps of the headline metric:
    every layer decoded from its 16 messages (data seeds 0..15, about 48 atoms per layer) and averaged, all 21
    layers in one launch.  GPU time of the decode launch from HIP events; the rank-K update runs on the matrix
    cores (2 m n K flops) and writes each output once (4 B per element)."""
    # the 16 gradients are encoded in one call (stream id = worker, layer): with 336 matrices per launch the chip is
    # full, where one gradient alone leaves most of it idle along the chain of dependent Jacobi rounds
    all_mats = [torch.from_numpy(g).cuda() for w in range(workers) for g in inputs.resnet18_layer_set(w)]
    ids = [inputs.worker_stream(w, j) for w in range(workers) for j in range(len(shapes))]
    flat_msgs = None
    for _ in range(2):
        flat_msgs = binding.atomo_encode_svd(ctx, all_mats, s, seed, 0, msgs=flat_msgs, stream_ids=ids)
    torch.cuda.synchronize()
    if ctx.status()[0] != 0:
        return None
    t0 = time.perf_counter()
    for _ in range(3):
        binding.atomo_encode_svd(ctx, all_mats, s, seed, 0, msgs=flat_msgs, stream_ids=ids)
    torch.cuda.synchronize()
    enc16 = (time.perf_counter() - t0) / 3
    ctx.status()
    sweeps16 = ctx.svd_sweeps(len(all_mats))
    dense16 = dense_equivalent_flops(list(shapes) * workers, sweeps16)
    del all_mats
    msgs = [flat_msgs[w * len(shapes):(w + 1) * len(shapes)] for w in range(workers)]
    groups = [[msgs[w][j] for w in range(workers)] for j in range(len(shapes))]
    outs = [torch.empty(m, n, dtype=torch.float32, device="cuda") for m, n in shapes]
    atoms = [sum(int(x.count.item()) for x in g) for g in groups]
    for _ in range(3):
        binding.atomo_decode_svd_batch(ctx, groups, 1.0 / workers, outs=outs)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        binding.atomo_decode_svd_batch(ctx, groups, 1.0 / workers, outs=outs)
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / reps
    ctx.profile_enable(True)
    ctx.profile_read()
    for _ in range(reps):
        binding.atomo_decode_svd_batch(ctx, groups, 1.0 / workers, outs=outs)
    gpu_ms = ctx.profile_read()["decode_svd"][0] / reps
    # the whole parameter-server step in the same launch: params += (-gamma / P) * sum of the messages
    params = [torch.zeros(m, n, dtype=torch.float32, device="cuda") for m, n in shapes]
    for _ in range(reps):
        binding.atomo_apply_svd_batch(ctx, groups, -0.01 / workers, params)
    apply_ms = ctx.profile_read()["decode_svd"][0] / reps
    ctx.profile_enable(False)
    flops = sum(2.0 * m * n * k for (m, n), k in zip(shapes, atoms))
    nbytes = 4.0 * sum(m * n for m, n in shapes)
    return {"workload": "21 ResNet-18 layers, 16 messages each (s=3), decode + average in one launch",
            "kept_atoms": sum(atoms), "gpu_us_per_call": round(gpu_ms * 1e3, 2), "wall_us_per_call": round(wall * 1e6, 2),
            "mfma_tflops": round(flops / (gpu_ms * 1e-3) / 1e12, 3),
            "mfma_frac": round(flops / (gpu_ms * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS, 5),
            "hbm_write_gbs": round(nbytes / (gpu_ms * 1e-3) / 1e9, 1),
            "hbm_frac": round(nbytes / (gpu_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
            "encode_16_gradients_one_call_ms": round(enc16 * 1e3, 2),
            "encode_16_gradients_elements_per_s": workers * sum(m * n for m, n in shapes) / enc16,
            # the same sweeps in the textbook data-space form, sweeps x (8 M r^2 + 4 r^3): flops that are not executed
            "encode_16_gradients_dense_equivalent_not_executed_tflops": round(dense16 / enc16 / 1e12, 2),
            "fused_sgd_update_gpu_us_per_call": round(apply_ms * 1e3, 2),
            "fused_sgd_update_hbm_gbs": round(2.0 * nbytes / (apply_ms * 1e-3) / 1e9, 1)}


def section6_leg(ctx, torch, binding, inputs, s, seed, reps=20):
    """The same encode + decode on the layer sets in the reshape of Section 6 ([x*y/2, 2*k*k] per convolution):
    ResNet-18 (every matrix has at most 18 columns, all on the thin path) and VGG-11-BN (eight such matrices
    plus two 512 x 512 fully connected layers, which take the Gram-space iteration).  Wall time per step, and
    the GPU time of the thin kernels against the bytes they have to move (see executed_work)."""
    out = {}
    for name, shapes in (("resnet18", inputs.RESNET18_SECTION6_SHAPES), ("vgg11bn", inputs.VGG11BN_SECTION6_SHAPES)):
        host = inputs.section6_layer_set(0, shapes)
        mats = [torch.from_numpy(g).cuda() for g in host]
        n_elem = sum(g.size for g in host)
        msgs = [binding.alloc_svd_message(m, n, binding.default_capacity(s, min(m, n)), "cuda") for m, n in shapes]
        outs = [torch.empty(m, n, dtype=torch.float32, device="cuda") for m, n in shapes]
        groups = [[m] for m in msgs]

        def step():
            binding.atomo_encode_svd(ctx, mats, s, seed, 0, msgs=msgs)
            binding.atomo_decode_svd_batch(ctx, groups, 1.0, outs=outs)

        for _ in range(3):
            step()
        torch.cuda.synchronize()
        status, _ = ctx.status()
        t0 = time.perf_counter()
        for _ in range(reps):
            step()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / reps
        sweeps = ctx.svd_sweeps(len(shapes))
        ctx.profile_enable(True)
        prof = {}
        for _ in range(reps):
            step()
            for k, (ms, cnt) in ctx.profile_read().items():
                if cnt:
                    prof[k] = prof.get(k, 0.0) + ms
        ctx.profile_enable(False)
        thin_bytes = sum(4.0 * m * n * (3 + 2 * sw) for (m, n), sw in zip(shapes, sweeps) if min(m, n) <= 32)
        thin_ms = prof.get("svd_thin", 0.0) / reps
        out[name] = {"elements": n_elem, "status": status, "us_per_step": round(dt * 1e6, 1),
                     "elements_per_s": n_elem / dt,
                     "gpu_us_by_kernel_class": {k: round(v / reps * 1e3, 1) for k, v in sorted(prof.items())},
                     "thin_hbm_gbs": round(thin_bytes / (thin_ms * 1e-3) / 1e9, 1) if thin_ms > 0 else None,
                     "thin_hbm_frac": round(thin_bytes / (thin_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4) if thin_ms > 0 else None}
    return out


def single_layer_leg(ctx, torch, binding, inputs, reps=50):
    """One 64 x 576 conv-layer gradient (rank-4 signal + N(0, 0.01^2)), s = 2: encode + decode of a single small
    matrix is a chain of dependent launches on a handful of compute units, so the figure is a latency, not a rate."""
    g = torch.from_numpy(inputs.single_conv_layer(0)).cuda()
    msgs = [binding.alloc_svd_message(64, 576, binding.default_capacity(2.0, 64), "cuda")]
    out = torch.empty(64, 576, dtype=torch.float32, device="cuda")

    def step():
        binding.atomo_encode_svd(ctx, [g], 2.0, 0, 0, msgs=msgs, adaptive=1)
        binding.atomo_decode(ctx, msgs, out=out)

    for _ in range(5):
        step()
        torch.cuda.synchronize()
    status, sweeps = ctx.status()
    t0 = time.perf_counter()
    for _ in range(reps):
        step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / reps
    lat = []
    for _ in range(10):                                         # one step at a time: what a caller that waits sees
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        step()
        torch.cuda.synchronize()
        lat.append(time.perf_counter() - t1)
    flops = sweeps * (8.0 * 576 * 64 * 64 + 4.0 * 64 ** 3)
    return {"workload": "one 64 x 576 matrix, rank-4 signal 1, .5, .25, .125 + N(0, 0.01^2), s = 2, encode + decode",
            "status": status, "jacobi_sweeps": sweeps, "kept_atoms": int(msgs[0].count.item()),
            "us_per_step_back_to_back": round(dt * 1e6, 1), "us_per_step_waiting_each_time": round(1e6 * sorted(lat)[len(lat) // 2], 1),
            "elements_per_s": 64 * 576 / dt,
            "dense_equivalent_gflops_not_a_roofline": round(flops / dt / 1e9, 2)}


def batch64_leg(ctx, torch, binding, inputs, with_oracle, reps=3):
    """64 matrices 512 x 4608 (rank-16 signal, sigma ~ U(0.1, 1), + N(0, 0.01^2)), s = 4, encoded in one call and
    decoded in one launch: the configuration that fills the chip.  Encode: contraction flops executed (Gram
    matrices, rotation of the data, two-sided updates of C, accumulation of the rotations, the blocks the pair
    problems bring up to date; real data, measured sweep and refresh counts) over the encode time, against the fp32
    matrix-core peak.  Decode: 604 MB written once, against the HBM peak."""
    s, seed = 4.0, 0
    host = inputs.vgg_deep_conv_batch(0)
    shapes = [g.shape for g in host]
    mats = [torch.from_numpy(g).cuda() for g in host]
    n_elem = sum(g.size for g in host)
    msgs = [binding.alloc_svd_message(m, n, binding.default_capacity(s, min(m, n)), "cuda") for m, n in shapes]
    outs = [torch.empty(m, n, dtype=torch.float32, device="cuda") for m, n in shapes]
    groups = [[m] for m in msgs]
    for _ in range(4):          # enough for every slot of the library's staging ring to have grown to this batch
        binding.atomo_encode_svd(ctx, mats, s, seed, 0, msgs=msgs, adaptive=1)
        binding.atomo_decode_svd_batch(ctx, groups, 1.0, outs=outs)
        torch.cuda.synchronize()
    status, _ = ctx.status()
    e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
    enc_ms = dec_ms = 0.0
    t0 = time.perf_counter()
    for _ in range(reps):
        e0.record()
        binding.atomo_encode_svd(ctx, mats, s, seed, 0, msgs=msgs, adaptive=1)
        e1.record()
        binding.atomo_decode_svd_batch(ctx, groups, 1.0, outs=outs)
        e2.record()
        torch.cuda.synchronize()
        enc_ms += e0.elapsed_time(e1) / reps
        dec_ms += e1.elapsed_time(e2) / reps
    wall = (time.perf_counter() - t0) / reps
    status2, _ = ctx.status()
    sweeps = ctx.svd_sweeps(len(mats))
    refreshes = ctx.svd_refreshes(len(mats))
    kept = [int(m.count.item()) for m in msgs]
    binding.atomo_encode_svd(ctx, mats, s, seed, 0, msgs=msgs, adaptive=1)   # counters of exactly one encode
    ctx.status()
    pair_visits, jacobi_steps, row_update_tiles = ctx.last_counters()
    work = executed_work(shapes, sweeps, refreshes, pair_visits, jacobi_steps, row_update_tiles, n_elem, kept)
    rotations = jacobi_steps * 32 * ROTATION_UNITS * 64 * 6
    contraction = sum(work[k][1] for k in ("svd_gram", "svd_update", "svd_refresh")) + work["svd_eig"][1] - rotations
    dec_bytes = work["decode_svd"][1]
    out = {"workload": "64 matrices 512 x 4608, rank-16 signal sigma ~ U(0.1, 1) + N(0, 0.01^2), s = 4, one encode call + "
                       "one decode launch", "elements": n_elem, "status": max(status, status2, key=abs),
           "ms_per_step": round(wall * 1e3, 2), "elements_per_s": n_elem / wall,
           "encode_gpu_ms": round(enc_ms, 2), "decode_gpu_ms": round(dec_ms, 3),
           "jacobi_sweeps": [min(sweeps), max(sweeps)], "gram_refreshes": [min(refreshes), max(refreshes)],
           "kept_atoms": sum(kept),
           "encode_roofline": {"bound": "mfma", "achieved": round(contraction / (enc_ms * 1e-3) / 1e12, 2),
                               "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                               "frac": round(contraction / (enc_ms * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS, 4),
                               "executed_contraction_flops": contraction, "vector_alu_rotation_flops": rotations,
                               "dense_equivalent_not_executed_flops": dense_equivalent_flops(shapes, sweeps)},
           "decode_roofline": {"bound": "hbm", "achieved": round(dec_bytes / (dec_ms * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBS,
                               "unit": "GB/s", "frac": round(dec_bytes / (dec_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                               "algorithmic_bytes": dec_bytes}}
    del mats, outs, msgs
    torch.cuda.empty_cache()
    if with_oracle and os.environ.get("ATOMO_BENCH_SKIP_CPU") != "1":
        from concurrent.futures import ThreadPoolExecutor

        import oracle

        sample = [0, 21, 42, 63]

        def one(j):
            enc = oracle.encode_svd(host[j], s, seed, j)
            oracle.decode_svd([enc], *host[j].shape)
            return host[j].size

        oracle.svd(np.eye(2))
        t0 = time.perf_counter()
        with ThreadPoolExecutor(max_workers=len(sample)) as pool:
            done = sum(pool.map(one, sample))
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": done / dt, "unit": "elements/s", "cores": len(sample), "kind": "oracle",
                               "sample": f"4 of the 64 matrices (indices {sample}), encode + decode, one thread each, "
                                         f"{dt:.1f} s wall; the 64 matrices are independent, so the whole batch on these "
                                         f"{len(sample)} threads would take 16 times as long at the same rate"}
    return out


def entrywise_leg(ctx, torch, binding, inputs, reps=40, sets=8):
    """The entry-wise path on the full flat gradient (11,173,962 elements, s = N/100), outside the timed
    steps of the headline metric: encode + decode, HBM-bound.  Eight input/message/output sets are rotated
    so that one repetition does not find the previous one's data in the last-level cache.  Algorithmic
    traffic: two reads of g (a global reduction must precede sampling) and one dense write, 12 B per
    element, plus 8 B out and 12 B in/out per kept pair."""
    n = inputs.RESNET18_PARAMETERS
    g = torch.from_numpy(inputs.flat_heavy_tail(0))
    s = n / 100
    gs = [g.cuda() for _ in range(sets)]
    outs = [torch.empty(n, dtype=torch.float32, device="cuda") for _ in range(sets)]
    msgs = [binding.alloc_entrywise_message(n, binding.default_capacity(s, n), "cuda") for _ in range(sets)]

    def step(i):
        k = i % sets
        binding.atomo_encode_entrywise(ctx, gs[k], s, 0, 0, msg=msgs[k])
        binding.atomo_decode(ctx, [msgs[k]], out=outs[k])

    for i in range(sets):
        step(i)
    torch.cuda.synchronize()
    if ctx.status()[0] != 0:
        return None
    t0 = time.perf_counter()
    for i in range(reps):
        step(i)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / reps
    kept = int(msgs[0].count.item())
    ctx.profile_enable(True)
    ctx.profile_read()
    prof = {}
    for i in range(reps):
        step(i)
        for name, (ms, cnt) in ctx.profile_read().items():
            if cnt:
                prof[name] = prof.get(name, 0.0) + ms
    ctx.profile_enable(False)
    nbytes = 12.0 * n + 20.0 * kept
    # l_q quantisation of the same gradient (1-bit QSGD, TernGrad): norm pass instead of the histograms
    lq = {}
    for name, q in (("qsgd_1bit_q2", 2.0), ("terngrad_qinf", float("inf"))):
        lmsgs = [binding.alloc_lq_message(n, binding.lq_capacity(n, q), "cuda") for _ in range(sets)]

        def lstep(i):
            k = i % sets
            binding.atomo_encode_lq(ctx, gs[k], q, 0, 0, msg=lmsgs[k])
            binding.atomo_decode(ctx, [lmsgs[k]], out=outs[k])

        for i in range(sets):
            lstep(i)
        torch.cuda.synchronize()
        if ctx.status()[0] != 0:
            continue
        t0 = time.perf_counter()
        for i in range(reps):
            lstep(i)
        torch.cuda.synchronize()
        ldt = (time.perf_counter() - t0) / reps
        lkept = int(lmsgs[0].count.item())
        lbytes = 12.0 * n + 8.0 * lkept
        lq[name] = {"us_per_step": round(ldt * 1e6, 2), "kept": lkept, "elements_per_s": n / ldt,
                    "hbm_gbs": round(lbytes / ldt / 1e9, 1), "hbm_frac": round(lbytes / ldt / 1e9 / PEAK_HBM_GBS, 4)}
    # the same path on a gradient a hundred times larger (2^30 elements, 4.3 GB, generated on the device): the
    # launches and single-workgroup steps that dominate at 44.7 MB are amortised there
    large = None
    try:
        nl = 1 << 30
        gl = torch.empty(nl, dtype=torch.float32, device="cuda").normal_(0.0, 1e-3)
        gl[::1000] *= 100.0
        sl = nl / 100
        ml = binding.alloc_entrywise_message(nl, binding.default_capacity(sl, nl), "cuda")
        ol = torch.empty(nl, dtype=torch.float32, device="cuda")
        for _ in range(2):
            binding.atomo_encode_entrywise(ctx, gl, sl, 0, 0, msg=ml)
            binding.atomo_decode(ctx, [ml], out=ol)
        torch.cuda.synchronize()
        if ctx.status()[0] == 0:
            t0 = time.perf_counter()
            for _ in range(5):
                binding.atomo_encode_entrywise(ctx, gl, sl, 0, 0, msg=ml)
                binding.atomo_decode(ctx, [ml], out=ol)
            torch.cuda.synchronize()
            dl = (time.perf_counter() - t0) / 5
            kl = int(ml.count.item())
            bl = 12.0 * nl + 20.0 * kl
            large = {"elements": nl, "kept": kl, "ms_per_step": round(dl * 1e3, 3), "elements_per_s": nl / dl,
                     "hbm_gbs": round(bl / dl / 1e9, 1), "hbm_frac": round(bl / dl / 1e9 / PEAK_HBM_GBS, 4)}
        del gl, ml, ol
        torch.cuda.empty_cache()
    except RuntimeError:
        large = None
    return {"workload": "flat_heavy_tail: N=11,173,962 fp32, N(0,1e-3^2) + 11,173 entries x100, s=N/100, encode + decode",
            "elements_per_s": n / dt, "us_per_step": round(dt * 1e6, 2), "kept": kept,
            "roofline": {"bound": "hbm", "achieved": round(nbytes / dt / 1e9, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                         "frac": round(nbytes / dt / 1e9 / PEAK_HBM_GBS, 4), "algorithmic_bytes_per_step": nbytes},
            "us_per_step_by_kernel_class": {k: round(v / reps * 1e3, 2) for k, v in sorted(prof.items())},
            "lq_quantisation": lq,
            "same_path_at_2^30_elements": large}


def cpu_baseline(host_mats, s, seed):
    """The oracle (fp64, plain C, as it stands) on the same workload: one encode + decode of the whole
    21-layer set, host threads over layers (largest layers first so the threads stay busy); and, on one thread, a
    sample of the set (one layer of every shape but the two largest), about ten seconds of work."""
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
    # single thread: one layer per distinct shape, leaving out 512 x 4608 and 512 x 2304 (tens of seconds each)
    seen, single = set(), []
    for j, g in enumerate(host_mats):
        if g.shape not in seen and g.shape not in ((512, 4608), (512, 2304)):
            seen.add(g.shape)
            single.append((j, g))
    t1 = time.perf_counter()
    n_single = sum(one(item) for item in single)
    dt1 = time.perf_counter() - t1
    return {"value": n_elem / dt, "unit": "elements/s", "cores": cores, "kind": "oracle",
            "sample": f"one full step (all 21 layers, {n_elem} elements), encode + decode, {dt:.1f} s wall on "
                      f"{cores} threads",
            "single_thread": {"value": n_single / dt1, "unit": "elements/s", "cores": 1,
                              "sample": f"one layer of each of the {len(single)} shapes other than 512 x 4608 and 512 x 2304 "
                                        f"({n_single} elements), encode + decode, {dt1:.1f} s on one thread"}}


if __name__ == "__main__":
    main()
