#!/usr/bin/env python3
"""Benchmark of Flora's hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input:
  * Algorithm-1 workloads (1, 2, 4): one accumulation cycle = tau grouped compress
    launches over tau distinct gradient sets (the first one overwrites the accumulator,
    which is the cycle's reset), then decompress + update, then a new seed per matrix.
  * Algorithm-2 workloads (3, 5): one optimizer step = flora_fused_step
    ((transfer when t = 0 mod kappa) + EMA compress + decompress + SGD update).

With no --config the top-level fields of the JSON line describe the largest of the benchmark's
configurations that fits one GPU (configuration 4: T5-3B shapes, bf16 gradients, r = 256,
tau = 16, factored update), and "configs" carries the same fields for configurations 1, 2, 3
and 5, run in the same process with capped step counts.  --config N runs that one alone and
accepts the variant flags below.  Inputs are resident in HBM before the timed region starts;
gradient sets rotate so that no set is re-read from cache.

Prints ONE JSON line; --gpus above 1 is refused: this build is single-GPU by design.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published
BF16_MFMA_PEAK_TFLOPS = 2500.0  # dense bf16 matrix cores, published
GEN_RATE_MEASURED = 1.88e12     # normals/s of the generator alone on the whole chip (measured)
HEADLINE = 4
DEFAULT_STEPS = {1: 500, 2: 200, 3: 300, 4: 20, 5: 40}
DEFAULT_WARM = {1: 20, 2: 10, 3: 10, 4: 2, 5: 3}
# step counts of the configurations that ride along in the default run
SIDE_STEPS = {1: 300, 2: 100, 3: 300, 5: 40}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--config", type=int, default=None,
                    help="run workload 1..5 alone (default: 4 as the headline plus 1, 2, 3, 5 in \"configs\")")
    ap.add_argument("--grad-sets", type=int, default=None, help="distinct gradient sets in the ring")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch the library's plain 1 GiB copy kernel 3 times (profiler yardstick)")
    ap.add_argument("--event-every", type=int, default=4,
                    help="bracket the launches of every N-th timed step with HIP events")
    ap.add_argument("--tune", default="", help="launch-shape overrides for sweeps: name=value[,name=value...] "
                                               "(names of flora_set_tuning)")
    ap.add_argument("--rule", default=None, choices=["adafactor", "unfactored"],
                    help="replace the workload's update rule by the whole Adafactor step (factored second "
                         "moment, published schedules, step relative to the carried parameter scale) or by "
                         "its unfactored variant")
    ap.add_argument("--momentum", default=None, choices=["folded", "direct"],
                    help="Algorithm-1 workloads only: feed the accumulation cycle into a compressed momentum "
                         "(beta 0.9) and update from that.  folded: accumulate into C under one projection, "
                         "then M <- beta M + ((1-beta)/tau) C A_c^T A_m (flora_transfer_accumulate); direct: one "
                         "projection for both, every micro-batch is compressed straight into M")
    ap.add_argument("--rank", type=int, default=None, choices=[8, 16, 32, 64, 128, 256],
                    help="run the configuration's shapes at another rank (a variant, named as such in config.workload)")
    ap.add_argument("--grad-dtype", default=None, choices=["f32", "bf16"],
                    help="run the configuration's shapes with gradients of another type (a variant)")
    ap.add_argument("--weights", default="f32", choices=["f32", "bf16"],
                    help="dtype of the weights (the workloads are defined with fp32 weights; bf16 weights are "
                         "updated in fp32 and rounded to nearest even when stored)")
    ap.add_argument("--input-map", default=None, choices=["square"],
                    help="compress the elementwise square of the gradients (flora_compress_mapped: the compressed "
                         "EMA of the second moment) instead of the gradients; same launches otherwise")
    ap.add_argument("--layerwise", type=int, default=0, metavar="K",
                    help="Algorithm-2 workloads only: one flora_fused_step call per K consecutive matrices (the "
                         "layer-by-layer invocation of an update-in-backward training loop; K = 4 is one "
                         "transformer block of workloads 3 and 5) instead of one grouped call")
    ap.add_argument("--separate-calls", action="store_true",
                    help="Algorithm-2 workloads: issue every step as flora_compress + flora_apply_update instead "
                         "of flora_fused_step (the same kernels in the same order)")
    ap.add_argument("--ceilings", action="store_true",
                    help="instead of a workload, time plain kernels that bound the hot path on this chip (streaming "
                         "read, the compress kernels' operand pattern, copy, register-resident matrix-core loops, the "
                         "generator alone) and print them as one JSON line")
    ap.add_argument("--cpu-budget-gflop", type=float, default=16.0,
                    help="size of the oracle's sample (fp64 GFLOP)")
    ap.add_argument("--cpu-seconds", type=float, default=10.0,
                    help="oracle time to collect for the all-cores baseline of the headline workload")
    return ap.parse_args()


def median(xs):
    s = sorted(xs)
    k = len(s)
    return s[k // 2] if k % 2 else 0.5 * (s[k // 2 - 1] + s[k // 2])


def generated_normals(flora, shapes, r, gdt, kind):
    """Entries of A one grouped launch regenerates (every workgroup rebuilds the slice of A its
    columns and rank slice meet), from the library's own work table (host only)."""
    items, info = flora.debug_work_items(kind, shapes, r, gdt)
    if kind == 0:
        wide = info[0] >= 8
        width = r if r <= 32 else ((64 if r == 64 else 128) if wide else 64)
        cols = 0
        for it in items:
            m = shapes[int(it[0])][1]
            c1 = int(it[6]) if int(it[6]) > 0 else m
            cols += min(m, c1) - int(it[3])
        return cols * width
    colsper = 256 if info[1] else 128
    tot = 0
    for it in items:
        m = shapes[int(it[0])][1]
        tot += min(colsper, m - int(it[3])) * r
    return tot


def ceilings():
    """What plain kernels reach on this chip (the library's measurement hooks, HIP events on the
    launch stream, median over the launches)."""
    import torch
    from paper_2402_03293_amd import flora

    dev = "cuda:0"
    stream = torch.cuda.current_stream()
    sink = torch.zeros(64, dtype=torch.float32, device=dev)
    out = {"what": "ceilings of plain kernels on this chip", "unit_note": "GB = 1e9 bytes", "kernels": {}}

    def time_launches(fn, n):
        for i in range(3):
            fn(i)
        torch.cuda.synchronize()
        ms = []
        for i in range(n):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            fn(i)
            e1.record(stream)
            ms.append((e0, e1))
        torch.cuda.synchronize()
        v = sorted(a.elapsed_time(b) for a, b in ms)
        return v[len(v) // 2], v[0]

    tiny = torch.zeros(64, dtype=torch.float32, device=dev)
    med, mn = time_launches(lambda i: flora.debug_read(tiny, 16, sink, 0, 0, 0, stream), 200)
    out["kernels"]["empty launch"] = {"median_us": med * 1e3, "min_us": mn * 1e3}

    # workload 2's size: 176 MB per launch, a ring of 8 buffers so that nothing is served from cache
    rows, row_bytes = 21504, 8192
    small = [torch.zeros(rows * row_bytes // 4, dtype=torch.float32, device=dev) for _ in range(8)]
    nb = rows * row_bytes
    for name, pat, chunk in (("stream read, 176 MB", 0, 0), ("operand-pattern read (16 rows x 64 B per instruction, "
                                                              "2048 B per wave and row), 176 MB", 1, 2048)):
        med, mn = time_launches(lambda i: flora.debug_read(small[i % 8], nb, sink, pat, row_bytes, chunk, stream), 80)
        out["kernels"][name] = {"median_us": med * 1e3, "min_us": mn * 1e3, "GBps": nb / (med * 1e-3) / 1e9}
    del small
    big = [torch.zeros(1 << 28, dtype=torch.float32, device=dev) for _ in range(3)]
    nb = 1 << 30
    for name, pat, chunk, rb in (("stream read, 1 GiB", 0, 0, 0),
                                 ("operand-pattern read, 1 GiB (rows of 8192 B, 2048 B per wave and row)", 1, 2048, 8192),
                                 ("operand-pattern read, 1 GiB (rows of 32768 B, whole rows per wave)", 1, 32768, 32768)):
        med, mn = time_launches(lambda i: flora.debug_read(big[i % 3], nb, sink, pat, rb, chunk, stream), 20)
        out["kernels"][name] = {"median_us": med * 1e3, "min_us": mn * 1e3, "GBps": nb / (med * 1e-3) / 1e9}
    med, mn = time_launches(lambda i: flora.debug_copy(big[i % 2], big[2], nb, stream), 20)
    out["kernels"]["copy, 1 GiB read + 1 GiB written"] = {"median_us": med * 1e3, "min_us": mn * 1e3,
                                                          "GBps": 2 * nb / (med * 1e-3) / 1e9}
    del big
    for name, kind, iters in (("v_mfma_f32_16x16x32_bf16 loop", 0, 20000), ("v_mfma_f32_32x32x16_bf16 loop", 1, 20000),
                              ("v_mfma_f32_16x16x4_f32 loop", 2, 20000)):
        work = [0.0]

        def fn(i, kind=kind, iters=iters):
            work[0] = flora.debug_compute_loop(kind, iters, sink, stream)
        med, mn = time_launches(fn, 5)
        out["kernels"][name] = {"median_ms": med, "TFLOPs": work[0] / (med * 1e-3) / 1e12}
    work = [0.0]

    def gen(i):
        work[0] = flora.debug_compute_loop(3, 2000, sink, stream)
    med, mn = time_launches(gen, 5)
    out["kernels"]["generator alone (Philox4x32-10 + Box-Muller)"] = {"median_ms": med, "normals_per_s": work[0] / (med * 1e-3)}
    out["published_peaks"] = {"hbm_GBps": HBM_PEAK_GBS, "bf16_mfma_TFLOPs": BF16_MFMA_PEAK_TFLOPS, "fp32_mfma_TFLOPs": 157.3}
    return out


def run_config(args, index, steps, warmup, cpu_seconds, variants=True):
    """Runs one workload and returns its record (the fields of the JSON line)."""
    import torch
    from paper_2402_03293_amd import flora, workloads

    dev = "cuda:0"
    wl = workloads.workload(index)
    if variants and (args.rank or args.grad_dtype):
        import dataclasses
        wl = dataclasses.replace(wl, r=args.rank or wl.r, grad_dtype=args.grad_dtype or wl.grad_dtype,
                                 name="%s-shapes-%s-r%d" % (wl.name, args.grad_dtype or wl.grad_dtype, args.rank or wl.r))
    r = wl.r
    shapes = wl.shapes
    count = len(shapes)
    gdt = flora.F32 if wl.grad_dtype == "f32" else flora.BF16
    gbytes = 4 if wl.grad_dtype == "f32" else 2
    a_rule = args.rule if variants else None
    a_momentum = args.momentum if variants else None
    a_layerwise = args.layerwise if variants else 0
    a_map = args.input_map if variants else None
    a_weights = args.weights if variants else "f32"
    a_separate = args.separate_calls if variants else False

    # ---- inputs, resident in HBM -------------------------------------------------
    gen = workloads.make_generator(wl.seed, dev)
    if args.grad_sets is not None and variants:
        nsets = args.grad_sets
    elif wl.algorithm == 1:
        nsets = wl.tau if wl.index != 4 else 4
    else:
        nsets = max(4, min(8, int(2e9 // max(1, wl.grad_bytes)) + 1))
    grad_sets = [workloads.make_grad_set(wl, gen, dev) for _ in range(nsets)]
    W = workloads.make_weight_set(wl, gen, dev)
    wdt, wbytes = flora.F32, 4
    if a_weights == "bf16":
        W = [w.to(torch.bfloat16) for w in W]
        wdt, wbytes = flora.BF16, 2
    states = [torch.zeros((n, r), device=dev, dtype=torch.float32) for n, _ in shapes]
    row_stats = col_stats = second = sumsq = None
    rule = a_rule or wl.rule
    if rule in ("adafactor", "unfactored"):
        sumsq_buf = torch.zeros((count, 4), device=dev)
        sumsq = [sumsq_buf[i] for i in range(count)]
    if rule == "unfactored":
        # resumed from a typical second moment (from zero the first steps are sign descent)
        second = [torch.full((n, m), 1.0, device=dev) for n, m in shapes]
    if rule in ("factored", "adafactor"):
        row_stats = [torch.zeros((n,), device=dev) for n, _ in shapes]
        col_stats = [torch.zeros((m,), device=dev) for _, m in shapes]
    torch.cuda.synchronize()

    if a_layerwise and wl.algorithm != 2:
        sys.stderr.write("bench.py: --layerwise applies to the momentum workloads (3, 5)\n")
        sys.exit(2)
    if a_momentum and wl.algorithm != 1:
        sys.stderr.write("bench.py: --momentum applies to the accumulation workloads (1, 2, 4)\n")
        sys.exit(2)
    mom = mom_seeds = None
    if a_momentum:
        mom = [torch.zeros((n, r), device=dev, dtype=torch.float32) for n, _ in shapes]
        mom_seeds = flora.derive_seeds(4321, 0, count, 0)     # the momentum keeps its projection
    torch.cuda.synchronize()

    stream = torch.cuda.current_stream()
    gseed = 1234
    epoch = 0
    seeds = flora.derive_seeds(gseed, 0, count, epoch)

    # one descriptor array per gradient set, built once; only the seed fields change later
    mats_sets = [flora.matrices(shapes, grads=grad_sets[g], weights=W, states=states, row_stats=row_stats,
                                col_stats=col_stats, seeds=seeds, seeds_next=seeds, second_moments=second,
                                weight_sumsqs=sumsq) for g in range(nsets)]
    views = [flora.fields(mt) for mt in mats_sets]
    mats_one = None
    if a_layerwise:
        # one descriptor per (gradient set, matrix), built once
        K = a_layerwise
        groups = [list(range(l0, min(count, l0 + K))) for l0 in range(0, count, K)]

        def pick(xs, idx):
            return [xs[l] for l in idx] if xs is not None else None

        mats_one = [[flora.matrices(pick(shapes, idx), grads=pick(grad_sets[g], idx), weights=pick(W, idx),
                                    states=pick(states, idx), row_stats=pick(row_stats, idx),
                                    col_stats=pick(col_stats, idx), second_moments=pick(second, idx),
                                    weight_sumsqs=pick(sumsq, idx), seeds=pick(seeds, idx),
                                    seeds_next=pick(seeds, idx)) for idx in groups]
                    for g in range(nsets)]
    mats_mom = None
    if a_momentum:
        # descriptors whose state is the momentum: the update reads it; in direct mode the
        # micro-batches are compressed into it as well
        mats_mom = [flora.matrices(shapes, grads=grad_sets[g], weights=W, states=mom, row_stats=row_stats,
                                   col_stats=col_stats, seeds=mom_seeds, seeds_next=mom_seeds,
                                   second_moments=second, weight_sumsqs=sumsq) for g in range(nsets)]

    def set_seeds(cur, nxt=None):
        for v in views:
            v["seed"][:] = cur
            v["seed_next"][:] = cur if nxt is None else nxt

    alpha_u = 1.0 / wl.tau if wl.algorithm == 1 else 1.0
    zero_after = False      # Algorithm 1's reset is the a = 0 of the next cycle's first compress

    if a_momentum:
        alpha_u, zero_after = 1.0, False     # the momentum is not reset and its decompression carries no 1/tau

    # calls that cover a few matrices each tell the library how large the whole step's set of weights is
    step_mib = 0.0
    if a_layerwise:
        step_mib = sum(n * m for n, m in wl.shapes) * (wbytes + (4 if rule == "unfactored" else 0)) / 2.0 ** 20

    def adafactor_update(t):
        # step t = 1, 2, ... of the published schedules, relative to the parameter scale
        rho, beta2 = flora.adafactor_schedule(t)
        mk = flora.factored_update if rule == "adafactor" else flora.unfactored_update
        return mk(rho, alpha_u, beta2, 1e-30, 1.0, zero_state_after=zero_after, scale_parameter=True, eps2=1e-3,
                  step_weight_mib=step_mib)

    if rule in ("adafactor", "unfactored"):
        flora.weight_sumsq(mats_sets[0], wdt, stream)     # once: the updates carry it from here on
        upd = adafactor_update(1)
    elif wl.rule == "factored":
        ex = wl.extra
        upd = flora.factored_update(wl.lr, 1.0 / wl.tau, ex["beta2"], ex["eps1"], ex["clip_d"])
    elif wl.algorithm == 1:
        upd = flora.sgd_update(wl.lr, 1.0 / wl.tau)
    else:
        upd = flora.sgd_update(wl.lr, 1.0)

    upd.step_weight_mib = step_mib

    upd_mom = None
    if a_momentum:
        if rule in ("adafactor", "unfactored"):
            upd_mom = upd
        elif wl.rule == "factored":
            ex = wl.extra
            upd_mom = flora.factored_update(wl.lr, 1.0, ex["beta2"], ex["eps1"], ex["clip_d"])
        else:
            upd_mom = flora.sgd_update(wl.lr, 1.0)

    ev_pairs = {"compress": [], "update": [], "transfer": [], "layerwise": [], "fused_step": []}
    record = {"on": False}

    def timed(kind, fn):
        if record["on"]:
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            fn()
            e1.record(stream)
            ev_pairs[kind].append((e0, e1))
        else:
            fn()

    tstate = {"t": 0, "gi": 0, "u": 0}

    def do_compress(mt, a_, b_):
        if a_map == "square":
            flora.compress_mapped(mt, r, gdt, flora.INPUT_SQUARE, a_, b_, stream)
        else:
            flora.compress(mt, r, gdt, a_, b_, stream)

    # Algorithm-2 steps go through flora_fused_step.  Its kernels cannot be bracketed from here, so
    # the steps whose launches are timed (every --event-every-th) are issued as the equivalent
    # separate calls, the same kernels in the same order, unless the library runs the step as a
    # single launch (then the whole call is the kernel that is timed).
    fused_ok = (wl.algorithm == 2 and not a_layerwise and not a_separate and a_map is None)
    one_launch = fused_ok and hasattr(flora, "fused_step_is_single_launch") and \
        flora.fused_step_is_single_launch(mats_sets[0], r, gdt, wdt, upd)

    def one_step():
        nonlocal seeds, epoch, upd
        if rule in ("adafactor", "unfactored"):
            tstate["u"] += 1
            upd = adafactor_update(tstate["u"])
        if wl.algorithm == 1 and a_momentum:
            beta = 0.9
            for i in range(wl.tau):
                g = tstate["gi"] % nsets
                tstate["gi"] += 1
                if a_momentum == "direct":
                    mt = mats_mom[g]
                    a_, b_ = (beta if i == 0 else 1.0), (1.0 - beta) / wl.tau
                    timed("compress", lambda: do_compress(mt, a_, b_))
                else:
                    mt = mats_sets[g]
                    a0_ = 0.0 if i == 0 else 1.0
                    timed("compress", lambda: do_compress(mt, a0_, 1.0))
            if a_momentum == "folded":
                for v in views:
                    v["seed_next"][:] = mom_seeds
                mt = mats_sets[0]
                timed("transfer", lambda: flora.transfer_accumulate(mt, r, beta, (1.0 - beta) / wl.tau, mom, stream))
            mt = mats_mom[0]
            u_ = upd if rule in ("adafactor", "unfactored") else upd_mom
            timed("update", lambda: flora.apply_update(mt, r, wdt, u_, stream))
            epoch += 1
            seeds = flora.derive_seeds(gseed, 0, count, epoch)
            set_seeds(seeds)
        elif wl.algorithm == 1:
            for i in range(wl.tau):
                mt = mats_sets[tstate["gi"] % nsets]
                tstate["gi"] += 1
                # the cycle's accumulator starts at zero: the first micro-batch overwrites it (a = 0)
                a_ = 0.0 if i == 0 else 1.0
                timed("compress", lambda: do_compress(mt, a_, 1.0))
            mt = mats_sets[0]
            timed("update", lambda: flora.apply_update(mt, r, wdt, upd, stream))
            epoch += 1
            seeds = flora.derive_seeds(gseed, 0, count, epoch)
            set_seeds(seeds)
        else:
            t = tstate["t"]
            resample = t % wl.kappa == 0
            nxt = seeds
            if resample:
                epoch += 1
                nxt = flora.derive_seeds(gseed, 0, count, epoch)
                set_seeds(seeds, nxt)
            if a_layerwise:
                if resample:
                    mt = mats_sets[0]
                    timed("transfer", lambda: flora.momentum_transfer(mt, r, stream))
                    seeds = nxt
                    set_seeds(seeds)
                ones = mats_one[tstate["gi"] % nsets]
                tstate["gi"] += 1

                def all_layers():
                    for gi in range(len(groups) - 1, -1, -1):  # the order gradients appear in backward
                        flora.fields(ones[gi])["seed"][:] = seeds[groups[gi][0]:groups[gi][-1] + 1]
                        flora.fused_step(ones[gi], r, gdt, wdt, wl.beta, 1.0 - wl.beta, False, upd, stream)
                timed("layerwise", all_layers)
                tstate["t"] += 1
                return
            mt = mats_sets[tstate["gi"] % nsets]
            tstate["gi"] += 1
            if fused_ok and (one_launch or not record["on"]) and not (resample and record["on"]):
                fs = lambda: flora.fused_step(mt, r, gdt, wdt, wl.beta, 1.0 - wl.beta, resample, upd, stream)  # noqa: E731
                if one_launch and not resample:
                    timed("fused_step", fs)
                else:
                    fs()
                if resample:
                    seeds = nxt
                    set_seeds(seeds)
            else:
                if resample:
                    m0 = mats_sets[0]
                    timed("transfer", lambda: flora.momentum_transfer(m0, r, stream))
                    seeds = nxt
                    set_seeds(seeds)
                timed("compress", lambda: do_compress(mt, wl.beta, 1.0 - wl.beta))
                timed("update", lambda: flora.apply_update(mt, r, wdt, upd, stream))
            tstate["t"] += 1

    if args.calibrate_copy:
        a_ = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
        b_ = torch.empty_like(a_)
        for _ in range(3):
            flora.debug_copy(a_, b_, 1 << 30, stream)
        torch.cuda.synchronize()
        del a_, b_

    for _ in range(warmup):
        one_step()
    torch.cuda.synchronize()
    # one event per step boundary gives the per-step durations (median, min); the wall clock
    # around the whole region gives the throughput
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    marks[0].record(stream)
    for i in range(steps):
        record["on"] = (i % max(1, args.event_every) == 0)
        one_step()
        marks[i + 1].record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    record["on"] = False
    elapsed = t1 - t0
    step_ms = [marks[i].elapsed_time(marks[i + 1]) for i in range(steps)]

    grads_per_step = wl.tau if wl.algorithm == 1 else 1
    grad_bytes_step = wl.elements * gbytes * grads_per_step
    value = grad_bytes_step * steps / elapsed / 1e9

    # ---- per-kernel launch durations from the events of the timed region -------------
    E, S = wl.elements, wl.state_elements
    alg_bytes = {
        "compress": gbytes * E + 8 * S,
        "update": {"sgd": 4 * S + 2 * wbytes * E, "factored": 3 * 4 * S + 2 * wbytes * E,
                   "adafactor": 3 * 4 * S + 2 * wbytes * E, "unfactored": 2 * 4 * S + (12 + 2 * wbytes) * E}[rule],
        "transfer": 8 * S if not a_momentum else 12 * S,     # folded: reads C, reads and writes M
    }
    alg_bytes["layerwise"] = alg_bytes["compress"] + alg_bytes["update"]
    alg_bytes["fused_step"] = gbytes * E + 2 * wbytes * E + 8 * S
    alg_flops = {"compress": 2.0 * E * r,
                 "update": 2.0 * E * r * {"sgd": 1, "factored": 3, "adafactor": 3, "unfactored": 2}[rule],
                 "transfer": sum(2.0 * m * r * r + 2.0 * n * r * r for n, m in shapes)}
    alg_flops["layerwise"] = alg_flops["compress"] + alg_flops["update"]
    alg_flops["fused_step"] = alg_flops["compress"] + alg_flops["update"]
    normals = {"compress": generated_normals(flora, shapes, r, gdt, 0),
               "update": generated_normals(flora, shapes, r, gdt, 1) *
               {"sgd": 1, "factored": 3, "adafactor": 3, "unfactored": 2}[rule]}
    kern = {}
    for k, pairs in ev_pairs.items():
        if not pairs:
            continue
        ms = [a.elapsed_time(b) for a, b in pairs]
        avg = sum(ms) / len(ms)
        kern[k] = {
            "launches": len(ms), "avg_ms": avg, "min_ms": min(ms), "median_ms": median(ms),
            "alg_GBps": alg_bytes[k] / (avg * 1e-3) / 1e9,
            "alg_TFLOPs": alg_flops[k] / (avg * 1e-3) / 1e12,
        }
        if k in normals:
            kern[k]["generated_normals_per_s"] = normals[k] / (avg * 1e-3)
    dominant = max((k for k in kern if k != "transfer"), key=lambda k: kern[k]["avg_ms"] * kern[k]["launches"])
    dk = kern[dominant]
    traffic = None
    try:
        for line in open(os.path.join(ROOT, "profiles", "hbm_traffic.txt")):
            f = line.split()
            if len(f) == 4 and f[0] == wl.name and f[1] == dominant and rule == wl.rule:
                traffic = int(f[2]) + int(f[3])     # profiler-measured bytes per launch (read + written)
    except OSError:
        pass
    roofline = {
        "kernel": {"compress": "compress (state <- a*state + b*G*A)",
                   "update": "decompress + update (W <- W - rule(alpha*state*A^T))",
                   "fused_step": "fused step (EMA compress + decompress + update in one launch)",
                   "layerwise": "fused step, one call per %d matrices" % max(1, a_layerwise)}[dominant],
        "bound": "hbm", "achieved": dk["alg_GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": dk["alg_GBps"] / HBM_PEAK_GBS, "traffic": traffic,
        "bytes_per_launch": alg_bytes[dominant], "avg_launch_ms": dk["avg_ms"],
        "timing": "HIP events around the call on the launch stream, every %d-th timed step (they add about "
                  "2 us of launch gap per call; the rocprofv3 kernel-only average of the same command is in "
                  "profiles/)" % max(1, args.event_every),
    }
    if r >= 64:
        roofline["mfma_frac_of_bf16_peak"] = dk["alg_TFLOPs"] / BF16_MFMA_PEAK_TFLOPS
        roofline["achieved_TFLOPs"] = dk["alg_TFLOPs"]
    if dominant in normals:
        # third bound, plain ALU work: the generator alone reaches GEN_RATE_MEASURED on the whole chip
        roofline["generator"] = {"normals_per_launch": normals[dominant],
                                 "normals_per_s": normals[dominant] / (dk["avg_ms"] * 1e-3),
                                 "frac_of_generator_alone": normals[dominant] / (dk["avg_ms"] * 1e-3) / GEN_RATE_MEASURED}

    out = {
        "metric": "gradient GB/s through compress+decompress+update",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": elapsed / steps * 1e3, "median_ms_per_step": median(step_ms), "min_ms_per_step": min(step_ms),
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": wl.grad_dtype, "data": "synthetic",
        "config": {"workload": wl.name, "matrices": count, "elements": E, "r": r,
                   "algorithm": wl.algorithm, "tau": wl.tau if wl.algorithm == 1 else None,
                   "beta": wl.beta if wl.algorithm == 2 else None,
                   "kappa": wl.kappa if wl.algorithm == 2 else None,
                   "rule": rule, "momentum_from_accumulator": a_momentum, "input_map": a_map,
                   "weights": a_weights, "layerwise": a_layerwise, "grad_sets_in_ring": nsets,
                   "grad_bytes_per_step": grad_bytes_step,
                   "step_call": ("flora_fused_step" + (" (one launch)" if one_launch else
                                                       "; timed steps as flora_compress + flora_apply_update"))
                   if fused_ok else ("flora_fused_step per group" if a_layerwise else
                                     "flora_compress x tau + flora_apply_update" if wl.algorithm == 1 else
                                     "flora_compress + flora_apply_update")},
        "roofline": roofline,
        "kernels": kern,
    }

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, grad_sets, W, args.cpu_budget_gflop, min_seconds=cpu_seconds, rule=rule)
    del grad_sets, W, states, mats_sets, views, row_stats, col_stats, second, sumsq, mom, mats_one, mats_mom
    torch.cuda.empty_cache()
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        sys.stderr.write("bench.py: this build runs on one GPU only (no collectives are part of it); "
                         "--gpus %d is not supported, use --gpus 1\n" % args.gpus)
        sys.exit(2)

    import torch
    from paper_2402_03293_amd import flora

    if not torch.cuda.is_available():
        sys.stderr.write("bench.py: no GPU visible\n")
        sys.exit(1)
    flora.lib()                       # fail loudly if the HIP library is missing
    for kv in args.tune.split(","):
        if kv:
            name, val = kv.split("=")
            flora.set_tuning(name, int(val))
    torch.cuda.set_device(0)

    if args.ceilings:
        print(json.dumps(ceilings()))
        return

    if args.config is not None:
        idx = args.config
        steps = args.steps if args.steps is not None else DEFAULT_STEPS[idx]
        warmup = args.warmup if args.warmup is not None else DEFAULT_WARM[idx]
        out = run_config(args, idx, steps, warmup, args.cpu_seconds)
        print(json.dumps(out))
        return

    steps = args.steps if args.steps is not None else DEFAULT_STEPS[HEADLINE]
    warmup = args.warmup if args.warmup is not None else DEFAULT_WARM[HEADLINE]
    out = run_config(args, HEADLINE, steps, warmup, args.cpu_seconds, variants=False)
    sys.stderr.write("bench.py: headline workload done (%.3f ms per step)\n" % out["ms_per_step"])
    sys.stderr.flush()
    out["configs"] = []
    for idx in (1, 2, 3, 5):
        rec = run_config(args, idx, SIDE_STEPS[idx], DEFAULT_WARM[idx], min(args.cpu_seconds, 6.0), variants=False)
        for k in ("metric", "unit", "n_gpus", "higher_is_better", "scaling", "vs_baseline", "data"):
            rec.pop(k, None)
        out["configs"].append(rec)
        sys.stderr.write("bench.py: workload %d done (%.4f ms per step)\n" % (idx, rec["ms_per_step"]))
        sys.stderr.flush()
    print(json.dumps(out))


def cpu_baseline(wl, grad_sets, W, budget_gflop, min_seconds=10.0, rule=None):
    """The fp64 oracle, as it stands, timed on this host over a bounded sample of the same
    workload: whole matrices taken in order until the flop budget is used (at least one).
    All cores first (about `min_seconds` of oracle calls), then one pass of the same sample with
    the OpenMP runtime held to a single thread."""
    import ctypes

    import numpy as np
    import torch

    import oracle

    r = wl.r
    rule = rule or wl.rule
    passes = (wl.tau + 1) if wl.algorithm == 1 else 2
    chosen, fl = [], 0.0
    for l, (n, m) in enumerate(wl.shapes):
        f = 2.0 * n * m * r * passes / 1e9
        if chosen and fl + f > budget_gflop:
            continue
        chosen.append(l)
        fl += f
        if fl >= budget_gflop:
            break

    def to64(t):
        return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)

    def base_update(Wl, Gt, n, m):
        if rule == "sgd":
            oracle.sgd(Wl, Gt, wl.lr)
        elif rule == "factored":
            ex = wl.extra
            oracle.factored_update(Wl, Gt, np.zeros(n), np.zeros(m), ex["beta2"], ex["eps1"], ex["clip_d"], wl.lr)
        elif rule == "adafactor":
            oracle.adafactor_step(Wl, Gt, R=np.zeros(n), K=np.zeros(m), beta2=0.0, step=1e-2)
        else:
            oracle.adafactor_step(Wl, Gt, V=np.ones((n, m)), beta2=0.5, step=1e-2)

    gb = 4 if wl.grad_dtype == "f32" else 2

    def one_pass(mats, rep, max_rows=None):
        spent, nbytes = 0.0, 0
        for l in mats:
            n, m = wl.shapes[l]
            if max_rows is not None:
                n = min(n, max_rows)      # the first rows of the matrix: rows are independent units of work
            seed = oracle.derive_seed(99, l, rep)
            Wl = to64(W[l][:n])
            if wl.algorithm == 1:
                C = np.zeros((n, r))
                for i in range(wl.tau):
                    G = to64(grad_sets[i % len(grad_sets)][l][:n])
                    t0 = time.perf_counter()
                    C = oracle.compress(G, r, seed, state=C)
                    spent += time.perf_counter() - t0
                    nbytes += n * m * gb
                t0 = time.perf_counter()
                Gt = oracle.decompress(C, m, seed, alpha=1.0 / wl.tau)
                base_update(Wl, Gt, n, m)
                spent += time.perf_counter() - t0
            else:
                G = to64(grad_sets[0][l][:n])
                M = np.zeros((n, r))
                t0 = time.perf_counter()
                M = oracle.compress(G, r, seed, state=M, a=wl.beta, b=1.0 - wl.beta)
                Gt = oracle.decompress(M, m, seed)
                base_update(Wl, Gt, n, m)
                spent += time.perf_counter() - t0
                nbytes += n * m * gb
        return spent, nbytes

    # the sample is repeated until about `min_seconds` of oracle time have been measured
    # (small workloads would otherwise be timed over a fraction of a second)
    spent, nbytes, reps = 0.0, 0, 0
    while reps == 0 or (spent < min_seconds and reps < 200):
        reps += 1
        s_, b_ = one_pass(chosen, reps)
        spent += s_
        nbytes += b_
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count() or 1
    omp = os.environ.get("OMP_NUM_THREADS")
    threads = min(cores, int(omp)) if omp and omp.isdigit() else cores
    res = {
        "value": nbytes / spent / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
        "sample": "%d of %d matrices, whole %s, %d time(s) over: %.1f fp64 GFLOP, %.2f s of oracle calls"
                  % (len(chosen), len(wl.shapes),
                     "accumulation cycle" if wl.algorithm == 1 else "optimizer step", reps, fl * reps, spent),
    }
    # single thread: the same code with the OpenMP runtime told to use one thread, on the first
    # matrix of the sample only (the oracle itself is not changed for this)
    try:
        gomp = ctypes.CDLL("libgomp.so.1")
        gomp.omp_get_max_threads.restype = ctypes.c_int
        before = gomp.omp_get_max_threads()
        gomp.omp_set_num_threads(1)
        n1, m1 = wl.shapes[chosen[0]]
        rows1 = max(32, min(n1, int(5e9 / (2.0 * m1 * r * passes))))     # about 5 fp64 GFLOP
        try:
            s1, b1 = one_pass(chosen[:1], 1, max_rows=rows1)
        finally:
            gomp.omp_set_num_threads(before)
        res["single_thread"] = {"value": b1 / s1 / 1e9, "unit": "GB/s", "cores": 1,
                                "sample": "first %d rows of the sample's first matrix (%d x %d), %.2f s of oracle calls"
                                          % (rows1, n1, m1, s1)}
    except OSError:
        pass
    return res


if __name__ == "__main__":
    main()
