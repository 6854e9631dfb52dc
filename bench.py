#!/usr/bin/env python3
"""Benchmark of the sharded reduce + AdamW + bf16-cast step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A step is one pass of the whole hot path over one batch of synthetic gradient
contributions for one device's shard.  The default workload is the 70B ZeRO-3
shard (8.75e9 elements, N = 8) updated bucket by bucket, 33 buckets of 2^28
elements.  All inputs are resident in HBM before the timed region starts: the
eight contributions of every bucket (140 GB, every element distinct, nothing
cache-assisted), which the bucket loop reads where they lie.  The staged
two-stream pipeline for contributions that have to be moved first is timed by
--copy-engine kernel|memcpy and by --extras.  Prints ONE JSON line.
"""
import argparse
import ctypes as C
import json
import os
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0   # MI355X published HBM3E bandwidth


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def bytes_per_elem(w, clip=False):
    """Algorithmic bytes per element of one step: every byte touched once."""
    g = 4 if w.grad_dtype == "f32" else 2
    if clip:   # phase 1: N reads + fp32 spill; phase 2: spill + state in, state + bf16 out
        return g * w.n_devices + 4 + 4 + 12 + 14
    if w.strategy == "zero1":          # one all-reduced gradient
        return g + 12 + 12 + 2
    if w.micro_batches > 1:            # k - 1 accumulations (the first only writes), then the update
        k = w.micro_batches            # from the last micro-batch and the accumulator
        return k * g * w.n_devices + (k - 1) * 4 + (k - 2) * 4 + 4 + 12 + 14
    return g * w.n_devices + 12 + 12 + 2


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="70b_zero3",
                    choices=["tiny", "gpt2s", "7b_zero2", "70b_zero3", "13b_clip", "7b_zero1",
                             "7b_accum4", "7b_verify", "7b_offload", "7b_zero2_f16", "placement_map"])
    ap.add_argument("--pool-elems", type=int, default=0,
                    help="elements per contribution of the resident bucket source; 0 (default): the "
                         "whole shard length, every bucket distinct; shorter: a pool that repeats")
    ap.add_argument("--copy-engine", choices=["none", "kernel", "memcpy", "reduce"], default="none",
                    help="none: the update reads each bucket of the resident source in place; kernel, "
                         "memcpy: the two-stream pipeline that stages each bucket first; reduce: the "
                         "same pipeline with the reduce kernel as its staging engine (the FP32 sum is "
                         "what gets staged)")
    ap.add_argument("--alloc", choices=["arena", "plain"], default="arena",
                    help="bucketed workload with the whole source resident: arena = flat buffers whose "
                         "physical memory is created bucket by bucket (ps_arena_create), so that a "
                         "bucket's streams lie close together; plain = one allocation per buffer")
    ap.add_argument("--arena-chunk-elems", type=int, default=0,
                    help="elements per physical chunk of the arena (0 = the bucket size)")
    ap.add_argument("--waves-per-cu", type=int, default=0,
                    help="override the update kernel's residency cap (measurement aid; 0 = library's choice)")
    ap.add_argument("--schedule", choices=["auto", "overlap", "alternate"], default="auto")
    ap.add_argument("--source-host", action="store_true",
                    help="keep the bucket source in pinned host memory (the step is then bound by "
                         "the host link; reported for reference, never the headline value)")
    ap.add_argument("--bucket-elems", type=int, default=0, help="override the workload's bucket size")
    ap.add_argument("--clip-on-host", action="store_true",
                    help="clipped workload: read the sum of squares back and form the coefficient "
                         "on the host (one device->host sync per step) instead of on the device")
    ap.add_argument("--offload-layout", choices=["packed", "flat"], default="packed",
                    help="7b_offload: host state as one image packed bucket by bucket (one copy per "
                         "direction per bucket) or as four flat arrays (three copies up, four down)")
    ap.add_argument("--sync-each-step", action="store_true",
                    help="7b_offload: wait for the device after every step instead of enqueueing the "
                         "steps back to back")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-baseline-seconds", type=float, default=15.0,
                    help="about how much CPU work the oracle baseline may take")
    ap.add_argument("--extras", action="store_true",
                    help="also time the update kernel alone, the other pipeline schedule and a plain copy")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: the step runs on ONE GPU (the other N-1 devices of the placement are "
              "modelled as input buffers); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2601_02311_amd as ps
    from synth import WORKLOADS
    from synth import device as dgen

    if args.workload == "placement_map":
        return placement_map(args)
    if args.workload == "7b_verify":
        return verify_bench(args)
    if args.workload == "7b_offload":
        return offload_bench(args)
    w = WORKLOADS[args.workload]
    torch.cuda.set_device(0)
    info = ps.ps_device_info()
    n, N = w.shard_len, w.n_devices
    spec = ps.ps_spec_preset(w.strategy, N, w.shard_index, w.psi, align_elems=w.align_elems)
    cost = ps.ps_cost_eval(spec)
    assert cost.shard_len == n
    dt = {"bf16": ps.PS_BF16, "f16": ps.PS_F16, "f32": ps.PS_F32}[w.grad_dtype]
    esz = 4 if w.grad_dtype == "f32" else 2
    tdt = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[w.grad_dtype]
    pdt, ptd = ((ps.PS_F16, torch.float16) if w.param_dtype == "f16" else (ps.PS_BF16, torch.bfloat16))
    log("device %s (%s), %d CUs, %.1f GB free" % (info.name.decode(), info.arch.decode(),
                                                  info.compute_units, info.free_bytes / 1e9))
    log("workload %s: shard of %d elements, N=%d, %s gradients" % (w.name, n, N, w.grad_dtype))

    t_setup = time.time()
    free_at_start = torch.cuda.mem_get_info()[0]
    bucketed = w.bucket_elems > 0
    arena = None
    out_len = cost.psi_padded if spec.theta == ps.PS_R else n
    clip = w.max_grad_norm > 0
    # Which buffers come out of the arena (flat, physical memory created chunk by chunk):
    # contributions 0..N-1, master, m, v, then the parameters where they are shard-sized, the
    # reduced gradient of a clipped step and the accumulator of micro-batches.
    a_out = a_red = a_acc = None
    eb = [esz] * N + [4, 4, 4]
    if out_len == n:
        a_out, eb = len(eb), eb + [2]
    if clip:
        a_red, eb = len(eb), eb + [4]
    if w.micro_batches > 1:
        a_acc, eb = len(eb), eb + [4]
    want_arena = args.alloc == "arena" and not args.pool_elems and not args.source_host
    if want_arena and (bucketed or (w.strategy != "zero1" and n >= (1 << 29))):
        try:
            arena = ps.ps_arena_create(n, args.arena_chunk_elems or args.bucket_elems or w.bucket_elems
                                       or (1 << 28), eb)
        except ps.PsError as err:
            log("arena not created (%s): plain allocations instead" % err.detail)
    if arena is not None:
        a_buf = [ps.ps_arena_buffer(arena, k) for k in range(len(eb))]
        master, m, v = dgen.workload_state(w, into=[dgen.as_tensor(a_buf[N + j], n, torch.float32)
                                                    for j in range(3)])
    else:
        master, m, v = dgen.workload_state(w)
    if arena is not None and a_out is not None:
        out = dgen.as_tensor(a_buf[a_out], n, ptd).zero_()
    else:
        out = torch.zeros(out_len, dtype=ptd, device="cuda")
    shard = ps.ps_shard_t(master.data_ptr(), m.data_ptr(), v.data_ptr(), out.data_ptr(), n,
                          cost.valid_len, pdt, 0)
    compute = torch.cuda.Stream()
    copy = torch.cuda.Stream()
    step_no = [w.first_step]

    def hp(clip_coef=0.0, grad_scale=0.0):
        if grad_scale == 0.0 and w.loss_scale != 1.0:       # the mean and the loss scale in one factor
            grad_scale = 1.0 / (N * w.loss_scale)
        return ps.ps_adamw_t(w.lr, w.beta1, w.beta2, w.eps, w.weight_decay, step_no[0],
                             grad_scale, clip_coef)

    kernel_ms = []          # per-launch durations of the dominant kernel
    if args.waves_per_cu:
        ps.ps_probe_set_update_residency(args.waves_per_cu)
    if bucketed:
        B = args.bucket_elems or w.bucket_elems
        n_b = -(-n // B)
        staged = args.copy_engine != "none"
        # The source: every bucket of every contribution resident and distinct (the whole shard
        # length), unless a shorter pool is asked for or the device cannot hold it.
        pool_elems = args.pool_elems or n
        need = N * pool_elems * esz + (2 * N * B * esz if staged or args.extras else 0) + (2 << 30)
        free_now = torch.cuda.mem_get_info()[0]
        if not args.pool_elems and need > free_now and arena is None:
            pool_elems = 2 * B
            log("source of %d elements per contribution does not fit (%.0f GB free): using a "
                "pool of two buckets that repeats" % (n, free_now / 1e9))
        pool_elems = -(-pool_elems // 512) * 512
        pool = [dgen.fill_gradient_(dgen.as_tensor(a_buf[r], n, tdt) if arena is not None else
                                    torch.empty(pool_elems, dtype=tdt, device="cuda"),
                                    w.seed, w.first_step, r, w.grad_std, w.outlier_frac,
                                    w.outlier_mult, w.student_t_dof) for r in range(N)]
        if args.source_host:
            pool = [p.cpu().pin_memory() for p in pool]
        staging = ([torch.empty(N * B, dtype=tdt, device="cuda") for _ in range(2)]
                   if staged or args.extras else None)
        src = (C.c_void_p * N)(*[p.data_ptr() for p in pool])
        ms = (C.c_float * n_b)()
        plan = ps.ps_bucket_plan_t()
        plan.source = C.cast(src, C.POINTER(C.c_void_p))
        plan.n_contrib, plan.dtype = N, dt
        plan.bucket_elems, plan.source_elems = B, pool_elems
        plan.copy_engine = {"none": ps.PS_COPY_NONE, "kernel": ps.PS_COPY_KERNEL,
                            "memcpy": ps.PS_COPY_MEMCPY, "reduce": ps.PS_COPY_REDUCE}[args.copy_engine]
        plan.schedule = {"auto": ps.PS_SCHED_AUTO, "overlap": ps.PS_SCHED_OVERLAP,
                         "alternate": ps.PS_SCHED_ALTERNATE}[args.schedule]
        if staging:
            plan.staging[0], plan.staging[1] = staging[0].data_ptr(), staging[1].data_ptr()
        plan.copy_stream, plan.compute_stream = copy.cuda_stream, compute.cuda_stream
        launches_per_step = n_b

        def step(record):
            # the timed region runs the asynchronous loop: no per-launch events, no host wait
            plan.kernel_ms, plan.kernel_ms_len = None, 0
            ps.ps_step_update_bucketed(spec, hp(), shard, plan)
            step_no[0] += 1

        def timed_pass(steps):
            """Per-launch durations of the update kernel (HIP events recorded by the library on
            the compute stream around each bucket's launch), in a pass of its own."""
            plan.kernel_ms, plan.kernel_ms_len = ms, n_b
            for _ in range(steps):
                ps.ps_step_update_bucketed(spec, hp(), shard, plan)
                kernel_ms.extend(ms[b] for b in range(n_b))   # every launch, the short last bucket too
                step_no[0] += 1
            plan.kernel_ms, plan.kernel_ms_len = None, 0
        elems_per_launch = cost.valid_len / n_b               # average over the launches of a step
    else:
        zero1, k_mb = w.strategy == "zero1", w.micro_batches
        if zero1:      # the all-reduced gradient: one replicated buffer of psi_padded elements
            grads = [dgen.fill_gradient_(torch.empty(cost.psi_padded, dtype=tdt, device="cuda"),
                                         w.seed, w.first_step, 0, w.grad_std)]
        elif arena is not None:
            grads = [dgen.fill_gradient_(dgen.as_tensor(a_buf[r], n, tdt), w.seed, w.first_step, r,
                                         w.grad_std * w.loss_scale, w.outlier_frac, w.outlier_mult,
                                         w.student_t_dof) for r in range(N)]
        else:
            grads = dgen.workload_gradients(w, w.first_step)
        g = ps.make_grads([t.data_ptr() for t in grads], dt)
        if k_mb > 1:
            accum = (dgen.as_tensor(a_buf[a_acc], n, torch.float32) if arena is not None
                     else torch.empty(n, dtype=torch.float32, device="cuda"))
            g_last = ps.make_grads([t.data_ptr() for t in grads], dt, accum=accum.data_ptr())
        launches_per_step = 1
        elems_per_launch = cost.valid_len
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(args.steps)]
        if clip:
            red = (dgen.as_tensor(a_buf[a_red], n, torch.float32) if arena is not None
                   else torch.empty(n, dtype=torch.float32, device="cuda"))
            ssd = torch.zeros(1, dtype=torch.float64, device="cuda")
            ws = torch.empty(ps.ps_workspace_bytes(n), dtype=torch.uint8, device="cuda")
            gred = ps.make_grads([red.data_ptr()], ps.PS_F32)
            others = torch.zeros(1, dtype=torch.float64, device="cuda")
            coef_dev = torch.zeros(1, dtype=torch.float32, device="cuda")
        rec = [0]

        def step(record):
            with torch.cuda.stream(compute):
                s = compute.cuda_stream
                if record:
                    ev[rec[0]][0].record(compute)
                if clip:
                    ps.ps_step_reduce_sumsq(spec, g, 0.0, red.data_ptr(), ssd.data_ptr(), 0,
                                            ws.data_ptr(), ws.numel(), 0, n, cost.valid_len, s)
                    if args.clip_on_host:
                        ss = float(ssd.item())      # the one device->host sync of such a step
                        coef = ps.ps_clip_coef(ss, 5.0 * ss, w.max_grad_norm)   # five iid peer shards
                        ps.ps_step_update(spec, hp(coef, 1.0), shard, gred, 0, n, s)
                    else:                           # everything stays on the stream
                        torch.mul(ssd, 5.0, out=others)     # stands for the peers' all-reduced sums
                        ps.ps_step_clip_coef(ssd.data_ptr(), others.data_ptr(), w.max_grad_norm,
                                             coef_dev.data_ptr(), s)
                        h = hp(0.0, 1.0)
                        h.clip_coef_device = coef_dev.data_ptr()
                        ps.ps_step_update(spec, h, shard, gred, 0, n, s)
                elif k_mb > 1:
                    for j in range(k_mb - 1):   # the same resident contributions stand for each micro-batch
                        ps.ps_step_accumulate(spec, g, accum.data_ptr(), j == 0, 0, n,
                                              cost.valid_len, s)
                    # the last one goes straight into the update, beside the accumulator
                    ps.ps_step_update(spec, hp(0.0, 1.0 / (N * k_mb)), shard, g_last, 0, n, s)
                else:
                    ps.ps_step_update(spec, hp(), shard, g, 0, n, s)
                if record:
                    ev[rec[0]][1].record(compute)
                    rec[0] += 1
            step_no[0] += 1
    torch.cuda.synchronize()
    log("setup %.1f s, %.1f GB allocated" % (time.time() - t_setup,
                                             (free_at_start - torch.cuda.mem_get_info()[0]) / 1e9))

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    if bucketed:
        timed_pass(args.steps)
    else:
        kernel_ms.extend(a.elapsed_time(b) for a, b in ev)
    elems_per_step = cost.valid_len
    value = elems_per_step / (ms_per_step * 1e-3)
    bpe = bytes_per_elem(w, clip)
    avg_ms = sum(kernel_ms) / len(kernel_ms)
    achieved = bpe * elems_per_launch / (avg_ms * 1e-3) / 1e9
    log("%.3f ms/step, %.3e elements/s; dominant kernel %.3f ms avg -> %.0f GB/s" %
        (ms_per_step, value, avg_ms, achieved))

    # Other ways through the same bucket loop on the same source, as context; none of them is
    # the headline value: the pipeline that stages each bucket first (copy kernel taking turns
    # with the update, or side by side; DMA copies), and the loop that reads in place.
    extras = {}
    if bucketed and args.extras:
        variants = [("in_place", ps.PS_COPY_NONE, ps.PS_SCHED_AUTO),
                    ("staged_copy_kernel_alternate", ps.PS_COPY_KERNEL, ps.PS_SCHED_ALTERNATE),
                    ("staged_copy_kernel_overlap", ps.PS_COPY_KERNEL, ps.PS_SCHED_OVERLAP),
                    ("staged_reduce_kernel_alternate", ps.PS_COPY_REDUCE, ps.PS_SCHED_ALTERNATE),
                    ("staged_reduce_kernel_overlap", ps.PS_COPY_REDUCE, ps.PS_SCHED_OVERLAP)]
        if pool_elems % B == 0:
            variants.append(("staged_memcpy_overlap", ps.PS_COPY_MEMCPY, ps.PS_SCHED_OVERLAP))
        keep = (plan.copy_engine, plan.schedule)
        for name, eng, sch in variants:
            plan.copy_engine, plan.schedule = eng, sch
            step(False)
            torch.cuda.synchronize()
            o0 = time.perf_counter()
            for _ in range(3):
                step(False)
            torch.cuda.synchronize()
            o_ms = (time.perf_counter() - o0) * 1e3 / 3
            before = len(kernel_ms)
            timed_pass(1)
            k_ms = kernel_ms[before:]
            del kernel_ms[before:]
            extras[name] = {"ms_per_step": o_ms, "step_GBps": bpe * elems_per_step / (o_ms * 1e-3) / 1e9,
                            "update_kernel_ms_avg": sum(k_ms) / len(k_ms)}
        plan.copy_engine, plan.schedule = keep
    # One plain copy of known size: the yardstick that hardware byte counters are scaled by.
    nbytes = min(master.numel() * 4, 1 << 32)
    reps = 5 if args.extras else 1
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(compute):
        e0.record(compute)
        for _ in range(reps):
            ps.ps_probe_copy(m.data_ptr(), v.data_ptr(), nbytes, compute.cuda_stream)
        e1.record(compute)
    torch.cuda.synchronize()
    cp_ms = e0.elapsed_time(e1) / reps
    extras["copy_probe"] = {"bytes": nbytes, "ms": cp_ms, "GBps": 2 * nbytes / (cp_ms * 1e-3) / 1e9}
    log("extras: %s" % json.dumps(extras))

    result = {
        "metric": "fused shard reduce+AdamW+cast: HBM GB/s and % of MI355X peak, elements/s",
        "value": value, "unit": "elements/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "psi": w.psi, "n_devices": N, "shard_index": w.shard_index,
                   "shard_elems": n, "grad_dtype": w.grad_dtype, "param_dtype": w.param_dtype, "strategy": w.strategy,
                   "bucket_elems": (B if bucketed else 0), "launches_per_step": launches_per_step,
                   "bucket_source": ((("every bucket of every contribution resident in HBM and distinct "
                                       "(%d elements per contribution, %.1f GB in all)"
                                       % (n, N * n * esz / 1e9)) if pool_elems >= n else
                                      ("resident pool of %d elements per contribution (%.2f GB in all), "
                                       "repeating" % (pool_elems, N * pool_elems * esz / 1e9))) +
                                     ("; read in place by the update kernel, one launch per bucket"
                                      if args.copy_engine == "none" else
                                      "; staged per bucket into two slots: copy engine %s, schedule %s"
                                      % (args.copy_engine, args.schedule)) +
                                     (" (source in pinned HOST memory)" if args.source_host else ""))
                                    if bucketed else None,
                   "staged_pipeline": ("not in this figure: the source is resident, nothing is copied; the "
                                       "two-stream pipeline that stages each bucket first is timed by --extras "
                                       "and in profiles/stage_update__70b_zero3__hbm_traffic.txt (70-105 ms per "
                                       "step from a source in HBM)") if bucketed and args.copy_engine == "none"
                                      else None,
                   "allocation": ("arena: flat buffers, physical memory created chunk by chunk (%s)"
                                  % ("bucket by bucket" if bucketed else "2^28 elements")
                                  if arena is not None else "one plain allocation per buffer"),
                   "clip_coefficient": (("host (one sync per step)" if args.clip_on_host
                                         else "device (no host round trip)") if clip else None),
                   "bytes_per_elem": bpe, "step_GBps": bpe * elems_per_step / (ms_per_step * 1e-3) / 1e9,
                   "device": info.name.decode(), "arch": info.arch.decode(),
                   "compute_units": info.compute_units, "memory_clock_khz": info.memory_clock_khz,
                   "memory_bus_bits": info.memory_bus_bits, "hbm_total_GB": info.total_bytes / 1e9},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": achieved / PEAK_HBM_GBS,
                     # the same bytes over the wall time of whole steps (the target metric);
                     # `achieved` and `frac` above are the dominant kernel's own launches
                     "step_achieved": bpe * elems_per_step / (ms_per_step * 1e-3) / 1e9,
                     "step_frac": bpe * elems_per_step / (ms_per_step * 1e-3) / 1e9 / PEAK_HBM_GBS,
                     "traffic": measured_traffic(w, elems_per_launch),
                     "kernel": ("reduce_sumsq_tiles+update_tiles" if clip else
                                "accumulate_tiles x%d + update_tiles (last micro-batch and accumulator)" % (w.micro_batches - 1)
                                if w.micro_batches > 1 else "update_tiles"),
                     "elems_per_launch": elems_per_launch, "avg_launch_ms": avg_ms,
                     "median_launch_ms": sorted(kernel_ms)[len(kernel_ms) // 2],
                     "best_launch_ms": min(kernel_ms), "launches_timed": len(kernel_ms),
                     "launch_timing": ("a pass of %d steps after the timed region, HIP events around "
                                       "each launch on the compute stream" % args.steps) if bucketed
                                      else "HIP events around each step's launches in the timed region"},
        "extras": extras,
    }
    # the plain copy kernel of the same launch shape as a second yardstick beside the nominal peak
    result["roofline"]["copy_yardstick"] = extras["copy_probe"]["GBps"]
    result["roofline"]["frac_of_copy_yardstick"] = achieved / extras["copy_probe"]["GBps"]
    if arena is not None:       # every view of its buffers is dead from here on
        torch.cuda.synchronize()
        ps.ps_arena_destroy(arena)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, bpe, args.cpu_baseline_seconds)
    print(json.dumps(result), flush=True)


def placement_map(args):
    """Measurement aid behind ps_arena_create: the update kernel on one 2^28-element bucket
    of the 70B workload whose eight contributions (a cluster of 4 GiB) and whose state and
    parameters (a cluster of 3.5 GiB) are placed at chosen offsets of ONE 248 GiB allocation.
    Prints the time per launch for every pair of offsets on a 16 GiB grid: which parts of the
    address space go together, and what it costs when they do not."""
    import torch

    import paper_2601_02311_amd as ps
    from synth import WORKLOADS

    w = WORKLOADS["70b_zero3"]
    torch.cuda.set_device(0)
    info = ps.ps_device_info()
    GiB, B, N = 1 << 30, w.bucket_elems, w.n_devices
    total = 248 * GiB
    big = torch.zeros(total, dtype=torch.uint8, device="cuda")
    base = big.data_ptr()
    spec = ps.ps_spec_preset(w.strategy, N, 0, B * N)          # one bucket stands for the shard
    hp = ps.ps_adamw_t(w.lr, w.beta1, w.beta2, w.eps, w.weight_decay, w.first_step, 0.0, 0.0)
    st = torch.cuda.current_stream().cuda_stream
    xs = list(range(0, 248 - 3, 16))
    ys = list(range(4, 248 - 3, 16))
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    rows = []
    for x in xs:
        row = []
        for y in ys:
            g = ps.make_grads([base + x * GiB + r * (GiB // 2) for r in range(N)], ps.PS_BF16)
            sh = ps.ps_shard_t(base + y * GiB, base + (y + 1) * GiB, base + (y + 2) * GiB,
                               base + (y + 3) * GiB, B, B, ps.PS_BF16, 0)
            ps.ps_step_update(spec, hp, sh, g, 0, B, st)
            e0.record()
            for _ in range(args.steps):
                ps.ps_step_update(spec, hp, sh, g, 0, B, st)
            e1.record()
            torch.cuda.synchronize()
            row.append(e0.elapsed_time(e1) / args.steps)
        rows.append(row)
        log("contributions at %3d GiB: " % x + " ".join("%.3f" % t for t in row))
    # Second table: relative alignment of the twelve streams.  All of them in one placement
    # group (the first 16 GiB), stream k at k GiB + k * shift bytes for a few shifts.
    shifts = [0, 256, 4096, 4352, 65536, 260 << 10, (1 << 20) + 8192]
    align_ms = []
    for sh_b in shifts:
        at = lambda k: base + k * GiB + k * sh_b
        g = ps.make_grads([at(r) for r in range(N)], ps.PS_BF16)
        sh = ps.ps_shard_t(at(8), at(9), at(10), at(11), B, B, ps.PS_BF16, 0)
        ps.ps_step_update(spec, hp, sh, g, 0, B, st)
        e0.record()
        for _ in range(args.steps):
            ps.ps_step_update(spec, hp, sh, g, 0, B, st)
        e1.record()
        torch.cuda.synchronize()
        align_ms.append(e0.elapsed_time(e1) / args.steps)
    log("stream k at k GiB + k * shift: " + ", ".join("%d B: %.3f ms" % p for p in zip(shifts, align_ms)))
    flat = sorted(t for r in rows for t in r)
    fast = [t for t in flat if t < (flat[0] + flat[-1]) / 2]
    slow = [t for t in flat if t >= (flat[0] + flat[-1]) / 2]
    print(json.dumps({
        "metric": "update kernel, ms per 2^28-element bucket, by placement of its operands",
        "value": sum(fast) / len(fast), "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": 1,
        "ms_per_step": sum(flat) / len(flat), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "placement_map", "device": info.name.decode(),
                   "allocation_GiB": 248, "contribution_offsets_GiB": xs, "state_offsets_GiB": ys,
                   "ms": rows, "fast_pairs": len(fast), "fast_ms_avg": sum(fast) / len(fast),
                   "slow_pairs": len(slow), "slow_ms_avg": sum(slow) / max(1, len(slow)),
                   "alignment_shift_bytes": shifts, "alignment_ms": align_ms},
        "roofline": {"bound": "hbm", "achieved": 42 * B / (sum(fast) / len(fast)) / 1e6,
                     "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": 42 * B / (sum(fast) / len(fast)) / 1e6 / PEAK_HBM_GBS, "traffic": None,
                     "kernel": "update_tiles, operands in parts of the address space that go together"}}),
          flush=True)


def offload_bench(args):
    """ZeRO-Offload row: state in pinned host memory, streamed through three device slots."""
    import torch

    import paper_2601_02311_amd as ps
    from synth import WORKLOADS
    from synth import device as dgen

    w = WORKLOADS["7b_offload"]
    torch.cuda.set_device(0)
    info = ps.ps_device_info()
    n, N, B = w.shard_len, w.n_devices, (args.bucket_elems or w.bucket_elems)
    spec = ps.ps_spec_preset(w.strategy, N, w.shard_index, w.psi)
    plan = ps.ps_offload_plan_t()
    n_b = -(-n // B)
    state = dgen.workload_state(w)
    if args.offload_layout == "packed":
        # one pinned image, bucket by bucket master | m | v | parameters: one copy per direction
        image = torch.empty(n_b * 14 * B, dtype=torch.uint8).pin_memory()
        for b in range(n_b):
            lo, hi = b * B, min((b + 1) * B, n)
            for j, t in enumerate(state):
                image[b * 14 * B + 4 * B * j:b * 14 * B + 4 * B * j + 4 * (hi - lo)].copy_(
                    t[lo:hi].view(torch.uint8))
        plan.host_layout, plan.host_packed = ps.PS_HOST_PACKED, image.data_ptr()
    else:
        master, m, v = [t.cpu().pin_memory() for t in state]
        out = torch.zeros(n, dtype=torch.bfloat16).pin_memory()
        plan.host_master, plan.host_m, plan.host_v, plan.host_param_out = (master.data_ptr(), m.data_ptr(),
                                                                           v.data_ptr(), out.data_ptr())
    del state
    torch.cuda.empty_cache()
    grads = dgen.workload_gradients(w, w.first_step)
    slots = [torch.empty(14 * B, dtype=torch.uint8, device="cuda") for _ in range(3)]
    s1, s2, s3 = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    plan.len, plan.valid_len, plan.bucket_elems, plan.n_slots = n, n, B, 3
    for k, t in enumerate(slots):
        plan.slot[k] = t.data_ptr()
    plan.h2d_stream, plan.compute_stream, plan.d2h_stream = s1.cuda_stream, s2.cuda_stream, s3.cuda_stream
    g = ps.make_grads([t.data_ptr() for t in grads], ps.PS_BF16)
    t_no = [w.first_step]

    def step():
        hp = ps.ps_adamw_t(w.lr, w.beta1, w.beta2, w.eps, w.weight_decay, t_no[0], 0.0, 0.0)
        ps.ps_step_update_offloaded(spec, hp, plan, g)     # consecutive steps are ordered on the streams
        t_no[0] += 1
        if args.sync_each_step:
            torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    up, down = 12 * n, 14 * n
    log("%.3f ms/step: %.1f GB/s up, %.1f GB/s down over the host link" %
        (ms_per_step, up / ms_per_step / 1e6, down / ms_per_step / 1e6))

    # Yardstick, like the copy kernel for HBM: the same bytes over the same link as plain
    # pinned copies, 12 B bytes up and 14 B bytes down per bucket, both directions at once.
    # The host side of the probe walks the step's own pinned memory, bucket after bucket (its
    # contents are not needed any more): a small buffer copied over and over would stay in the
    # host's caches and hide what the host's memory costs when other jobs share it.
    host = image if args.offload_layout == "packed" else master.view(torch.uint8)
    span = (host.numel() - 14 * B) // 4096 * 4096
    dev_up = torch.empty(12 * B, dtype=torch.uint8, device="cuda")
    dev_down = torch.empty(14 * B, dtype=torch.uint8, device="cuda")

    def probe(do_up, do_down):
        torch.cuda.synchronize()
        p0 = time.perf_counter()
        for b in range(n_b):
            at = (b * 14 * B) % span if span > 0 else 0
            if do_up:
                with torch.cuda.stream(s1):
                    dev_up.copy_(host[at:at + 12 * B], non_blocking=True)
            if do_down:
                with torch.cuda.stream(s3):
                    host[at:at + 14 * B].copy_(dev_down, non_blocking=True)
        torch.cuda.synchronize()
        return (time.perf_counter() - p0) * 1e3
    probe(True, True)
    both_ms, up_ms, down_ms = probe(True, True), probe(True, False), probe(False, True)
    link = {"both_directions_ms": both_ms,
            "up_GBps_both": 12 * B * n_b / both_ms / 1e6, "down_GBps_both": 14 * B * n_b / both_ms / 1e6,
            "up_GBps_alone": 12 * B * n_b / up_ms / 1e6, "down_GBps_alone": 14 * B * n_b / down_ms / 1e6,
            "note": "plain pinned copies of the step's bytes over the step's own host memory, one per "
                    "direction per bucket"}
    log("link probe: %s" % json.dumps(link))
    print(json.dumps({
        "metric": "offloaded shard reduce+AdamW+cast: host-link GB/s, elements/s",
        "value": n / (ms_per_step * 1e-3), "unit": "elements/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "shard_elems": n, "n_devices": N, "bucket_elems": B,
                   "slots": 3, "host_layout": args.offload_layout, "device": info.name.decode()},
        "roofline": {"bound": "host link (PCIe, full duplex)", "achieved": down / ms_per_step / 1e6,
                     "peak": 64.0, "unit": "GB/s", "frac": down / ms_per_step / 1e6 / 64.0,
                     "frac_of_link_probe": both_ms * n / (n_b * B) / ms_per_step,
                     "traffic": None, "note": "the busier direction: 14 bytes per element device to host; "
                     "peak is PCIe 5.0 x16 per direction; frac_of_link_probe = time plain pinned copies "
                     "of the same bytes take / time of the step"},
        "extras": {"link_probe": link}}), flush=True)


def verify_bench(args):
    """The verification protocol's two scans on buffers of the 7B shard: relative difference
    of two bf16 gradient copies and the checksum of the FP32 master shard."""
    import torch

    import paper_2601_02311_amd as ps
    from synth import WORKLOADS
    from synth import device as dgen

    w = WORKLOADS["7b_zero2"]
    torch.cuda.set_device(0)
    info = ps.ps_device_info()
    n = w.shard_len
    a = dgen.fill_gradient_(torch.empty(n, dtype=torch.bfloat16, device="cuda"), w.seed, 1, 0, w.grad_std)
    b = a.clone()
    b[12345] += 1.0
    master, _, _ = dgen.workload_state(w)
    ws = torch.empty(ps.ps_verify_workspace_bytes(n * 4), dtype=torch.uint8, device="cuda")
    out2 = torch.zeros(2, dtype=torch.float64, device="cuda")
    outc = torch.zeros(1, dtype=torch.int64, device="cuda")
    st = torch.cuda.current_stream().cuda_stream

    def step():
        ps.ps_verify_diff_sumsq(a.data_ptr(), b.data_ptr(), ps.PS_BF16, n, out2.data_ptr(), 0,
                                ws.data_ptr(), ws.numel(), st)
        ps.ps_verify_checksum(master.data_ptr(), n * 4, 0, outc.data_ptr(), 0, ws.data_ptr(),
                              ws.numel(), st)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    t_diff = t_sum = 0.0
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ev[0].record()
        ps.ps_verify_diff_sumsq(a.data_ptr(), b.data_ptr(), ps.PS_BF16, n, out2.data_ptr(), 0,
                                ws.data_ptr(), ws.numel(), st)
        ev[1].record()
        ps.ps_verify_checksum(master.data_ptr(), n * 4, 0, outc.data_ptr(), 0, ws.data_ptr(),
                              ws.numel(), st)
        ev[2].record()
        torch.cuda.synchronize()
        t_diff += ev[0].elapsed_time(ev[1])
        t_sum += ev[1].elapsed_time(ev[2])
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    t_diff /= args.steps
    t_sum /= args.steps
    sd, sa = out2.cpu().tolist()
    achieved = (4 * n + 4 * n) / ((t_diff + t_sum) * 1e-3) / 1e9
    log("diff scan %.3f ms (%.0f GB/s), checksum %.3f ms (%.0f GB/s); relative difference %.3e" %
        (t_diff, 4 * n / t_diff / 1e6, t_sum, 4 * n / t_sum / 1e6, (sd / sa) ** 0.5))
    print(json.dumps({
        "metric": "verification scans (relative gradient difference + state checksum): HBM GB/s, elements/s",
        "value": 2 * n / ((t_diff + t_sum) * 1e-3), "unit": "elements/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64",
        "data": "synthetic",
        "config": {"workload": "7b_verify", "shard_elems": n, "device": info.name.decode(),
                   "diff_ms": t_diff, "checksum_ms": t_sum},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": achieved / PEAK_HBM_GBS, "traffic": None,
                     "kernel": "diff_sumsq_tiles + checksum_tiles"}}), flush=True)


def measured_traffic(w, elems_per_launch):
    """HBM bytes per launch of the dominant kernel from the committed hardware-counter summary
    (profiles/update_tiles__<workload>__hbm_traffic.txt).  None when there is no summary for this
    workload or when the kernel sources have changed since the counters were taken."""
    import hashlib
    path = os.path.join(ROOT, "profiles", "update_tiles__%s__hbm_traffic.txt" % w.name)
    if not os.path.exists(path):
        return None
    kv = {}
    for line in open(path):
        if "=" in line and not line.lstrip().startswith("#"):
            k, v = line.split("=", 1)
            kv[k.strip()] = v.split("#", 1)[0].strip()
    h = hashlib.sha256()
    for f in ("ps_kernel_templates.h", "ps_kernels.hip"):
        h.update(open(os.path.join(ROOT, "paper_2601_02311_amd", "csrc", f), "rb").read())
    if kv.get("kernel_sources_sha256") != h.hexdigest() or kv.get("workload") != w.name:
        return None
    return float(kv["hbm_bytes_per_element"]) * elems_per_launch


def cpu_baseline(w, bpe, seconds=15.0):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: contiguous
    index ranges of the sample handed to host threads that share nothing."""
    import numpy as np

    from oracle import step as orc
    from synth import host as gen

    cores = min(16, os.cpu_count() or 1)
    sample = min(w.shard_len, 1 << 26)
    grads = [gen.gradient(sample, w.seed, w.first_step, r, w.grad_dtype, w.grad_std * w.loss_scale,
                          w.outlier_frac, w.outlier_mult, w.student_t_dof)
             for r in range(w.n_devices)]
    th = gen.master(sample, w.seed)
    m, v = gen.moments(sample, w.seed, True)
    p = np.zeros(sample, np.float16 if w.param_dtype == "f16" else np.uint16)
    s = orc.derive_scalars(w.lr, w.beta1, w.beta2, w.eps, w.weight_decay, w.first_step,
                           w.n_devices, grad_scale=(1.0 / (w.n_devices * w.loss_scale)
                                                    if w.loss_scale != 1.0 else 0.0))
    bounds = [sample * k // cores for k in range(cores + 1)]

    def one_pass():
        ts = [threading.Thread(target=orc.step_f32, args=(grads, s, th, m, v, p, bounds[k], bounds[k + 1]))
              for k in range(cores)]
        t0 = time.perf_counter()
        for t in ts:
            t.start()
        for t in ts:
            t.join()
        return time.perf_counter() - t0
    first = one_pass()
    reps = max(1, min(2000, int(seconds / max(first, 1e-3))))
    total = sum(one_pass() for _ in range(reps))
    rate = sample * reps / total
    # and one thread alone on an eighth of the sample
    t0 = time.perf_counter()
    orc.step_f32(grads, s, th, m, v, p, 0, sample // 8)
    single = (sample // 8) / (time.perf_counter() - t0)
    cpu = "?"
    try:
        cpu = [l.split(":", 1)[1].strip() for l in open("/proc/cpuinfo") if l.startswith("model name")][0]
    except (OSError, IndexError):
        pass
    log("cpu oracle on %s (%d logical cpus): %d threads, %d x %d elements in %.1f s -> %.3e "
        "elements/s; one thread %.3e elements/s" %
        (cpu, os.cpu_count() or 0, cores, reps, sample, total, rate, single))
    return {"value": rate, "unit": "elements/s", "cores": cores, "kind": "oracle",
            "GBps": rate * bpe / 1e9, "single_thread_value": single, "cpu_model": cpu,
            "logical_cpus": os.cpu_count(),
            "sample": "%d passes over the first %d elements of the shard (%s gradients, N=%d), "
                      "split into %d contiguous ranges" % (reps, sample, w.grad_dtype, w.n_devices, cores)}


if __name__ == "__main__":
    main()
