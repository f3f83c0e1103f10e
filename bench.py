#!/usr/bin/env python3
"""Benchmark of the shadow update on one MI355X.

A step is one whole iteration of the hot path over one batch of synthetic
gradients: every bucket of the model is folded over its W worker views, the
global gradient norm is formed, and the optimizer (AdamW) is applied to the fp32 replica.
Inputs (replica and all W views of every bucket) are resident in HBM before
the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llama7b]
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

HBM_PEAK_GBS = 8000.0     # MI355X HBM3E, published peak

# HBM bytes per launch of the roofline kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this file with
# its defaults (profiles/*_bench_rocprofv3.md), each counter scaled by what it reads for the library's plain copy
# kernel over 1 GiB.  Keyed by (workload, kernel, --refold, --no-clip); only reported for default settings and while
# the kernel sources (comments and white space aside) still hash to the value the counters were taken at.
MEASURED_TRAFFIC_SOURCES_SHA256 = "b26970498f3cd84845e40be7b5e0d562d40d35006827bf5db9ad782edabe3bc7"
MEASURED_TRAFFIC = {
    ("llama7b", "k_adamw", False, False): 188694396768.8,
    ("ragged7b", "k_fold_sumsq", False, False): 5669610391.2,
    ("gpt1p3b", "k_fold_sumsq", False, False): 4744638522.5,
    ("llama7b_w1", "k_fold_adamw", True, False): 21903620378.2,
    ("gpt2s", "k_fold_adamw", False, False): 4978158580.1,
    ("llama7b", "k_fold_adamw", False, True): 11231687037.0,
}
KERNEL_SOURCES = ("paper_2507_13522_amd/csrc/shadow_kernels.hip.h", "paper_2507_13522_amd/csrc/shadow.hip")


def kernel_sources_hash() -> str:
    """sha256 of the kernel and launch sources with comments and white space taken out: it changes when the code does."""
    import hashlib
    import re
    h = hashlib.sha256()
    for f in KERNEL_SOURCES:
        with open(os.path.join(ROOT, f), "r") as fh:
            text = fh.read()
        text = re.sub(r"/\*.*?\*/", " ", text, flags=re.S)
        text = re.sub(r"//[^\n]*", " ", text)
        h.update(" ".join(text.split()).encode())
    return h.hexdigest()


def measured_traffic(workload: str, kernel: str, refold: bool, noclip: bool, defaults: bool):
    rec = MEASURED_TRAFFIC.get((workload, kernel, refold, noclip))
    if rec is None or not defaults:
        return None
    return rec if kernel_sources_hash() == MEASURED_TRAFFIC_SOURCES_SHA256 else None


VIEW_RING_BYTES = 96 << 30       # ring of gradient views for workloads whose views do not all fit in HBM

KERNEL_NAMES = {0: "k_fold_adamw", 1: "k_fold_sumsq", 2: "k_norm_finalize", 3: "k_adamw", 4: "snapshot_copies"}


def algorithmic_bytes_per_param(wl, refold: bool = False, optimizer: str = "adamw") -> dict:
    """Bytes the method must move per parameter and step, by kernel: every gradient view read once (W*G), p, m
    (and v) read and written once, and with clipping the fp32 reduced gradient written and read once (or the views
    read a second time when no scratch arena is given)."""
    g = wl.grad_bytes * wl.num_workers
    st = 16 if optimizer == "sgd" else 24        # state read + written: p, m (, v)
    if wl.max_grad_norm > 0 and refold:          # views folded twice, reduced gradient never stored
        return {"k_fold_sumsq": g, "k_fold_adamw": g + st, "total": 2 * g + st}
    if wl.max_grad_norm > 0:
        return {"k_fold_sumsq": g + 4, "k_adamw": 4 + st, "total": g + 8 + st}
    return {"k_fold_adamw": g + st, "total": g + st}


def cpu_baseline(wl, inputs, target_seconds: float = 15.0, optimizer: str = "adamw") -> dict:
    """Time the oracle, as it stands, on this machine's host cores over a bounded sample of the same workload."""
    import numpy as np
    import oracle

    lay = oracle.build_layout([(t.numel, t.weight_decay) for t in wl.tensors], wl.grad_bytes, wl.bucket_cap_bytes,
                              wl.explicit_buckets)
    starts = lay.logical_starts()
    hp = oracle.HParams(lr=wl.lr, beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps, weight_decay=wl.weight_decay,
                        max_grad_norm=wl.max_grad_norm, mean=True, optimizer=optimizer)
    threads = oracle.get_threads()
    # sample: buckets in id order until ~64M elements (bounded host memory), repeated until the time budget is used
    chosen, total = [], 0
    for b, bk in enumerate(lay.buckets):
        chosen.append(b)
        total += bk.numel
        if total >= 64_000_000:
            break
    data = {}
    for b in chosen:
        n = lay.buckets[b].numel
        data[b] = dict(g=[inputs.grad_np(1, w, starts[b], n) for w in range(wl.num_workers)],
                       p=inputs.param_np(starts[b], n), m=np.zeros(n, np.float32), v=np.zeros(n, np.float32))
    params = [data[b]["p"] if b in data else None for b in range(len(lay.buckets))]
    orc = oracle.OracleShadow(lay, hp, params)
    t = 0

    def timed(budget: float, max_iters: int):
        nonlocal t
        done, t_used, iters = 0, 0.0, 0
        while t_used < budget and iters < max_iters:
            t += 1
            iters += 1
            t0 = time.perf_counter()
            r = {b: oracle.fold(data[b]["g"], hp.mean) for b in chosen}
            c = None
            if hp.max_grad_norm > 0:
                s = oracle.SumSq()
                for b in chosen:
                    s.add(r[b])
                c = s.coef(hp.max_grad_norm)
            for b in chosen:
                orc.update_bucket(b, r[b], t, c)
            t_used += time.perf_counter() - t0
            done += total
        return done / t_used, iters, t_used

    rate, iters, t_used = timed(target_seconds, 200)
    # the same loop on one thread, a third of the budget
    oracle.set_threads(1)
    try:
        rate1, iters1, t_used1 = timed(target_seconds / 3, 50)
    finally:
        oracle.set_threads(threads)
    cpu = "unknown"
    try:
        with open("/proc/cpuinfo") as fh:
            cpu = next((ln.split(":", 1)[1].strip() for ln in fh if ln.startswith("model name")), cpu)
    except OSError:
        pass
    return {"value": rate, "unit": "params/s", "cores": threads, "kind": "oracle",
            "sample": f"{len(chosen)} buckets ({total} params) of {wl.name}, {iters} oracle iterations "
                      f"(fold W={wl.num_workers} {wl.grad_dtype}, norm, {optimizer}), {t_used:.1f} s of CPU work, "
                      f"OpenMP threads={threads}, host cpus={os.cpu_count()}, cpu={cpu}",
            "value_single_thread": rate1,
            "sample_single_thread": f"same buckets, {iters1} iterations, {t_used1:.1f} s on one thread"}


PROBE_SHAPES = ((64, 12), (128, 8), (128, 16), (256, 16), (256, 0), (1024, 0))     # (threads per block, waves per CU; 0 = no bound)


def stream_probe(torch, sh, reps: int, gib: int) -> int:
    """What the chip sustains for the update kernels' mixes of streams: the same access pattern (one 16-byte vector per
    lane and array, all loads first, non-temporal), launch shape and placement in HBM, without the arithmetic."""
    GiB = 1 << 30
    n = gib * GiB                                             # bytes per array
    try:
        block = torch.empty(256 * GiB, dtype=torch.uint8, device="cuda:0")
        a = n + GiB
        assert 3 * a <= 96 * GiB and 97 * GiB + a + 16 * (n + (2 << 20) + 4096) <= 256 * GiB, "arrays too large for the block"
        off = {"r": 96 * GiB - 3 * a, "p": 96 * GiB - 2 * a, "m": 96 * GiB - a, "v": 97 * GiB}
        for k in range(16):
            off[f"g{k}"] = 97 * GiB + a + k * (n + (2 << 20) + 4096)
        placement = "state arrays end the first 96 GiB of a 256 GiB block and start the second, views behind them"
    except torch.OutOfMemoryError:
        torch.cuda.empty_cache()
        names = ["r", "p", "m", "v"] + [f"g{k}" for k in range(16)]
        block = torch.empty(len(names) * (n + (2 << 20) + 4096), dtype=torch.uint8, device="cuda:0")
        off = {name: i * (n + (2 << 20) + 4096) for i, name in enumerate(names)}
        placement = "one allocation, arrays back to back"
    for name, o in off.items():
        block[o:o + n].zero_()
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda:0")
    ptr = lambda name: block.data_ptr() + off[name]
    views = lambda k: [f"g{i}" for i in range(k)]
    mixes = [  # name, sources, destinations, block, waves per CU (the update kernel's own default shape)
        ("copy", ["p"], ["v"], 256, 0),
        ("reads alone, 4 arrays", ["r", "p", "m", "v"], [], 256, 16),
        ("writes alone, 3 arrays", [], ["p", "m", "v"], 256, 16),
        ("k_adamw: r, p, m, v in; p, m, v out in place", ["r", "p", "m", "v"], ["p", "m", "v"], 256, 16),
        ("k_fold_sumsq W=8 bf16: 16 B/param in, r out", views(4), ["r"], 1024, 0),
        ("k_fold_sumsq W=16 bf16: 32 B/param in, r out", views(8), ["r"], 128, 12),
        ("k_fold_sumsq W=32 bf16: 64 B/param in, r out", views(16), ["r"], 128, 8),
        ("k_fold_adamw W=8 bf16: 16 B/param of views, p, m, v in; p, m, v out in place", views(4) + ["p", "m", "v"], ["p", "m", "v"], 64, 11),
    ]
    def timed(src, dst, blk, waves):
        call = lambda: sh.shadow_stream_probe([ptr(d) for d in dst], [ptr(x) for x in src], n, sink=sink.data_ptr(), block=blk,
                                              waves_per_cu=waves)
        assert call() == 0
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            call()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        return ms, (len(src) + len(dst)) * n / (ms * 1e-3) / 1e9

    rows = []
    for name, src, dst, blk, waves in mixes:
        ms, gbps = timed(src, dst, blk, waves)
        best = max(((timed(src, dst, b, w)[1], b, w) for b, w in PROBE_SHAPES), key=lambda t: t[0])
        rows.append({"mix": name, "arrays_in": len(src), "arrays_out": len(dst), "block": blk, "waves_per_cu": waves or 32,
                     "ms": ms, "GBps": gbps, "frac_of_peak": gbps / HBM_PEAK_GBS,
                     "best_of_shapes": {"GBps": best[0], "block": best[1], "waves_per_cu": best[2] or 32}})
    print(json.dumps({"stream_probe": rows, "bytes_per_array": n, "launches_timed": reps, "placement": placement, "peak_GBps": HBM_PEAK_GBS,
                      "shapes_tried": [[b, w or 32] for b, w in PROBE_SHAPES]}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="llama7b")
    ap.add_argument("--streams", type=int, default=None)
    ap.add_argument("--batch-mib", type=int, default=None,
                    help="bucket scheduling: gradient MiB buffered per stream before one fold launch (0 = every bucket "
                         "its own launch; default: the whole iteration in as few launches as the descriptor allows)")
    ap.add_argument("--refold", action="store_true",
                    help="clipping without a scratch arena: fold the views twice instead of storing the reduced gradient")
    ap.add_argument("--optimizer", default="adamw", choices=["adamw", "adam", "sgd"])
    ap.add_argument("--no-clip", action="store_true", help="run the workload without global-norm clipping (fused kernel)")
    ap.add_argument("--workers", type=int, default=0, help="override the workload's number of workers W")
    ap.add_argument("--grad-dtype", default=None, choices=["bf16", "f32"], help="override the workload's gradient type")
    ap.add_argument("--ingest-slots", type=int, default=0,
                    help="hand the buckets over as pinned HOST views through a device ring of this many slots "
                         "(PCIe-inclusive rate; never the headline value)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-yardstick", action="store_true", help="skip timing the plain copy kernel")
    ap.add_argument("--fold-block", type=int, default=0)
    ap.add_argument("--fused-block", type=int, default=0)
    ap.add_argument("--sweep-block", type=int, default=0)
    ap.add_argument("--fold-waves", type=int, default=0, help="upper bound on the waves per CU of the fold + sum-of-squares kernel")
    ap.add_argument("--fused-waves", type=int, default=0, help="upper bound on the waves per CU of the fold + optimizer kernel")
    ap.add_argument("--sweep-waves", type=int, default=0, help="upper bound on the waves per CU of the optimizer sweep")
    ap.add_argument("--drain-blocks", type=int, default=0, help="blocks of the kernel that drains a snapshot to the host")
    ap.add_argument("--placement", default="auto", choices=["auto", "plan", "stride", "separate"],
                    help="where the arenas and views lie in HBM (auto: the library's device plan, else its stride advice)")
    ap.add_argument("--offsets-gib", default=None,
                    help="placement experiments: GiB offsets 'param,m,v,scratch,staging' inside one 256 GiB allocation")
    ap.add_argument("--snapshot-every", type=int, default=0,
                    help="take a snapshot of the replica every N-th timed iteration (0 = never)")
    ap.add_argument("--snapshot-mode", default="staged", choices=["staged", "copy"],
                    help="staged: the iteration's update also writes a staging set (shadow_snapshot_arm); "
                         "copy: device-to-device copies at the boundary (shadow_snapshot)")
    ap.add_argument("--snapshot-host", action="store_true",
                    help="drain every snapshot to pinned host memory (staged: from the staging set, concurrently with "
                         "later iterations; copy: straight from the replica)")
    ap.add_argument("--view-ring-gib", type=int, default=0,
                    help="let the buckets' views take turns in a ring of this many GiB instead of keeping all resident")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also launch the library's plain copy kernel once over this many MiB (known-traffic "
                         "yardstick for rocprofv3 byte counters)")
    ap.add_argument("--stream-probe", action="store_true",
                    help="instead of the update: time the library's streaming kernel (no arithmetic) for the mixes of read "
                         "and written arrays that the update kernels have, and print one JSON line")
    ap.add_argument("--probe-gib", type=int, default=4, help="GiB per array of --stream-probe (at most 8)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the shadow update runs on ONE GPU (no sharding across GPUs, no collectives); run with --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    import paper_2507_13522_amd as sh
    import synth
    from paper_2507_13522_amd.replica import BENCH_BATCH_BYTES, BENCH_STREAMS, GpuShadow
    from synth.inputs import TILE_PERIOD, Inputs
    streams = BENCH_STREAMS if args.streams is None else args.streams
    batch_bytes = BENCH_BATCH_BYTES if args.batch_mib is None else args.batch_mib << 20

    default_settings = (args.streams is None and args.batch_mib is None and args.optimizer == "adamw" and not args.ingest_slots
                        and not args.fold_block and not args.fused_block and not args.sweep_block and not args.fold_waves and not args.fused_waves and not args.sweep_waves
                        and args.placement == "auto" and not args.workers and not args.grad_dtype and not args.offsets_gib and not args.snapshot_every and not args.view_ring_gib)

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    if args.stream_probe:
        return stream_probe(torch, sh, args.steps, args.probe_gib)
    launch = sh.LaunchShape(fold_block=args.fold_block, fused_block=args.fused_block, sweep_block=args.sweep_block, fold_waves_per_cu=args.fold_waves,
                            fused_waves_per_cu=args.fused_waves, sweep_waves_per_cu=args.sweep_waves, drain_blocks=args.drain_blocks)

    wl = synth.get_workload(args.workload)
    if args.no_clip:
        wl.max_grad_norm = 0.0
    if args.workers:
        wl.num_workers = args.workers
    if args.grad_dtype:
        wl.grad_dtype = args.grad_dtype
    inputs = Inputs(wl, period=TILE_PERIOD)
    ingest = args.ingest_slots > 0
    # all W views of every bucket resident when they fit beside the replica; otherwise (W = 32 at 7B: 445 GB) the
    # buckets take turns in a ring of views, which moves the same bytes per step (values do not affect timing)
    ring_bytes = args.view_ring_gib << 30
    snapshots = args.snapshot_every > 0
    staged = snapshots and args.snapshot_mode == "staged"
    if not ingest and not ring_bytes:
        lay = sh.Layout([(t.numel, t.weight_decay) for t in wl.tensors], wl.grad_bytes, wl.bucket_cap_bytes, wl.explicit_buckets)
        state_bytes = lay.arena_numel * (16 + (12 if snapshots else 0))
        if state_bytes + lay.staging_bytes(wl.num_workers) > (250 << 30):
            ring_bytes = VIEW_RING_BYTES if not snapshots else 32 << 30
        lay.close()
    offsets = None
    if args.offsets_gib:
        vals = [int(float(x) * (1 << 30)) for x in args.offsets_gib.split(",")]
        offsets = dict(zip(("param", "m", "v", "scratch", "staging"), vals))
    g = GpuShadow(wl, inputs, num_streams=streams, batch_bytes=batch_bytes, refold=args.refold, optimizer=args.optimizer,
                  resident_grads=not ingest, ring_bytes=ring_bytes, placement="explicit" if offsets else args.placement, offsets=offsets,
                  snapshot_set=staged or (snapshots and not args.snapshot_host), attach_snapshot_set=staged, launch=launch)
    P = g.layout.num_params
    A = g.layout.arena_numel
    snap_dev = snap_host = None
    if snapshots and args.snapshot_host:
        # pinned host arrays for param, m, v; where the host cannot pin that much, as many of them as it can (the rest
        # of the snapshot then stays in the staging set / is not copied)
        snap_host = []
        for _ in range(3):
            try:
                snap_host.append(torch.empty(A, dtype=torch.float32, pin_memory=True))
            except RuntimeError:
                torch.cuda.synchronize()
                break
        if not snap_host:
            print("bench.py: cannot pin host memory for one array of the replica", file=sys.stderr)
            return 2
    elif snapshots and not staged:
        snap_dev = g.snap                      # a second set of arenas, placed with everything else
    snap_taken, snap_skipped = 0, 0

    def before_step(i):
        """staged snapshots are armed before the iteration whose end state they hold"""
        nonlocal snap_taken, snap_skipped
        if staged and (i + 1) % args.snapshot_every == 0:
            rc = g.ctx.try_snapshot_arm(*(([h.data_ptr() for h in snap_host] + [None, None])[:3] if snap_host else [None, None, None]))
            if rc == sh.binding.OK:
                snap_taken += 1
            elif rc == sh.binding.EBUSY:
                snap_skipped += 1          # the previous drain to the host is still running
            else:
                raise sh.ShadowError(rc, "shadow_snapshot_arm")

    def after_step(i):
        nonlocal snap_taken
        if snapshots and not staged and (i + 1) % args.snapshot_every == 0:
            dst = snap_host if snap_host else snap_dev
            g.ctx.snapshot(*([d.data_ptr() for d in dst] + [None, None])[:3])
            snap_taken += 1

    if ingest:
        # one pinned host buffer per worker, as long as the largest bucket, serves every bucket (values do not
        # affect timing); the device ring holds ingest_slots buckets
        nmax = max(n for _, n, _ in g.buckets)
        view_bytes = (nmax * wl.grad_bytes + 255) // 256 * 256
        host = [torch.zeros(view_bytes, dtype=torch.uint8).pin_memory() for _ in range(wl.num_workers)]
        ring = torch.empty(args.ingest_slots * wl.num_workers * view_bytes, dtype=torch.uint8, device="cuda:0")
        g.ctx.ingest_attach(ring.data_ptr(), ring.numel())
        hv = g.ctx.views_array([h.data_ptr() for h in host])

        def run_step(s):
            for b in range(len(g.buckets)):
                g.ctx.ingest_bucket(b, hv, s)
    else:
        if ring_bytes:
            g._stage.zero_()
        else:
            g.fill_grads(1)    # the same resident views serve every timed step (values do not affect timing)
        run_step = g.apply_step
    step = 0
    for _ in range(args.warmup):
        step += 1
        run_step(step)
    g.ctx.sync()
    if args.copy_probe_mib:
        nbytes = args.copy_probe_mib << 20
        src = torch.zeros(nbytes, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        sh.shadow_copy_probe(dst.data_ptr(), src.data_ptr(), nbytes, 0)
        torch.cuda.synchronize()
        del src, dst
    # yardstick: the library's plain copy kernel over 2 GiB (read 2 GiB + write 2 GiB), timed with events
    yard = None
    if not args.no_yardstick:
        nb = 2 << 30
        src = torch.zeros(nb, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        sh.shadow_copy_probe(dst.data_ptr(), src.data_ptr(), nb, 0)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            sh.shadow_copy_probe(dst.data_ptr(), src.data_ptr(), nb, 0)
        e1.record()
        torch.cuda.synchronize()
        yard = 5 * 2 * nb / (e0.elapsed_time(e1) * 1e-3) / 1e9
        del src, dst
    torch.cuda.synchronize()
    # per-step marks on the library's own stream (single-stream runs): no host synchronisation inside the timed region
    marks, mark_stream = None, None
    if streams == 1 and not ingest:
        mark_stream = torch.cuda.ExternalStream(g.ctx.bucket_stream(0))
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    # Inside the timed region only the kernel the roofline reports on is bracketed by events (the event records around
    # all 50-odd launches of an iteration cost about 0.2 ms of a 49.4 ms llama7b iteration); the other kernels' averages
    # come from a few more iterations behind the timed region.  With snapshots or host ingest every kind stays on.
    bpp = algorithmic_bytes_per_param(wl, args.refold, args.optimizer)
    dom = max((k for k in bpp if k != "total" and bpp[k] > 0), key=lambda k: bpp[k])
    dom_kind = next(kind for kind, name in KERNEL_NAMES.items() if name == dom)
    light = not snapshots and not ingest
    g.ctx.profile_kinds((1 << dom_kind) if light else (1 << len(KERNEL_NAMES)) - 1)
    g.ctx.profile_enable(True)
    t0 = time.perf_counter()
    if marks:
        marks[0].record(mark_stream)
    for i in range(args.steps):
        step += 1
        before_step(i)
        run_step(step)
        after_step(i)
        if marks:
            marks[i + 1].record(mark_stream)
    t_updates = None
    if snapshots:
        # the updates are done when the library's compute streams are; a drain to the host may still be running
        for b in range(min(streams, len(g.buckets))):
            torch.cuda.ExternalStream(g.ctx.bucket_stream(b)).synchronize()
        t_updates = time.perf_counter() - t0
    g.ctx.sync()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    g.ctx.profile_enable(False)

    ms_per_step = 1e3 * elapsed / args.steps
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps)) if marks else None
    kernels = {}
    for kind, name in KERNEL_NAMES.items():
        n, ms = g.ctx.profile_read(kind)
        if n:
            kernels[name] = {"launches": n, "avg_ms": ms / n, "ms_per_step": ms / args.steps, "from": "the timed iterations"}
    extra = 0
    if light:
        extra = min(3, args.steps)
        g.ctx.profile_kinds(((1 << len(KERNEL_NAMES)) - 1) & ~(1 << dom_kind))
        g.ctx.profile_enable(True)
        for _ in range(extra):
            step += 1
            run_step(step)
        g.ctx.sync()
        g.ctx.profile_enable(False)
        for kind, name in KERNEL_NAMES.items():
            n, ms = g.ctx.profile_read(kind)
            if n:
                kernels[name] = {"launches": n, "avg_ms": ms / n, "ms_per_step": ms / extra,
                                 "from": f"{extra} iterations behind the timed ones"}
    # dominant kernel = the one that moves the largest share of the step's algorithmic bytes (with clipping on,
    # the whole-arena AdamW sweep: 28 of 48 B/param, one launch per step, alone on its stream; per-bucket
    # kernels overlap across streams, which stretches their individual event durations)
    # algorithmic bytes of one launch: per-bucket kernels process P/B params on average
    launches_per_step = kernels[dom]["launches"] / args.steps
    bytes_per_launch = bpp[dom] * P / launches_per_step
    achieved = bytes_per_launch / (kernels[dom]["avg_ms"] * 1e-3) / 1e9
    total_gbs = bpp["total"] * P / (ms_per_step * 1e-3) / 1e9

    traffic = measured_traffic(wl.name, dom, bool(args.refold), bool(args.no_clip), default_settings and g.placement == "plan")
    traffic_source = None
    if traffic is not None:
        traffic_source = (f"stored, not measured in this run: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this command, "
                          f"profiles/{wl.name}{'_refold' if args.refold else ''}{'_noclip' if args.no_clip else ''}_bench_rocprofv3.md, "
                          f"taken at kernel sources (comments stripped) sha256 {MEASURED_TRAFFIC_SOURCES_SHA256[:16]}")
    out = {
        "metric": "shadow update params/sec and achieved HBM GB/s (% of peak) per iteration",
        "value": P / (ms_per_step * 1e-3),
        "unit": "params/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "untimed_steps_behind": extra,       # iterations run behind the timed region to time the other kernels
        "ms_per_step": ms_per_step,
        "ms_per_step_median": (per_step[len(per_step) // 2] if len(per_step) % 2 else
                               0.5 * (per_step[len(per_step) // 2 - 1] + per_step[len(per_step) // 2])) if per_step else None,
        "ms_per_step_min": per_step[0] if per_step else None,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: {P} fp32 params (+m, v) in {len(g.buckets)} buckets of <= "
                               f"{wl.bucket_cap_bytes >> 20} MiB, W={wl.num_workers} {wl.grad_dtype} gradient views per bucket, "
                               f"{args.optimizer}" + (f" + global-norm clip at {wl.max_grad_norm}" if wl.max_grad_norm > 0 else ""),
                   "num_params": P, "num_buckets": len(g.buckets), "num_workers": wl.num_workers,
                   "grad_dtype": wl.grad_dtype, "streams": streams,
                   "batch_bytes": batch_bytes, "refold": bool(args.refold), "optimizer": args.optimizer,
                   "ingest_slots": args.ingest_slots, "view_ring_bytes": ring_bytes, "placement": g.placement,
                   "offsets_gib": args.offsets_gib,
                   "snapshot_every": args.snapshot_every, "snapshot_mode": args.snapshot_mode if snapshots else None,
                   "snapshot_to_host": bool(snapshots and args.snapshot_host)},
        "hbm_GBps": total_gbs,
        "hbm_frac_of_peak": total_gbs / HBM_PEAK_GBS,
        "bytes_per_param": bpp["total"],
        "copy_kernel_GBps": yard,
        "hbm_frac_of_copy_kernel": (total_gbs / yard) if yard else None,
        "kernels": kernels,
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "bytes_per_launch": bytes_per_launch, "avg_launch_ms": kernels[dom]["avg_ms"]},
    }
    if snapshots:
        sc = kernels.get("snapshot_copies")
        nbytes = A * 4 * (len(snap_host) if snap_host else (2 if args.optimizer == "sgd" else 3))
        out["snapshots"] = {"taken": snap_taken, "skipped_while_draining": snap_skipped,
                            "host_arrays": len(snap_host) if snap_host else 0,
                            "copy_ms_each": sc["avg_ms"] if sc else None,
                            "copy_GBps": (nbytes / (sc["avg_ms"] * 1e-3) / 1e9) if sc and (args.snapshot_host or not staged) else None,
                            "ms_per_step_updates_only": 1e3 * t_updates / args.steps,
                            "extra_bytes_per_param_on_a_snapshot_step": 12 if staged else 24}
    g.close()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, inputs, optimizer=args.optimizer)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
