"""Randomized schedules against the oracle: workload shape, worker count, dtype, optimizer, clip mode, streams, launch
batching, arrival order, producer events, release events and snapshots of both kinds are drawn from a seed; the
replica after every iteration and every snapshot taken must equal the oracle's state of that iteration bit for bit."""
import sys

import numpy as np
import pytest
import torch

import paper_2507_13522_amd as sh
from paper_2507_13522_amd import binding
import synth
from harness import GpuShadow, Inputs, assert_state_matches, run_oracle_full

pytestmark = pytest.mark.gpu


def draw_case(seed: int):
    rng = np.random.default_rng(1000 + seed)
    T = int(rng.integers(3, 40))
    sizes = [(int(np.exp(rng.uniform(0, np.log(300_000)))), bool(rng.integers(0, 2))) for _ in range(T)]
    W = int(rng.choice([1, 2, 3, 4, 6, 8, 9, 16, 24]))
    dtype = str(rng.choice(["bf16", "f32"]))
    optimizer = str(rng.choice(["adamw", "adamw", "adam", "sgd"]))
    clip = float(rng.choice([0.0, 0.003, 1e6]))
    refold = bool(clip > 0 and rng.integers(0, 3) == 0)
    cap = int(rng.choice([20_000, 200_000, 2_000_000]))
    ts = [synth.TensorSpec(f"t{i}", n, f) for i, (n, f) in enumerate(sizes)]
    wl = synth.Workload(f"random{seed}", ts, num_workers=W, grad_dtype=dtype, grad_dist=str(rng.choice(["normal", "t3"])),
                        grad_sigma=1e-3, steps=5, max_grad_norm=clip, bucket_cap_bytes=cap, weight_decay=0.05,
                        lr=0.05 if optimizer == "sgd" else 1e-3, seed=77 + seed)
    cfg = dict(streams=int(rng.integers(1, 5)), batch_bytes=int(rng.choice([0, 50_000, 1 << 62])), refold=refold, optimizer=optimizer,
               staged=bool(rng.integers(0, 2)),
               launch=sh.LaunchShape(fold_block=int(rng.choice([0, 64, 256])), fused_block=int(rng.choice([0, 128, 512])),
                                     sweep_block=int(rng.choice([0, 64, 1024])), fused_waves_per_cu=int(rng.choice([0, 8, 20])),
                                     max_launch_threads=int(rng.choice([0, 0, 3000])), drain_blocks=int(rng.choice([0, 1, 7]))))
    return wl, cfg, rng


@pytest.mark.parametrize("seed", range(24))
def test_random_schedule(seed):
    wl, cfg, rng = draw_case(seed)
    print("case random schedule", seed, len(wl.tensors), "tensors W", wl.num_workers, wl.grad_dtype, "clip", wl.max_grad_norm, cfg["optimizer"],
          {k: v for k, v in cfg.items() if k != "launch"}, flush=True)
    sys.stdout.flush()
    steps = 5
    inp = Inputs(wl)
    sgd = cfg["optimizer"] == "sgd"
    states = {}
    run_oracle_full(wl, inp, steps, optimizer=cfg["optimizer"],
                    on_step=lambda t, o: states.__setitem__(t, [[x.copy() for x in o.p], [x.copy() for x in o.m], [x.copy() for x in o.v]]))
    g = GpuShadow(wl, inp, num_streams=cfg["streams"], batch_bytes=cfg["batch_bytes"], refold=cfg["refold"], optimizer=cfg["optimizer"],
                  snapshot_set=cfg["staged"], launch=cfg["launch"])
    A, B = g.layout.arena_numel, len(g.buckets)
    views = {}
    for t in range(1, steps + 1):
        g.fill_grads(t)
        views[t] = g._stage.clone()
    torch.cuda.synchronize()
    producer = torch.cuda.Stream()
    snaps = []        # (step, arrays, kind)
    armed_for = None

    def check(arrays, t, what):
        ref = states[t]
        for b, (off, n, _) in enumerate(g.buckets):
            got = tuple(np.asarray(a[off:off + n].cpu()) for a in arrays[:2]) + \
                  ((ref[2][b],) if sgd else (np.asarray(arrays[2][off:off + n].cpu()),))
            assert_state_matches(got, (ref[0][b], ref[1][b], ref[2][b]), f"seed {seed} {what} of iteration {t}, bucket {b}")

    for t in range(1, steps + 1):
        # release side: the previous iteration's readers of the views, then the producer overwrites them
        with torch.cuda.stream(producer):
            if t > 1:
                for s in range(min(cfg["streams"], B)):
                    rel = torch.cuda.Event()
                    rel.record(producer)
                    g.ctx.record_consumed(s, rel.cuda_event)
                    producer.wait_event(rel)
            g._stage.copy_(views[t], non_blocking=True)
            ready = torch.cuda.Event()
            ready.record(producer)
        if cfg["staged"] and armed_for is None and rng.integers(0, 2):
            host = [torch.full((A,), 3.0, dtype=torch.float32, pin_memory=True) for _ in range(3)] if rng.integers(0, 2) else None
            rc = g.ctx.try_snapshot_arm(*(([h.data_ptr() for h in host[:2]] + [None if sgd else host[2].data_ptr()]) if host else [None] * 3))
            if rc == binding.OK:
                armed_for = (t, host)
            else:
                assert rc == binding.EBUSY          # the previous drain still runs
        order = [int(x) for x in rng.permutation(B)]
        for b in order:
            g.ctx.apply_bucket(b, g._views[b], t, ready_event=ready.cuda_event)
        if armed_for is not None and armed_for[0] == t:
            if armed_for[1] is not None:
                snaps.append((t, armed_for[1], "staged to host"))
            else:
                g.ctx.snapshot_wait()                # device only: read the staging set before it can be armed again
                check(g.snap, t, "staging set")
            armed_for = None
        if rng.integers(0, 3) == 0:                  # a plain snapshot right behind the iteration
            where = int(rng.integers(0, 2))
            dst = [torch.empty(A, dtype=torch.float32, pin_memory=True) if where else torch.empty(A, dtype=torch.float32, device="cuda:0")
                   for _ in range(3)]
            assert g.ctx.snapshot(dst[0].data_ptr(), dst[1].data_ptr(), None if sgd else dst[2].data_ptr()) == t
            snaps.append((t, dst, "copy to " + ("host" if where else "device")))
        if rng.integers(0, 2):                       # sometimes look at the replica itself between iterations
            g.ctx.sync()
            check((g.p, g.m, g.v), t, "replica")
    g.ctx.sync()
    assert g.ctx.step() == (steps, 0)
    check((g.p, g.m, g.v), steps, "replica")
    for t, arrays, kind in snaps:
        check(arrays, t, kind)
    g.close()
