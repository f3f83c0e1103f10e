"""The named workloads at their full sizes, in the launch configuration bench.py times.

The GPU applies every bucket of every iteration.  The oracle cannot sweep 7e9 parameters for several
iterations in a test, so inputs are tiled (element e takes the tile's value at e mod L, L prime): the
oracle gets the exact global norm from one folded tile with multiplicities, hence the clip coefficient,
and then recomputes (a) whole sampled buckets and (b) scattered sampled elements one by one, for all
iterations, and those are compared bit for bit with the GPU's arenas.
"""
import gc
import sys
import time

import numpy as np
import pytest
import torch

import oracle
import synth
from harness import (BENCH_BATCH_BYTES, BENCH_STREAMS, GpuShadow, Inputs, TILE_PERIOD, assert_layouts_agree, assert_state_matches, lib_layout,
                     oracle_hparams, oracle_layout)

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(autouse=True)
def _free_gpu_memory():
    yield
    gc.collect()
    torch.cuda.empty_cache()


def pick_buckets(lay: oracle.Layout, budget: int):
    """Smallest bucket, a bucket whose tensors carry different decay flags, the last bucket, and the
    largest bucket that still fits the element budget."""
    sizes = [b.numel for b in lay.buckets]
    chosen = {int(np.argmin(sizes)), len(sizes) - 1}
    mixed = [i for i, b in enumerate(lay.buckets) if len({s.weight_decay for s in b.segments}) > 1]
    if mixed:
        chosen.add(min(mixed, key=lambda i: sizes[i]))
        chosen.add(mixed[len(mixed) // 2])
    out, used = [], 0
    for i in sorted(chosen, key=lambda i: sizes[i]):
        if used + sizes[i] <= budget or not out:
            out.append(i)
            used += sizes[i]
    fits = [i for i in range(len(sizes)) if i not in out and used + sizes[i] <= budget]
    if fits:
        out.append(max(fits, key=lambda i: sizes[i]))
    return sorted(out)


def run_fullsize(name: str, steps: int, bucket_budget: int, n_scatter: int, resident: bool, num_streams: int = 2,
                 batch_bytes: int = 0, refold: bool = False, also_sizes=(), staged_last: bool = False, wl=None, also_elements=None):
    """also_elements: {bucket: offsets inside it} joined to the scattered sample."""
    wl = wl or synth.get_workload(name)
    say(f"case fullsize {name}: P={wl.num_params} W={wl.num_workers} steps={steps}")
    t_start = time.time()
    L = TILE_PERIOD
    inp = Inputs(wl, period=L)
    lay = oracle_layout(wl)
    assert_layouts_agree(lay, lib_layout(wl))
    starts = lay.logical_starts()
    P = lay.num_params
    hp = oracle_hparams(wl)
    clip = wl.max_grad_norm > 0
    W = wl.num_workers

    g = GpuShadow(wl, inp, num_streams=num_streams, resident_grads=resident, batch_bytes=batch_bytes, refold=refold,
                  snapshot_set=staged_last)
    B = len(g.buckets)
    ring = None
    if not resident:
        nmax = max(n for _, n, _ in g.buckets)
        ring = [torch.empty(nmax, dtype=g.gdt, device=g.dev) for _ in range(W)]

    chosen = pick_buckets(lay, bucket_budget)
    for size in also_sizes:          # the first bucket of each of these sizes as well, whatever the budget
        chosen = sorted(set(chosen) | {next(i for i, b in enumerate(lay.buckets) if b.numel == size)})
    say(f"  buckets={B}, oracle recomputes buckets {chosen} ({sum(lay.buckets[b].numel for b in chosen)} elems) "
        f"and {n_scatter} scattered elements")
    # scattered sample: logical indices, their arena positions and decay flags
    rng = np.random.default_rng(wl.seed % (2 ** 32))
    sidx = rng.integers(0, P, n_scatter)
    for b, offsets in (also_elements or {}).items():
        sidx = np.concatenate([sidx, starts[b] + np.asarray(offsets, dtype=np.int64)])
    sidx = np.unique(sidx)
    bstart = np.array(starts + [P])
    sb = np.searchsorted(bstart, sidx, side="right") - 1
    arena_off = np.array([off for off, _, _ in g.buckets])
    s_arena = arena_off[sb] + (sidx - bstart[sb])
    seg_start, seg_flag = [], []
    for b, bk in enumerate(lay.buckets):
        for s in bk.segments:
            seg_start.append(starts[b] + s.offset)
            seg_flag.append(s.weight_decay)
    order = np.argsort(seg_start)
    seg_start, seg_flag = np.array(seg_start)[order], np.array(seg_flag)[order]
    s_flag = seg_flag[np.searchsorted(seg_start, sidx, side="right") - 1]
    sidx_t = torch.from_numpy(sidx)
    s_arena_t = torch.from_numpy(s_arena).to(g.dev)
    sp = inp.param_at(sidx_t).numpy().copy()
    sm, sv = np.zeros_like(sp), np.zeros_like(sp)

    params = [inp.param_np(starts[b], lay.buckets[b].numel) if b in chosen else None for b in range(B)]
    orc = oracle.OracleShadow(lay, hp, params)
    cnt = np.full(L, P // L, np.uint64)
    cnt[: P % L] += 1
    tile_idx = torch.arange(L, dtype=torch.int64)

    def to_np(t):
        a = t.numpy()
        return a.view(np.uint16).copy() if wl.grad_dtype == "bf16" else a.copy()

    for t in range(1, steps + 1):
        # ---- GPU: every bucket ----
        order_t = synth.arrival_order(wl.seed, t, B) if wl.random_arrival else list(range(B))
        if resident:
            g.fill_grads(t)
            if staged_last and t == steps:
                for off, n, _ in g.buckets:        # whatever the staging set held, the armed iteration must overwrite it
                    g.snap[0][off:off + n].fill_(7.0)
                g.ctx.snapshot_arm(None, None, None)
            g.apply_step(t, order_t)
        else:
            for b in order_t:
                off, n, _ = g.buckets[b]
                for w in range(W):
                    inp.fill_grad_dev(ring[w][:n], t, w, g.logical_start[b])
                torch.cuda.synchronize()
                g.ctx.apply_bucket(b, [r.data_ptr() for r in ring], t)
                g.ctx.sync()
        g.ctx.sync()
        # ---- oracle: norm from the tile, then the sampled parts ----
        c = None
        if clip:
            r_tile = oracle.fold([to_np(inp.grad_at(t, w, tile_idx)) for w in range(W)], hp.mean)
            S = oracle.SumSq().add(r_tile, cnt)
            c = S.coef(hp.max_grad_norm)
            gc_, gS = g.ctx.clip_state()
            assert np.float32(gc_) == c, f"{name} step {t}: clip coefficient {gc_} vs oracle {c}"
            assert abs(gS - S.value) <= 1e-12 * S.value
        for b in chosen:
            n = lay.buckets[b].numel
            r = oracle.fold([inp.grad_np(t, w, starts[b], n) for w in range(W)], hp.mean)
            orc.update_bucket(b, r, t, c)
        rs = oracle.fold([to_np(inp.grad_at(t, w, sidx_t)) for w in range(W)], hp.mean)
        for flag in (False, True):
            sel = np.flatnonzero(s_flag == flag)
            if sel.size:
                pp, mm, vv = sp[sel].copy(), sm[sel].copy(), sv[sel].copy()
                oracle.adamw_f32(pp, mm, vv, rs[sel].copy(), flag, hp, t, c)
                sp[sel], sm[sel], sv[sel] = pp, mm, vv
        # ---- compare ----
        if t == steps or t == 1:
            for b in chosen:
                assert_state_matches(g.bucket_state(b), (orc.p[b], orc.m[b], orc.v[b]), f"{name} step {t} bucket {b}")
            got = tuple(x[s_arena_t].cpu().numpy() for x in (g.p, g.m, g.v))
            assert_state_matches(got, (sp, sm, sv), f"{name} step {t} scattered sample")
            if staged_last and t == steps:
                # the staging set of the armed (last) iteration: same bits as the oracle where it was recomputed,
                # and equal to the replica everywhere
                assert g.ctx.snapshot_wait() == steps
                for b in chosen:
                    off, n, _ = g.buckets[b]
                    assert_state_matches(tuple(x[off:off + n].cpu().numpy() for x in g.snap), (orc.p[b], orc.m[b], orc.v[b]),
                                         f"{name} step {t} bucket {b} of the staging set")
                assert_state_matches(tuple(x[s_arena_t].cpu().numpy() for x in g.snap), (sp, sm, sv),
                                     f"{name} step {t} scattered sample of the staging set")
                for mine, theirs in zip(g.snap, (g.p, g.m, g.v)):
                    assert torch.equal(mine.view(torch.int32), theirs.view(torch.int32))
        say(f"  step {t} ok" + (f" (c={float(c):.6g})" if clip else "") + f"  [{time.time() - t_start:.0f} s]")
    assert g.ctx.step() == (steps, 0)
    # alignment gaps stay zero
    for (off, n, _), nxt in zip(g.buckets[:-1], g.buckets[1:]):
        if nxt[0] > off + n:
            assert float(g.p[off + n:nxt[0]].abs().max()) == 0.0 and float(g.v[off + n:nxt[0]].abs().max()) == 0.0
    g.close()
    del g, ring


@pytest.mark.parametrize("bench_config", [False, True])
def test_gpt2_small_full(bench_config):
    """Once with a launch per bucket on two streams, once as bench.py launches it (one stream, buckets batched)."""
    kw = dict(num_streams=BENCH_STREAMS, batch_bytes=BENCH_BATCH_BYTES) if bench_config else {}
    run_fullsize("gpt2s", steps=20, bucket_budget=45_000_000, n_scatter=2_000_000, resident=True, **kw)


def test_gpt_1p3b_full():
    """bench.py's launch configuration.  The last iteration is armed for a staged snapshot: its update kernels write a
    second set of arenas as well."""
    run_fullsize("gpt1p3b", steps=10, bucket_budget=30_000_000, n_scatter=5_000_000, resident=True, staged_last=True,
                 num_streams=BENCH_STREAMS, batch_bytes=BENCH_BATCH_BYTES)


def test_llama7b_full():
    """Same launch configuration as bench.py: one stream, the iteration's buckets folded in as few launches as possible.
    The oracle recomputes, besides the small buckets, a whole 131,072,000-element bucket (embedding / head size), a whole
    45,088,768-element one (feed-forward matrix) and five million scattered elements."""
    run_fullsize("llama7b", steps=5, bucket_budget=60_000_000, n_scatter=5_000_000, resident=True, num_streams=BENCH_STREAMS,
                 batch_bytes=BENCH_BATCH_BYTES, also_sizes=(131_072_000, 45_088_768))


def test_llama7b_full_one_launch_per_bucket():
    run_fullsize("llama7b", steps=2, bucket_budget=60_000_000, n_scatter=5_000_000, resident=True, num_streams=2, batch_bytes=0)


def test_llama7b_single_reduced_gradient_full():
    """W = 1 (the shadow is handed the already-reduced gradient, as in the paper), clipping without a scratch arena."""
    run_fullsize("llama7b_w1", steps=3, bucket_budget=60_000_000, n_scatter=5_000_000, resident=True, num_streams=BENCH_STREAMS,
                 batch_bytes=BENCH_BATCH_BYTES, refold=True, also_sizes=(131_072_000,))


def test_ragged7b_full():
    run_fullsize("ragged7b", steps=3, bucket_budget=30_000_000, n_scatter=5_000_000, resident=False, num_streams=4)


@pytest.mark.parametrize("W,dtype,clip,refold", [(1, "bf16", 1.0, False), (1, "bf16", 1.0, True), (2, "f32", 0.0, False)])
def test_bucket_beyond_two_to_the_32_elements(W, dtype, clip, refold):
    """One tensor of 2^32 + 2^20 + 3 elements in a bucket of its own, between two small buckets: element indices, vector
    indices times 16 and byte offsets inside one bucket all pass 2^32, and the bucket ends in a ragged tail.  The oracle
    recomputes the small buckets and a scattered sample that includes the elements around 2^32 and the last ones."""
    n = (1 << 32) + (1 << 20) + 3
    ts = [synth.TensorSpec("head", 1000, True), synth.TensorSpec("giant", n, True), synth.TensorSpec("tail", 5000, False)]
    wl = synth.Workload("giant", ts, num_workers=W, grad_dtype=dtype, grad_dist="normal", grad_sigma=1e-3, steps=2, max_grad_norm=clip,
                        bucket_cap_bytes=1 << 20, weight_decay=0.01)
    near = [0, 1, 2, 3, 4, (1 << 31) - 1, 1 << 31, (1 << 32) - 5, (1 << 32) - 1, 1 << 32, (1 << 32) + 1, (1 << 32) + 4, n - 8, n - 4, n - 3, n - 2, n - 1]
    run_fullsize("giant", steps=2, bucket_budget=1_000_000, n_scatter=3_000_000, resident=True, num_streams=BENCH_STREAMS,
                 batch_bytes=BENCH_BATCH_BYTES, refold=refold, wl=wl, also_elements={1: near})

