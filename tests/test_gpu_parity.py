"""HIP path vs CPU oracle, element by element, through the C ABI (needs an MI355X)."""
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2507_13522_amd as sh
from paper_2507_13522_amd import binding
import synth
from harness import (GpuShadow, Inputs, assert_layouts_agree, assert_state_matches, diff, lib_layout, oracle_hparams,
                     oracle_layout, run_oracle_full, REL_TOL)

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def custom(name, sizes_flags, W, dtype, clip=0.0, cap=1 << 16, steps=3, dist="normal", sigma=1e-3, wd=0.01, explicit=None,
           random_arrival=False, lr=1e-3):
    ts = [synth.TensorSpec(f"t{i}", n, f) for i, (n, f) in enumerate(sizes_flags)]
    return synth.Workload(name, ts, num_workers=W, grad_dtype=dtype, grad_dist=dist, grad_sigma=sigma, steps=steps,
                          max_grad_norm=clip, bucket_cap_bytes=cap, explicit_buckets=explicit, weight_decay=wd,
                          random_arrival=random_arrival, lr=lr)


def check_against_oracle(wl, steps=None, num_streams=2, mean=True, every_step=True, exact=True, torch_streams=False,
                         batch_bytes=0, refold=False, optimizer="adamw", launch=None):
    """Run both sides on the same inputs and compare param, m, v of every bucket."""
    steps = steps or wl.steps
    inp = Inputs(wl)
    assert_layouts_agree(oracle_layout(wl), lib_layout(wl))
    g = GpuShadow(wl, inp, num_streams=num_streams, mean=mean, torch_streams=torch_streams, batch_bytes=batch_bytes,
                  refold=refold, optimizer=optimizer, launch=launch)
    assert g.ctx.num_buckets() == len(g.buckets) and all(g.ctx.bucket_info(b) == g.buckets[b][:2] for b in range(len(g.buckets)))
    worst = {}

    def on_step(t, orc):
        order = synth.arrival_order(wl.seed, t, len(g.buckets)) if wl.random_arrival else None
        g.run_step(t, order)
        if every_step or t == steps:
            for b in range(len(g.buckets)):
                ds = assert_state_matches(g.bucket_state(b), (orc.p[b], orc.m[b], orc.v[b]), f"{wl.name} step {t} bucket {b}", exact)
                for k, d in zip("pmv", ds):
                    worst[k] = max(worst.get(k, 0.0), d.max_rel)
            if wl.max_grad_norm > 0:
                c, S = g.ctx.clip_state()
                assert np.float32(c) == orc.last_coef, (c, orc.last_coef)
                assert abs(S - orc.last_sumsq) <= 1e-12 * orc.last_sumsq

    run_oracle_full(wl, inp, steps, mean=mean, on_step=on_step, optimizer=optimizer)
    assert g.ctx.step() == (steps, 0)
    g.close()
    return worst


def test_tiny_config_every_step():
    """Config 'tiny': 1,048,576 params in 4 buckets, W=4 fp32 gradients, 10 steps, no clipping."""
    say("case tiny")
    wl = synth.get_workload("tiny")
    worst = check_against_oracle(wl)
    say("tiny worst rel", worst)


RAGGED = [(5000, True), (33, False), (70001, True), (1, False), (64, True), (12345, False), (300007, True), (999, True),
          (2048, False), (77777, True), (7, True), (3, False), (5, True), (1024, True), (8, False)]


@pytest.mark.parametrize("batch_bytes", [0, 1 << 20, 1 << 62])
@pytest.mark.parametrize("W,dtype", [(3, "bf16"), (8, "bf16"), (5, "f32")])
def test_ragged_clip_random_arrival(W, dtype, batch_bytes):
    """Several tiles, ragged tails, flags changing inside a vector, clipping active, shuffled bucket arrival;
    every bucket its own launch, a few buckets per launch, and the whole iteration in as few launches as possible."""
    say("case ragged", W, dtype, batch_bytes)
    wl = custom("ragged", RAGGED, W, dtype, clip=0.01, cap=200_000, steps=5, random_arrival=True)
    check_against_oracle(wl, num_streams=3, batch_bytes=batch_bytes)


@pytest.mark.parametrize("W,dtype,clip", [(64, "bf16", 0.0), (64, "f32", 0.01), (16, "bf16", 0.01), (2, "bf16", 0.0)])
def test_many_small_buckets_batched(W, dtype, clip):
    """More buckets than one launch descriptor holds (32 buckets / 320 pointers): batches split correctly."""
    say("case many buckets", W, dtype, clip)
    rng = np.random.default_rng(W)
    sizes = [(int(n), bool(f)) for n, f in zip(rng.integers(1, 3000, 150), rng.integers(0, 2, 150))]
    wl = custom("many", sizes, W, dtype, clip=clip, cap=4000, steps=2, random_arrival=True)
    for streams, bb in ((1, 1 << 62), (3, 1 << 62), (2, 100_000)):
        check_against_oracle(wl, num_streams=streams, batch_bytes=bb)


# 3, 6, 7: only the remainder of the worker loop; 9, 15, 17: whole chunks of 8 and a remainder; 24, 40: whole chunks only
@pytest.mark.parametrize("W", [1, 2, 3, 4, 6, 7, 8, 9, 15, 16, 17, 24, 32, 40, 64])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("clip", [0.0, 0.005])
def test_worker_counts(W, dtype, clip):
    say("case W", W, dtype, clip)
    wl = custom("wsweep", [(20011, True), (4099, False), (9000, True), (17, False)], W, dtype, clip=clip, cap=30_000, steps=2)
    check_against_oracle(wl, num_streams=2)


@pytest.mark.parametrize("W,dtype", [(1, "bf16"), (2, "bf16"), (4, "bf16"), (1, "f32"), (3, "bf16"), (8, "bf16"), (64, "f32")])
@pytest.mark.parametrize("batch_bytes", [0, 1 << 62])
def test_clip_without_scratch_folds_twice(W, dtype, batch_bytes):
    """Clipping with no scratch arena (W = 1 is the paper's case of one already-reduced gradient): the views are
    folded once for the norm and once more for the update; same bits as the oracle and as the stored path."""
    say("case refold", W, dtype, batch_bytes)
    wl = custom("refold", RAGGED, W, dtype, clip=0.01, cap=200_000, steps=4, random_arrival=True)
    check_against_oracle(wl, num_streams=2, batch_bytes=batch_bytes, refold=True)
    many = custom("refold-many", [(int(n), bool(n % 3)) for n in np.random.default_rng(W).integers(1, 2000, 90)], W, dtype,
                  clip=0.003, cap=3000, steps=2)
    check_against_oracle(many, num_streams=3, batch_bytes=batch_bytes, refold=True)


@pytest.mark.parametrize("optimizer", ["adam", "sgd"])
@pytest.mark.parametrize("W,dtype,clip,refold", [(8, "bf16", 0.0, False), (8, "bf16", 0.01, False), (1, "bf16", 0.01, True),
                                                 (5, "f32", 0.01, False), (4, "f32", 0.0, False)])
def test_other_functional_optimizers(optimizer, W, dtype, clip, refold):
    """Adam (L2 penalty in the gradient) and momentum SGD (section 4.2.4) against the oracle, bit for bit."""
    say("case optimizer", optimizer, W, dtype, clip, refold)
    wl = custom("opt-" + optimizer, RAGGED, W, dtype, clip=clip, cap=200_000, steps=5, random_arrival=True, wd=0.1,
                lr=1e-3 if optimizer == "adam" else 0.05)
    check_against_oracle(wl, num_streams=2, batch_bytes=1 << 20, refold=refold, optimizer=optimizer)


def test_sum_reduce_and_student_t():
    say("case sum/t3")
    wl = custom("sum", RAGGED[:8], 4, "bf16", clip=0.05, cap=150_000, steps=3, dist="t3")
    check_against_oracle(wl, mean=False)
    check_against_oracle(wl, mean=True)


def test_degenerate_buckets():
    """Buckets smaller than one vector, a one-element model, sizes that are exact multiples of the tile."""
    say("case degenerate")
    for sizes in ([(1, True)], [(7, False)], [(8, True)], [(3, True), (2, False), (1, True)], [(1024, True), (1024, False)],
                  [(2048, True)], [(2049, True)], [(65536, False), (5, True)]):
        for clip in (0.0, 1e-4):
            wl = custom("degenerate", sizes, 2, "bf16", clip=clip, cap=2048, steps=2)
            check_against_oracle(wl, num_streams=1)


def test_borrowed_torch_streams():
    say("case torch streams")
    wl = custom("tstreams", RAGGED, 4, "bf16", clip=0.01, cap=200_000, steps=3)
    check_against_oracle(wl, num_streams=4, torch_streams=True)


def test_clip_inactive_equals_no_clip():
    """With the norm below the threshold c == 1 and the two-pass path gives the bits of the fused path."""
    say("case clip inactive")
    sizes = RAGGED[:9]
    a = custom("noclip", sizes, 4, "bf16", clip=0.0, cap=150_000, steps=3)
    b = custom("clip", sizes, 4, "bf16", clip=1e6, cap=150_000, steps=3)
    ga, gb = GpuShadow(a, Inputs(a)), GpuShadow(b, Inputs(b))
    for t in range(1, 4):
        ga.run_step(t)
        gb.run_step(t)
        assert gb.ctx.clip_state()[0] == 1.0
    assert torch.equal(ga.p, gb.p) and torch.equal(ga.m, gb.m) and torch.equal(ga.v, gb.v)
    ga.close(); gb.close()


def test_ieee_divide_sqrt_denormals_bruteforce():
    """One AdamW step on 2^22 elements whose p, m, v, g span the whole float range (denormals,
    huge and tiny magnitudes): divide, sqrt and every multiply/add must round as on the host."""
    say("case ieee bruteforce")
    n = 1 << 22
    rng = np.random.default_rng(99)

    def wide(signed=True, emin=-149, emax=60):
        e = rng.uniform(emin, emax, n)
        x = np.exp2(e) * rng.uniform(1.0, 2.0, n)
        if signed:
            x = x * rng.choice([-1.0, 1.0], n)
        return x.astype(np.float32)

    p0, m0, v0, g0 = wide(), wide(), wide(signed=False, emin=-149, emax=40), wide(emin=-140, emax=15)
    v0[:1000] = 0.0
    g0[500:1500] = 0.0
    m0[2000:3000] = 0.0
    wl = custom("ieee", [(n // 2, True), (n // 2, False)], 1, "f32", clip=0.0, cap=1 << 30, steps=1)
    hp = oracle.HParams(lr=wl.lr, beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps, weight_decay=wl.weight_decay)
    for t in (1, 7, 1000):
        lay = lib_layout(wl)
        assert lay.num_buckets == 1 and lay.arena_numel == n
        dev = torch.device("cuda:0")
        p, m, v = (torch.from_numpy(x.copy()).to(dev) for x in (p0, m0, v0))
        gdev = torch.from_numpy(g0.copy()).to(dev)
        torch.cuda.synchronize()
        ctx = sh.Shadow(lay, sh.HParams(lr=wl.lr, beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps, weight_decay=wl.weight_decay,
                                        max_grad_norm=0.0, num_workers=1, grad_dtype=sh.GRAD_F32, reduce_op=sh.REDUCE_MEAN,
                                        num_streams=1), p.data_ptr(), m.data_ptr(), v.data_ptr(), None, t - 1)
        ctx.apply_bucket(0, [gdev.data_ptr()], t)
        ctx.sync()
        rp, rm, rv = p0.copy(), m0.copy(), v0.copy()
        # bucket order is last tensor first: the masked half comes first
        h = n // 2
        oracle.adamw_f32(rp[:h], rm[:h], rv[:h], g0[:h], False, hp, t)
        oracle.adamw_f32(rp[h:], rm[h:], rv[h:], g0[h:], True, hp, t)
        for name, got, ref in (("p", p, rp), ("m", m, rm), ("v", v, rv)):
            got = got.cpu().numpy()
            same = (got.view(np.uint32) == ref.view(np.uint32)) | (np.isnan(got) & np.isnan(ref))
            assert same.all(), f"t={t} {name}: {np.count_nonzero(~same)} elements differ, first {np.flatnonzero(~same)[:5]}"
        ctx.destroy()


def _same_bits_or_nan(a, b):
    return bool(np.all((a.view(np.uint32) == b.view(np.uint32)) | (np.isnan(a) & np.isnan(b))))


@pytest.mark.parametrize("clip", [0.0, 0.01])
def test_non_finite_gradients_propagate(clip):
    """No special handling of Inf/NaN gradients: they propagate exactly as in the oracle (without clipping only the
    poisoned elements change; with clipping an infinite norm gives c = 0 and 0*Inf = NaN in the poisoned element)."""
    say("case non-finite", clip)
    wl = custom("nonfinite", [(5000, True), (777, False), (4099, True)], 2, "f32", clip=clip, cap=20_000, steps=2)
    inp = Inputs(wl)
    g = GpuShadow(wl, inp, num_streams=2)
    lay = oracle_layout(wl)
    starts = lay.logical_starts()
    orc = oracle.OracleShadow(lay, oracle.HParams(lr=wl.lr, weight_decay=wl.weight_decay, max_grad_norm=clip),
                              [inp.param_np(s, b.numel) for s, b in zip(starts, lay.buckets)])
    poison = {(0, 0, 17): np.inf, (1, 1, 5): -np.inf, (0, 1, 4000): np.nan}      # (bucket, worker, element) -> value
    for t in (1, 2):
        g.fill_grads(t)
        grads = {b: [inp.grad_np(t, w, starts[b], lay.buckets[b].numel) for w in range(2)] for b in range(len(lay.buckets))}
        if t == 1:
            for (b, w, e), val in poison.items():
                if b < len(lay.buckets) and e < lay.buckets[b].numel:
                    grads[b][w][e] = val
                    g.view(b, w)[e] = float(val)
        torch.cuda.synchronize()
        g.apply_step(t)
        g.ctx.sync()
        orc.step(grads)
    n_bad = 0
    for b in range(len(lay.buckets)):
        got = g.bucket_state(b)
        for x, y in zip(got, (orc.p[b], orc.m[b], orc.v[b])):
            assert _same_bits_or_nan(x, y)
            n_bad += int(np.count_nonzero(~np.isfinite(x)))
    assert n_bad > 0
    if clip == 0.0:
        assert n_bad <= 3 * len(poison) * 1        # only the poisoned elements (p, m, v each)
    # the alignment gaps between buckets hold no parameter: they stay zero even though the coefficient is not finite
    n_gap = 0
    for (off, n, _), nxt in zip(g.buckets, g.buckets[1:] + [(g.layout.arena_numel, 0, 0)]):
        for x in (g.p, g.m, g.v) + ((g.r,) if g.r is not None else ()):
            gap = x[off + n:nxt[0]]
            n_gap += gap.numel()
            assert gap.numel() == 0 or (float(gap.abs().max()) == 0.0 and bool(torch.isfinite(gap).all()))
    assert n_gap > 0
    g.close()


@pytest.mark.parametrize("slots,streams,clip", [(1, 1, 0.01), (2, 2, 0.01), (5, 3, 0.0)])
def test_ingest_from_pinned_host(slots, streams, clip):
    """Buckets handed over as HOST views go through the device ring (copy overlapping the folds of earlier buckets);
    results equal the oracle's, also when host and device deliveries are mixed within an iteration."""
    say("case ingest", slots, streams, clip)
    W = 4
    wl = custom("ingest", RAGGED, W, "bf16", clip=clip, cap=150_000, steps=4, random_arrival=True)
    inp = Inputs(wl)
    g = GpuShadow(wl, inp, num_streams=streams)
    B = len(g.buckets)
    nmax = max(n for _, n, _ in g.buckets)
    slot_bytes = W * ((nmax * 2 + 255) // 256 * 256)
    ring = torch.empty(slots * slot_bytes, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(sh.ShadowError):
        g.ctx.ingest_bucket(0, [1, 2, 3, 4], 1)                      # no ring attached yet
    with pytest.raises(sh.ShadowError):
        g.ctx.ingest_attach(ring.data_ptr(), slot_bytes - 256)       # smaller than one bucket's views
    g.ctx.ingest_attach(ring.data_ptr(), ring.numel())
    with pytest.raises(sh.ShadowError):
        g.ctx.ingest_attach(ring.data_ptr(), ring.numel())           # only once
    lay = oracle_layout(wl)
    starts = lay.logical_starts()
    orc = oracle.OracleShadow(lay, oracle.HParams(lr=wl.lr, weight_decay=wl.weight_decay, max_grad_norm=clip),
                              [inp.param_np(s, b.numel) for s, b in zip(starts, lay.buckets)])
    for t in range(1, 5):
        host = {b: [torch.from_numpy(inp.grad_np(t, w, starts[b], lay.buckets[b].numel).view(np.int16)).pin_memory()
                    for w in range(W)] for b in range(B)}
        g.fill_grads(t)
        for b in synth.arrival_order(wl.seed, t, B):
            if (b + t) % 3 == 0:
                g.ctx.apply_bucket(b, g._views[b], t)                # device views
            else:
                ready = torch.cuda.Event()
                ready.record()              # stands for a device-side producer of the host views
                g.ctx.ingest_bucket(b, [h.data_ptr() for h in host[b]], t, ready_event=ready.cuda_event if b % 2 else None)
        assert g.ctx.try_apply_bucket(0, g._views[0], t) == binding.ESTEP   # iteration t is complete
        g.ctx.sync()
        orc.step({b: [h.numpy().view(np.uint16) for h in host[b]] for b in range(B)})
        for b in range(B):
            assert_state_matches(g.bucket_state(b), (orc.p[b], orc.m[b], orc.v[b]), f"ingest step {t} bucket {b}")
    g.close()
    # a replica that folds twice (no scratch arena) cannot use the ring: the views would have to outlive their slots
    wl2 = custom("ingest-refold", RAGGED[:5], 1, "bf16", clip=0.01, cap=150_000, steps=1)
    g2 = GpuShadow(wl2, Inputs(wl2), refold=True)
    with pytest.raises(sh.ShadowError):
        g2.ctx.ingest_attach(ring.data_ptr(), ring.numel())
    g2.close()


def test_sixteen_streams():
    say("case 16 streams")
    wl = custom("s16", RAGGED, 4, "bf16", clip=0.01, cap=60_000, steps=3, random_arrival=True)
    check_against_oracle(wl, num_streams=16, batch_bytes=200_000)


def test_order_partition_and_stream_invariance():
    """Functional optimizer (section 4.2.4): the result does not depend on bucket arrival order,
    on how tensors are split into buckets, or on how many streams carry the buckets."""
    say("case invariance")
    sizes = RAGGED
    T = len(sizes)
    results = []
    for label, cap, explicit, streams, shuffle in [("base", 200_000, None, 1, False), ("shuffled", 200_000, None, 4, True),
                                                   ("one bucket", 1 << 30, None, 2, False),
                                                   ("bucket per tensor", 0, list(range(T - 1, -1, -1)), 3, True)]:
        wl = custom("inv", sizes, 4, "bf16", clip=0.0, cap=cap, steps=3, explicit=explicit)
        g = GpuShadow(wl, Inputs(wl), num_streams=streams)
        # note: logical element order differs between partitions, so inputs are addressed per TENSOR here
        per_tensor = {}
        for t in range(T):
            b, ob, oa = g.layout.tensor(t)
            per_tensor[t] = (b, ob, oa)
        base = np.cumsum([0] + [n for n, _ in sizes])
        inp = Inputs(wl)
        for t in range(T):
            b, ob, oa = per_tensor[t]
            n = sizes[t][0]
            g.p[oa:oa + n].copy_(inp.param_at(torch.arange(base[t], base[t] + n)))
        torch.cuda.synchronize()
        for step in range(1, 4):
            for t in range(T):
                b, ob, oa = per_tensor[t]
                n = sizes[t][0]
                for w in range(4):
                    g.view(b, w)[ob:ob + n].copy_(inp.grad_at(step, w, torch.arange(base[t], base[t] + n)))
            torch.cuda.synchronize()
            order = synth.arrival_order(5, step, len(g.buckets)) if shuffle else None
            g.apply_step(step, order)
            g.ctx.sync()
        out = []
        for t in range(T):
            oa, n = per_tensor[t][2], sizes[t][0]
            out.append(tuple(x[oa:oa + n].cpu().numpy().copy() for x in (g.p, g.m, g.v)))
        results.append((label, out))
        g.close()
    for label, out in results[1:]:
        for t in range(T):
            for k in range(3):
                assert np.array_equal(out[t][k].view(np.uint32), results[0][1][t][k].view(np.uint32)), (label, t, "pmv"[k])


def test_clip_arrival_order_invariance():
    say("case clip order invariance")
    wl = custom("inv-clip", RAGGED, 8, "bf16", clip=0.01, cap=100_000, steps=3)
    outs = []
    for shuffle, streams, bb in [(False, 1, 0), (True, 4, 0), (True, 2, 1 << 62), (False, 3, 300_000)]:
        g = GpuShadow(wl, Inputs(wl), num_streams=streams, batch_bytes=bb)
        for step in range(1, 4):
            g.run_step(step, synth.arrival_order(11 + streams, step, len(g.buckets)) if shuffle else None)
        outs.append((g.p.clone(), g.m.clone(), g.v.clone(), g.ctx.clip_state()))
        g.close()
    for o in outs[1:]:
        assert o[3] == outs[0][3]
        assert all(torch.equal(a, b) for a, b in zip(o[:3], outs[0][:3]))


@pytest.mark.parametrize("clip,streams,batch_bytes", [(0.01, 2, 0), (0.0, 3, 300_000)])
def test_snapshot_restore_every_second_step(clip, streams, batch_bytes):
    """Section 6.5 protocol: a run that is interrupted and restored from the shadow's state every second
    iteration equals the uninterrupted run -- here: the ORACLE run straight through, and the oracle restarted
    from the same snapshots (start_step carries the bias-correction count)."""
    say("case snapshot/restore", clip, streams, batch_bytes)
    wl = custom("restore", RAGGED, 4, "bf16", clip=clip, cap=200_000, steps=6)
    inp = Inputs(wl)
    lay = oracle_layout(wl)
    starts = lay.logical_starts()
    B = len(lay.buckets)
    grads = lambda t: {b: [inp.grad_np(t, w, starts[b], lay.buckets[b].numel) for w in range(4)] for b in range(B)}
    straight = run_oracle_full(wl, inp, 6)
    g = GpuShadow(wl, inp, num_streams=streams, batch_bytes=batch_bytes)
    A = g.layout.arena_numel
    host = [torch.empty(A, dtype=torch.float32).pin_memory() for _ in range(3)]
    restarted = None
    for t in range(1, 7):
        g.fill_grads(t)
        g.apply_step(t)
        if restarted is not None:
            restarted.step(grads(t))
        if t % 2 == 0:
            # the snapshot is enqueued right behind the iteration, with no synchronisation in between
            assert g.ctx.snapshot(*(h.data_ptr() for h in host)) == t
            assert g.ctx.snapshot_wait() == t
            g.close()
            g = GpuShadow(wl, inp, init_from=[h.clone() for h in host], start_step=t, num_streams=streams, batch_bytes=batch_bytes)
            cut = lambda h: [h.numpy()[off:off + n].copy() for off, n, _ in g.buckets]
            if restarted is not None:
                for b in range(B):      # what the GPU handed over is what the restarted oracle holds
                    assert_state_matches(tuple(cut(h)[b] for h in host), (restarted.p[b], restarted.m[b], restarted.v[b]),
                                         f"snapshot at {t} bucket {b}")
            restarted = oracle.OracleShadow(lay, oracle_hparams(wl), cut(host[0]), start_step=t, m=cut(host[1]), v=cut(host[2]))
    for b in range(B):
        got = g.bucket_state(b)
        assert_state_matches(got, (straight.p[b], straight.m[b], straight.v[b]), f"restored run vs straight oracle, bucket {b}")
        assert_state_matches(got, (restarted.p[b], restarted.m[b], restarted.v[b]), f"restored run vs restarted oracle, bucket {b}")
    # device-side snapshot equals the arenas, and its step is the completed one
    dst = [torch.empty(A, dtype=torch.float32, device="cuda:0") for _ in range(3)]
    assert g.ctx.snapshot(*(d.data_ptr() for d in dst)) == 6
    g.ctx.sync()
    assert all(torch.equal(a, b) for a, b in zip(dst, (g.p, g.m, g.v)))
    g.close()


@pytest.mark.parametrize("clip,streams,batch_bytes", [(0.01, 3, 0), (0.0, 3, 1 << 21), (0.0, 4, 0)])
def test_snapshot_orders_before_next_iteration(clip, streams, batch_bytes):
    """A snapshot enqueued at a boundary holds that iteration's state even if the next iteration is enqueued right
    behind it: the copies run on the library's copy stream, the next iteration's folds may overlap them, and the
    kernels that write the replica wait (with clipping off those are the fused per-bucket kernels on every stream)."""
    say("case snapshot ordering", clip, streams, batch_bytes)
    wl = custom("snap-order", [(3_000_001, True), (2_000_003, False), (1_000_000, True), (500_000, True)], 4, "bf16", clip=clip,
                cap=1 << 22, steps=3)
    inp = Inputs(wl)
    g = GpuShadow(wl, inp, num_streams=streams, batch_bytes=batch_bytes)
    A = g.layout.arena_numel
    g.run_step(1)
    want = [x.clone() for x in (g.p, g.m, g.v)]
    dst = [torch.empty(A, dtype=torch.float32, device="cuda:0") for _ in range(3)]
    host = [torch.empty(A, dtype=torch.float32).pin_memory() for _ in range(3)]
    g.fill_grads(2)
    done = torch.cuda.Event()
    done.record()                       # creates the handle; the library records it again behind its copies
    assert g.ctx.snapshot(*(d.data_ptr() for d in dst)) == 1
    assert g.ctx.snapshot(*(h.data_ptr() for h in host), done_event=done.cuda_event) == 1
    g.apply_step(2)
    done.synchronize()                  # the copies are complete; iteration 2 may still be running
    assert all(torch.equal(a.cpu(), b) for a, b in zip(want, host))
    g.ctx.sync()
    assert all(torch.equal(a, b) for a, b in zip(dst, want))
    assert not torch.equal(g.p, want[0])
    orc = run_oracle_full(wl, inp, 2)
    for b in range(len(g.buckets)):
        assert_state_matches(g.bucket_state(b), (orc.p[b], orc.m[b], orc.v[b]), f"after the snapshot, bucket {b}")
    g.close()


def test_snapshot_destinations_device_pinned_and_pageable():
    """Pinned host memory is written by the library's drain kernel, device memory and pageable host memory by the
    runtime's copy; all three hold the same state."""
    say("case snapshot destinations")
    wl = custom("snap-dst", RAGGED, 2, "bf16", clip=0.01, cap=200_000, steps=2)
    g = GpuShadow(wl, Inputs(wl), num_streams=2, launch=sh.LaunchShape(drain_blocks=3))
    A = g.layout.arena_numel
    g.run_step(1)
    dev = [torch.empty(A, dtype=torch.float32, device="cuda:0") for _ in range(3)]
    pinned = [torch.empty(A, dtype=torch.float32, pin_memory=True) for _ in range(3)]
    pageable = [torch.empty(A, dtype=torch.float32) for _ in range(3)]
    inner = torch.empty(3 * A + 64, dtype=torch.float32, pin_memory=True)        # destinations inside a larger pinned block
    inside = [inner[64 + k * A:64 + (k + 1) * A] for k in range(3)]
    for dst in (dev, pinned, pageable, inside):
        assert g.ctx.snapshot(*(d.data_ptr() for d in dst)) == 1
    assert g.ctx.snapshot_wait() == 1
    g.ctx.sync()
    for dst in (dev, pinned, pageable, inside):
        assert all(torch.equal(d.cpu(), x.cpu()) for d, x in zip(dst, (g.p, g.m, g.v)))
    g.close()


@pytest.mark.parametrize("clip,refold,streams,batch_bytes,optimizer", [(0.01, False, 2, 0, "adamw"), (0.0, False, 3, 1 << 20, "adamw"),
                                                                       (0.01, True, 2, 1 << 62, "adamw"), (0.01, False, 1, 0, "sgd"),
                                                                       (0.0, False, 2, 0, "adam")])
def test_staged_snapshot_drains_while_later_iterations_run(clip, refold, streams, batch_bytes, optimizer):
    """Armed before iteration t, the update kernels of t write the staging set as well; iterations t+1 and t+2 are
    enqueued at once and the host copy drained from the staging set still equals the ORACLE's state after t."""
    say("case staged snapshot", clip, refold, streams, batch_bytes, optimizer)
    W = 1 if refold else 4
    wl = custom("staged", RAGGED + [(1_500_003, True), (900_001, False)], W, "bf16", clip=clip, cap=1 << 21, steps=5, wd=0.1,
                lr=0.05 if optimizer == "sgd" else 1e-3)
    inp = Inputs(wl)
    g = GpuShadow(wl, inp, num_streams=streams, batch_bytes=batch_bytes, refold=refold, optimizer=optimizer, snapshot_set=True)
    A, B = g.layout.arena_numel, len(g.buckets)
    sgd = optimizer == "sgd"
    host = [torch.full((A,), 7.0, dtype=torch.float32).pin_memory() for _ in range(3)]
    states = {}
    run_oracle_full(wl, inp, 5, optimizer=optimizer,
                    on_step=lambda t, o: states.__setitem__(t, [[x.copy() for x in o.p], [x.copy() for x in o.m], [x.copy() for x in o.v]]))
    with pytest.raises(sh.ShadowError) as e:
        g.ctx.snapshot_wait()                       # nothing requested yet
    assert e.value.status == binding.EINVAL
    # every iteration's views are kept on the device, so that nothing below has to wait for the host
    views = {}
    for t in range(1, 6):
        g.fill_grads(t)
        views[t] = g._stage.clone()

    def apply(t):
        cur = torch.cuda.current_stream()
        if t > 1 and not refold:
            # release side: the previous iteration's readers of the views, stream by stream
            for s in range(min(streams, B)):
                rel = torch.cuda.Event()
                rel.record()
                g.ctx.record_consumed(s, rel.cuda_event)
                cur.wait_event(rel)
        elif t > 1:
            rel = torch.cuda.Event()
            rel.record()
            g.ctx.record_consumed(0, rel.cuda_event)        # folding twice: the last reader ran at the iteration's end
            cur.wait_event(rel)
        g._stage.copy_(views[t])        # on torch's stream ...
        ev = torch.cuda.Event()
        ev.record()
        for b in range(B):              # ... ordered before the folds by the event, never by the host
            g.ctx.apply_bucket(b, g._views[b], t, ready_event=ev.cuda_event)

    apply(1)
    g.ctx.snapshot_arm(host[0].data_ptr(), host[1].data_ptr(), None if sgd else host[2].data_ptr())
    assert g.ctx.try_snapshot_arm() == binding.EBUSY            # already armed
    with pytest.raises(sh.ShadowError) as e:
        g.ctx.snapshot_wait()                                   # its iteration has not run yet
    assert e.value.status == binding.EBUSY
    apply(2)                                                    # the armed iteration
    apply(3)
    apply(4)
    assert g.ctx.snapshot_wait() == 2
    ref = states[2]
    for b, (off, n, _) in enumerate(g.buckets):
        got = tuple(h.numpy()[off:off + n] for h in host)
        if sgd:
            got = got[:2] + (ref[2][b],)
        assert_state_matches(got, (ref[0][b], ref[1][b], ref[2][b]), f"drained snapshot of iteration 2, bucket {b}")
    # the staging set has the replica's layout: its alignment gaps are zero as well
    for (off, n, _), nxt in zip(g.buckets[:-1], g.buckets[1:]):
        assert nxt[0] == off + n or float(host[0][off + n:nxt[0]].abs().max()) == 0.0
    # arming is refused inside an iteration
    g.ctx.sync()
    g._stage.copy_(views[5])
    torch.cuda.synchronize()
    g.ctx.apply_bucket(0, g._views[0], 5)
    if B > 1:
        assert g.ctx.try_snapshot_arm() == binding.EBUSY
    for b in range(1, B):
        g.ctx.apply_bucket(b, g._views[b], 5)
    g.ctx.sync()
    o = states[5]
    for b in range(B):
        assert_state_matches(g.bucket_state(b), (o[0][b], o[1][b], o[2][b]), f"replica after 5 iterations, bucket {b}")
    g.close()


def test_views_from_a_foreign_stream_need_no_host_sync():
    """The views are written by a producer on its own stream (here: a slow kernel, then copies); the event recorded
    behind them is all the ordering there is, also when the fold launch is deferred (batch_bytes > 0)."""
    say("case foreign producer stream")
    for bb, clip in ((0, 0.0), (1 << 62, 0.01), (1 << 20, 0.0)):
        wl = custom("producer", RAGGED + [(2_000_003, True)], 4, "bf16", clip=clip, cap=1 << 21, steps=2)
        inp = Inputs(wl)
        g = GpuShadow(wl, inp, num_streams=2, batch_bytes=bb)
        B = len(g.buckets)
        src = {}
        for t in (1, 2):
            g.fill_grads(t)
            src[t] = g._stage.clone()
        torch.cuda.synchronize()
        producer = torch.cuda.Stream()
        for t in (1, 2):
            with torch.cuda.stream(producer):
                if t == 2:
                    # the views of iteration 1 must have been read before they are overwritten
                    for s in range(min(2, B)):
                        rel = torch.cuda.Event()
                        rel.record(producer)
                        g.ctx.record_consumed(s, rel.cuda_event)
                        producer.wait_event(rel)
                g._stage.fill_(0x7F)                  # garbage (NaN patterns) until the producer is done
                torch.cuda._sleep(2_000_000)         # some milliseconds: a fold that did not wait would read the garbage
                g._stage.copy_(src[t], non_blocking=True)
                evs = []
                for b in range(B):
                    ev = torch.cuda.Event()
                    ev.record(producer)
                    evs.append(ev)
            for b in range(B):
                g.ctx.apply_bucket(b, g._views[b], t, ready_event=evs[b].cuda_event)
        orc = run_oracle_full(wl, inp, 2)
        for b in range(B):
            assert_state_matches(g.bucket_state(b), (orc.p[b], orc.m[b], orc.v[b]), f"producer bb={bb} bucket {b}")
        g.close()


@pytest.mark.parametrize("W,dtype,clip,refold", [(8, "bf16", 0.01, False), (3, "f32", 0.0, False), (1, "bf16", 0.01, True)])
def test_logical_launches_split_into_several(W, dtype, clip, refold):
    """max_launch_threads far below the sizes involved: the whole-arena sweep, the fold batches and the copy kernel
    each run as many launches (block_base > 0), with the bits of the oracle."""
    say("case split launches", W, dtype, clip, refold)
    wl = custom("split", RAGGED, W, dtype, clip=clip, cap=200_000, steps=3, random_arrival=True)
    nthreads = sum(n for n, _ in RAGGED) // 4
    for limit, fold_block, sweep_block in ((4096, 1024, 256), (1000, 256, 64), (1 << 16, 512, 1024)):
        assert nthreads // limit >= 1
        launch = sh.LaunchShape(fold_block=fold_block, fused_block=fold_block // 2, sweep_block=sweep_block, max_launch_threads=limit,
                                fold_waves_per_cu=16, fused_waves_per_cu=12, sweep_waves_per_cu=8)
        check_against_oracle(wl, num_streams=2, batch_bytes=1 << 62, refold=refold, launch=launch)
    n = 3_000_000
    src = torch.randint(0, 255, (n * 16,), dtype=torch.uint8, device="cuda:0")
    for limit in (0, 1 << 20, 5000, 256, 1):
        dst = torch.zeros_like(src)
        sh.shadow_copy_probe(dst.data_ptr(), src.data_ptr(), n * 16, 0, limit)
        torch.cuda.synchronize()
        assert torch.equal(src, dst), limit


@pytest.mark.parametrize("n_src,n_dst", [(0, 1), (0, 3), (1, 1), (2, 1), (4, 3), (7, 3), (8, 1), (16, 1), (4, 0), (16, 0)])
def test_stream_probe_writes_what_it_says(n_src, n_dst):
    """The bandwidth yardstick (a measurement aid, not part of the method): every destination holds the XOR of the
    sources with the destination's index added to the first word; with no destination nothing is written."""
    say("case stream probe", n_src, n_dst)
    n = 1_000_003                                    # vectors: several blocks and a ragged last one
    srcs = [torch.randint(-2 ** 31, 2 ** 31 - 1, (n, 4), dtype=torch.int32, device="cuda:0") for _ in range(n_src)]
    dsts = [torch.full((n + 1, 4), 5, dtype=torch.int32, device="cuda:0") for _ in range(n_dst)]
    sink = torch.full((4,), 5, dtype=torch.int32, device="cuda:0")
    torch.cuda.synchronize()
    for block, waves in ((0, 0), (64, 8), (1024, 32)):
        rc = sh.shadow_stream_probe([d.data_ptr() for d in dsts], [x.data_ptr() for x in srcs], n * 16,
                                    sink=sink.data_ptr() if n_dst == 0 else None, block=block, waves_per_cu=waves)
        assert rc == binding.OK
        torch.cuda.synchronize()
        if n_src:
            want = srcs[0].clone()
            for x in srcs[1:]:
                want ^= x
        else:
            want = torch.zeros((n, 4), dtype=torch.int32, device="cuda:0")
            want[:, 0] = torch.arange(n, dtype=torch.int64, device="cuda:0").to(torch.int32)
        for d, out in enumerate(dsts):
            exp = want.clone()
            exp[:, 0] += d                           # wraps like the kernel's unsigned add
            assert torch.equal(out[:n], exp), (n_src, n_dst, d, block)
            assert int(out[n].min()) == 5 and int(out[n].max()) == 5      # nothing past the end
            out.fill_(5)
        assert int(sink.min()) == 5 and int(sink.max()) == 5


def test_stream_probe_in_place():
    """Destinations that are sources as well, the shape of the optimizer sweep: every lane reads before it writes."""
    say("case stream probe in place")
    n = 300_007
    srcs = [torch.randint(-2 ** 31, 2 ** 31 - 1, (n, 4), dtype=torch.int32, device="cuda:0") for _ in range(4)]
    want = srcs[0] ^ srcs[1] ^ srcs[2] ^ srcs[3]
    torch.cuda.synchronize()
    assert sh.shadow_stream_probe([x.data_ptr() for x in srcs[1:]], [x.data_ptr() for x in srcs], n * 16, block=256, waves_per_cu=16) == binding.OK
    torch.cuda.synchronize()
    for d, out in enumerate(srcs[1:]):
        exp = want.clone()
        exp[:, 0] += d
        assert torch.equal(out, exp), d


def test_exactly_once_errors_leave_state_untouched():
    """Section 4.1: duplication or loss of a bucket must not go unnoticed."""
    say("case errors")
    wl = custom("errors", [(5000, True), (6000, False), (7000, True)], 2, "bf16", clip=0.01, cap=12_000, steps=2)
    g = GpuShadow(wl, Inputs(wl))
    B = len(g.buckets)
    assert B >= 2
    g.fill_grads(1)
    before = [x.clone() for x in (g.p, g.m, g.v)]
    v0 = g._views[0]
    assert g.ctx.try_apply_bucket(B, v0, 1) == binding.EBUCKET
    assert g.ctx.try_apply_bucket(0, v0, 2) == binding.ESTEP
    assert g.ctx.try_apply_bucket(0, v0, 0) == binding.ESTEP
    misaligned = g.ctx.views_array([g.view(0, 0)[1:].data_ptr(), g.view(0, 1).data_ptr()])
    assert g.ctx.try_apply_bucket(0, misaligned, 1) == binding.EINVAL
    assert g.ctx.try_apply_bucket(0, g.ctx.views_array([g.view(0, 0).data_ptr(), 0]), 1) == binding.EINVAL
    g.ctx.sync()
    assert all(torch.equal(a, b) for a, b in zip(before, (g.p, g.m, g.v))) and g.ctx.step() == (0, 0)
    assert g.ctx.try_apply_bucket(0, v0, 1) == binding.OK
    assert g.ctx.try_apply_bucket(0, v0, 1) == binding.EDUP
    assert g.ctx.step() == (0, B - 1)
    with pytest.raises(sh.ShadowError) as e:
        g.ctx.snapshot(None, None, None)
    assert e.value.status == binding.EBUSY
    with pytest.raises(sh.ShadowError) as e:
        g.ctx.set_lr(1e-4)
    assert e.value.status == binding.EBUSY
    assert g.ctx.try_apply_bucket(1, g._views[1], 2) == binding.ESTEP      # next iteration before this one is complete
    for b in range(1, B):
        assert g.ctx.try_apply_bucket(b, g._views[b], 1) == binding.OK
    g.ctx.sync()
    assert g.ctx.step() == (1, 0)
    assert g.ctx.try_apply_bucket(0, v0, 1) == binding.ESTEP                # replay of a finished iteration
    # the finished iteration equals the oracle's
    inp = Inputs(wl)
    orc = run_oracle_full(wl, inp, 1)
    for b in range(B):
        assert_state_matches(g.bucket_state(b), (orc.p[b], orc.m[b], orc.v[b]), f"errors bucket {b}")
    g.close()


def test_snapshot_and_event_calls_refuse_bad_arguments():
    """Argument checks of the staged-snapshot and producer/consumer calls; nothing they refuse changes the replica."""
    say("case snapshot/event errors")
    wl = custom("snap-errors", [(5000, True), (6000, False), (7000, True)], 2, "bf16", clip=0.01, cap=12_000, steps=1)
    g = GpuShadow(wl, Inputs(wl))
    L, h = sh.lib(), g.ctx._h
    A = g.layout.arena_numel
    B = len(g.buckets)
    stage = [torch.zeros(A + 64, dtype=torch.float32, device="cuda:0") for _ in range(3)]
    sp = [t.data_ptr() for t in stage]
    ev = torch.cuda.Event()
    ev.record()
    before = [x.clone() for x in (g.p, g.m, g.v)]
    assert L.shadow_snapshot_arm(h, None, None, None) == binding.EINVAL                 # no staging set lent yet
    assert L.shadow_snapshot_record(h, ev.cuda_event) == binding.EINVAL                 # no snapshot requested yet
    assert L.shadow_snapshot_attach(h, sp[0], sp[1], None) == binding.EINVAL            # AdamW has a second state array
    assert L.shadow_snapshot_attach(h, sp[0] + 4, sp[1], sp[2]) == binding.EINVAL       # misaligned
    assert L.shadow_snapshot_attach(h, sp[0], sp[0], sp[2]) == binding.EINVAL           # the same array twice
    assert L.shadow_snapshot_attach(h, g.p.data_ptr(), sp[1], sp[2]) == binding.EINVAL  # the replica itself
    assert L.shadow_snapshot_attach(h, sp[0], sp[1], sp[2]) == binding.OK
    assert L.shadow_snapshot_attach(h, sp[0], sp[1], sp[2]) == binding.EINVAL           # at most once
    assert L.shadow_record_consumed(h, B, ev.cuda_event) == binding.EBUCKET
    assert L.shadow_record_consumed(h, 0, None) == binding.EINVAL
    assert L.shadow_record_consumed(h, 0, ev.cuda_event) == binding.OK                  # nothing pending: records at once
    ev.synchronize()
    g.fill_grads(1)
    g.ctx.apply_bucket(0, g._views[0], 1, ready_event=ev.cuda_event)
    assert L.shadow_snapshot_attach(h, sp[0], sp[1], sp[2]) == binding.EINVAL
    assert L.shadow_snapshot_arm(h, None, None, None) == binding.EBUSY                  # an iteration is open
    for b in range(1, B):
        g.ctx.apply_bucket(b, g._views[b], 1)
    g.ctx.sync()
    assert all(not torch.equal(a, b) for a, b in zip(before[:1], (g.p,)))
    assert all(float(t.abs().max()) == 0.0 for t in stage)                              # never armed: staging set untouched
    g.close()
    # folding twice (no scratch arena): the views are read again at the end of the iteration, no release before that
    wl2 = custom("snap-errors-refold", [(5000, True), (6000, False), (7000, True)], 1, "bf16", clip=0.01, cap=12_000, steps=1)
    g2 = GpuShadow(wl2, Inputs(wl2), refold=True)
    g2.fill_grads(1)
    g2.ctx.apply_bucket(0, g2._views[0], 1)
    assert sh.lib().shadow_record_consumed(g2.ctx._h, 0, ev.cuda_event) == binding.EBUSY
    for b in range(1, len(g2.buckets)):
        g2.ctx.apply_bucket(b, g2._views[b], 1)
    assert sh.lib().shadow_record_consumed(g2.ctx._h, 0, ev.cuda_event) == binding.OK
    ev.synchronize()
    g2.close()


def test_per_step_learning_rate():
    """Cosine-annealed learning rate (section 6) supplied per iteration by the caller."""
    say("case lr schedule")
    import math
    wl = custom("lr", RAGGED[:7], 2, "bf16", clip=0.0, cap=150_000, steps=5)
    inp = Inputs(wl)
    lrs = [float(np.float32(1e-3 * 0.5 * (1 + math.cos(math.pi * t / 5)))) for t in range(5)]
    g = GpuShadow(wl, inp)
    lay = oracle_layout(wl)
    starts = lay.logical_starts()
    orc = oracle.OracleShadow(lay, oracle.HParams(lr=lrs[0], weight_decay=wl.weight_decay),
                              [inp.param_np(s, b.numel) for s, b in zip(starts, lay.buckets)])
    for t in range(1, 6):
        g.ctx.set_lr(lrs[t - 1])
        orc.hp.lr = lrs[t - 1]
        g.run_step(t)
        orc.step({b: [inp.grad_np(t, w, starts[b], lay.buckets[b].numel) for w in range(2)] for b in range(len(lay.buckets))})
    for b in range(len(lay.buckets)):
        assert_state_matches(g.bucket_state(b), (orc.p[b], orc.m[b], orc.v[b]), f"lr bucket {b}")
    g.close()
