"""The entry point that allocates nothing (shadow_apply_iteration_static) against the context path and the oracle.

Run last: it shares nothing with the other tests, but a failure here must not hide theirs.
"""
import sys

import numpy as np
import pytest
import torch

import paper_2507_13522_amd as sh
from paper_2507_13522_amd import binding
import synth
from harness import GpuShadow, Inputs, assert_state_matches, run_oracle_full

pytestmark = pytest.mark.gpu

BIG = [(5000, True), (33, False), (700_001, True), (1, False), (64, True), (123_457, False), (300_007, True), (999, True),
       (2048, False), (77_777, True), (7, True), (3, False), (5, True), (1024, True), (8, False)]
SMALL = [(4099, True), (17, False), (20_011, True), (9000, False)]


def workload(name, sizes, W, dtype, clip, cap, optimizer):
    ts = [synth.TensorSpec(f"t{i}", n, f) for i, (n, f) in enumerate(sizes)]
    return synth.Workload(name, ts, num_workers=W, grad_dtype=dtype, grad_dist="normal", grad_sigma=1e-3, steps=2,
                          max_grad_norm=clip, bucket_cap_bytes=cap, weight_decay=0.1, lr=0.05 if optimizer == "sgd" else 1e-3)


def via_context(wl, inp, optimizer, refold, steps):
    g = GpuShadow(wl, inp, num_streams=2, batch_bytes=1 << 20, refold=refold, optimizer=optimizer)
    for t in range(1, steps + 1):
        g.run_step(t)
    out = [x.clone() for x in (g.p, g.m, g.v)]
    g.close()
    return out


class StaticRun:
    """Arenas and resident views for the static entry point (memory comes from torch; the call itself allocates nothing)."""

    def __init__(self, wl, inp, optimizer, refold):
        self.g = GpuShadow(wl, inp, num_streams=1, refold=refold, optimizer=optimizer)     # used for its memory and views only
        g = self.g
        g.ctx.sync()
        self.sgd = optimizer == "sgd"
        W = wl.num_workers
        self.views = (binding.C.c_void_p * (len(g.buckets) * W))(*[g.view(b, w).data_ptr() for b in range(len(g.buckets))
                                                                   for w in range(W)])

    def step(self, t, stream):
        g = self.g
        return sh.shadow_apply_iteration_static(g.layout, g.hp, g.p.data_ptr(), g.m.data_ptr(), None if self.sgd else g.v.data_ptr(),
                                                g.r.data_ptr() if g.r is not None else None, self.views, t, stream)


@pytest.mark.parametrize("W,dtype,clip,refold,optimizer", [(8, "bf16", 0.01, False, "adamw"), (4, "bf16", 0.0, False, "adamw"),
                                                           (1, "bf16", 0.01, True, "adamw"), (3, "f32", 0.01, False, "sgd"),
                                                           (2, "f32", 0.0, False, "adam")])
def test_two_calls_in_a_row_second_one_smaller(W, dtype, clip, refold, optimizer):
    """Two iterations of a larger replica, then -- with nothing in between but the stream's order -- two of a smaller
    one with another layout: the scratch still holds the first replica's tables and partials when the second starts.
    Both must equal the context path bit for bit, and the oracle."""
    print("case static", W, dtype, clip, refold, optimizer, flush=True)
    sys.stdout.flush()
    big = workload("static-big", BIG, W, dtype, clip, 400_000, optimizer)
    small = workload("static-small", SMALL, W, dtype, clip, 30_000, optimizer)
    ibig, ismall = Inputs(big), Inputs(small)
    want_big = via_context(big, ibig, optimizer, refold, 2)
    want_small = via_context(small, ismall, optimizer, refold, 2)
    rb, rs = StaticRun(big, ibig, optimizer, refold), StaticRun(small, ismall, optimizer, refold)
    stream = torch.cuda.Stream()
    # one set of views per replica: iteration 2 reuses them, so its inputs are written on the same stream, in order
    with torch.cuda.stream(stream):
        for t in (1, 2):
            rb.g.fill_grads(t)                  # synchronizes: the views are complete before the call
            assert rb.step(t, stream.cuda_stream) == binding.OK
            stream.synchronize()
        for t in (1, 2):
            rs.g.fill_grads(t)
            assert rs.step(t, stream.cuda_stream) == binding.OK
            stream.synchronize()
    for name, run, want, wl, inp in (("big", rb, want_big, big, ibig), ("small", rs, want_small, small, ismall)):
        g = run.g
        for a, b, what in zip((g.p, g.m, g.v), want, "pmv"):
            if optimizer == "sgd" and what == "v":
                continue
            assert torch.equal(a, b), f"{name} {what}: static entry point differs from the context path"
        orc = run_oracle_full(wl, inp, 2, optimizer=optimizer)
        for b in range(len(g.buckets)):
            off, n, _ = g.buckets[b]
            got = tuple(x[off:off + n].cpu().numpy() for x in (g.p, g.m, g.v))
            assert_state_matches(got, (orc.p[b], orc.m[b], orc.v[b]), f"static {name} bucket {b}")
    rb.g.close(); rs.g.close()


def test_back_to_back_without_host_sync():
    """The two calls really in a row on one stream: the larger replica's iteration, then the smaller one's, no
    synchronisation between them."""
    print("case static back to back", flush=True)
    big = workload("static-big", BIG, 8, "bf16", 0.01, 400_000, "adamw")
    small = workload("static-small", SMALL, 8, "bf16", 0.01, 30_000, "adamw")
    ibig, ismall = Inputs(big), Inputs(small)
    want_big = via_context(big, ibig, "adamw", False, 1)
    want_small = via_context(small, ismall, "adamw", False, 1)
    rb, rs = StaticRun(big, ibig, "adamw", False), StaticRun(small, ismall, "adamw", False)
    rb.g.fill_grads(1)
    rs.g.fill_grads(1)
    stream = torch.cuda.Stream()
    assert rb.step(1, stream.cuda_stream) == binding.OK
    assert rs.step(1, stream.cuda_stream) == binding.OK
    stream.synchronize()
    for run, want in ((rb, want_big), (rs, want_small)):
        for a, b in zip((run.g.p, run.g.m, run.g.v), want):
            assert torch.equal(a, b)
    rb.g.close(); rs.g.close()


def test_limits_and_arguments():
    print("case static limits", flush=True)
    hp = sh.HParams(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, max_grad_norm=1.0, num_workers=1,
                    grad_dtype=sh.GRAD_BF16, reduce_op=sh.REDUCE_MEAN, num_streams=1)
    too_big = sh.Layout([(binding.STATIC_MAX_ARENA_NUMEL + 64, True)], 2, 1 << 40)
    buf = torch.zeros(1024, dtype=torch.float32, device="cuda:0")
    before = buf.clone()
    p = buf.data_ptr()
    assert sh.shadow_apply_iteration_static(too_big, hp, p, p + 256, p + 512, p + 768, [p + 1024], 1) == binding.ETOOBIG
    many = sh.Layout([(1, True)] * (binding.STATIC_MAX_BUCKETS + 1), 2, 2)        # one bucket per tensor
    assert many.num_buckets == binding.STATIC_MAX_BUCKETS + 1
    assert sh.shadow_apply_iteration_static(many, hp, p, p + 256, p + 512, None, [p + 1024] * many.num_buckets, 1) == binding.ETOOBIG
    assert "static scratch" in sh.shadow_strerror(binding.ETOOBIG)
    ok = sh.Layout([(100, True)], 2, 1000)
    assert sh.shadow_apply_iteration_static(ok, hp, p, p + 256, p + 512, None, [p + 1024], 0) == binding.EINVAL       # steps count from 1
    assert sh.shadow_apply_iteration_static(ok, hp, p, p + 256, p + 512, None, [p + 1024 + 2], 1) == binding.EINVAL   # misaligned view
    assert sh.shadow_apply_iteration_static(ok, hp, p, p + 256, p + 512, None, [0], 1) == binding.EINVAL
    torch.cuda.synchronize()
    assert torch.equal(buf, before)              # nothing was enqueued by the refused calls
