"""A replica on cuda:0 over torch-allocated memory: placement of the arenas, the gradient views and an
optional snapshot staging set in HBM, then the context of ``binding.Shadow`` over them.

PyTorch is used for device memory and (optionally) streams only; every step of the update runs in the
library's kernels.  Placement follows the library's advice (``shadow_layout_device_plan``,
``shadow_layout_arena_stride``, ``shadow_layout_staging_*``) and degrades instead of failing:

    "plan"      ONE allocation of 256 GiB made first thing, everything at the advised offsets
                (arenas spread over the 96 GiB regions of the HBM) -- the fastest; needs the block
    "stride"    the arenas carved from one allocation, a power-of-two stride apart; views separate
    "separate"  every arena an allocation of its own, wherever the allocator puts it
    "packed"    the arenas back to back in one allocation (small test cases)
    "explicit"  ONE allocation of 256 GiB, byte offsets given by the caller (placement experiments)

``placement="auto"`` asks for the plan when the arenas reach 256 MiB and falls back to "stride" when
the plan does not fit or the block cannot be allocated; ``Memory.placement`` names what was used.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import torch

from . import binding as sh

DEVICE_PLAN_MIN_ARENA_BYTES = 256 << 20
# launch configuration of the benchmark: one stream, the iteration's buckets folded in as few launches as possible
BENCH_STREAMS = 1
BENCH_BATCH_BYTES = 4 << 30
OPTIMIZERS = {"adamw": sh.OPT_ADAMW, "adam": sh.OPT_ADAM, "sgd": sh.OPT_SGD}


class Memory:
    """p, m, v, the scratch arena r (or None), the views' staging buffer (or None) and the snapshot set (or None)."""

    def __init__(self, layout: sh.Layout, with_scratch: bool, staging_bytes: int, with_snapshot_set: bool = False,
                 placement: str = "auto", device: str = "cuda:0", offsets: Optional[dict] = None):
        """offsets (placement "explicit"): byte offsets {"param", "m", "v", "scratch", "staging"} inside a 256 GiB block."""
        dev = torch.device(device)
        A = layout.arena_numel
        narr = 4 if with_scratch else 3
        want = placement
        if placement == "auto":
            want = "plan" if A * 4 >= DEVICE_PLAN_MIN_ARENA_BYTES else "stride"
        self.block = None
        self.stage = None
        self.snap = None
        arenas: List[torch.Tensor] = []
        if want == "explicit":
            assert offsets is not None and not with_snapshot_set
            self.block = torch.empty(256 << 30, dtype=torch.uint8, device=dev)
            cut = lambda o: self.block[o:o + A * 4].view(torch.float32)
            arenas = [cut(offsets["param"]), cut(offsets["m"]), cut(offsets["v"])]
            if with_scratch:
                arenas.append(cut(offsets["scratch"]))
            if staging_bytes:
                self.stage = self.block[offsets["staging"]:offsets["staging"] + staging_bytes]
            spans = sorted([(offsets[k], A * 4) for k in ("param", "m", "v")] + ([(offsets["scratch"], A * 4)] if with_scratch else [])
                           + ([(offsets["staging"], staging_bytes)] if staging_bytes else []))
            assert all(a + n <= b for (a, n), (b, _) in zip(spans, spans[1:])) and spans[-1][0] + spans[-1][1] <= (256 << 30), "parts overlap"
        if want == "plan":
            plan = layout.device_plan(with_scratch, staging_bytes, with_snapshot_set)
            if plan is not None:
                try:
                    self.block = torch.empty(plan.block_bytes, dtype=torch.uint8, device=dev)
                except torch.OutOfMemoryError:
                    self.block = None
                    torch.cuda.empty_cache()
            if self.block is not None:
                cut = lambda o: self.block[o:o + A * 4].view(torch.float32)
                arenas = [cut(plan.param_offset), cut(plan.m_offset), cut(plan.v_offset)]
                if with_scratch:
                    arenas.append(cut(plan.scratch_offset))
                if staging_bytes:
                    self.stage = self.block[plan.staging_offset:plan.staging_offset + staging_bytes]
                if with_snapshot_set:
                    self.snap = [cut(plan.snap_param_offset), cut(plan.snap_m_offset), cut(plan.snap_v_offset)]
            else:
                want = "stride"                     # no plan for this size, or the block is not to be had
        if want in ("stride", "packed"):
            stride = layout.arena_stride() if want == "stride" else (A * 4 + 255) // 256 * 256
            self.block = torch.empty((narr - 1) * stride + A * 4, dtype=torch.uint8, device=dev)
            arenas = [self.block[k * stride:k * stride + A * 4].view(torch.float32) for k in range(narr)]
        elif want == "separate":
            arenas = [torch.empty(A, dtype=torch.float32, device=dev) for _ in range(narr)]
        elif want not in ("plan", "explicit"):
            raise ValueError(f"placement {placement!r}")
        if staging_bytes and self.stage is None:
            self.stage = torch.empty(staging_bytes, dtype=torch.uint8, device=dev)
        if with_snapshot_set and self.snap is None:
            self.snap = [torch.empty(A, dtype=torch.float32, device=dev) for _ in range(3)]
        self.p, self.m, self.v = arenas[:3]
        self.r = arenas[3] if with_scratch else None
        self.placement = want


class GpuShadow:
    """The library on cuda:0 over torch-allocated arenas for one workload (a ``synth.Workload``-shaped object:
    tensors, num_workers, grad_dtype, grad_bytes, hyper-parameters), with every bucket's W views resident in a
    bucket-major staging buffer, or taking turns in a ring of ``ring_bytes`` when they do not all fit.

    ``inputs`` fills parameters and views (``fill_param_dev`` / ``fill_grad_dev``).
    """

    def __init__(self, wl, inputs, num_streams: int = 2, mean: bool = True, torch_streams: bool = False,
                 resident_grads: bool = True, init_from=None, start_step: int = 0, advised_placement: bool = True,
                 batch_bytes: int = 0, refold: bool = False, optimizer: str = "adamw", ring_bytes: int = 0,
                 placement: Optional[str] = None, snapshot_set: bool = False, launch: Optional[sh.LaunchShape] = None,
                 attach_snapshot_set: bool = True, offsets: Optional[dict] = None):
        assert torch.cuda.is_available()
        self.wl, self.inputs = wl, inputs
        self.dev = torch.device("cuda:0")
        inputs.device = self.dev
        self.layout = sh.Layout([(t.numel, t.weight_decay) for t in wl.tensors], wl.grad_bytes, wl.bucket_cap_bytes,
                                wl.explicit_buckets)
        L = self.layout
        self.buckets = [L.bucket(b) for b in range(L.num_buckets)]
        self.logical_start, acc = [], 0
        for off, n, _ in self.buckets:
            self.logical_start.append(acc)
            acc += n
        clip = wl.max_grad_norm > 0
        W = wl.num_workers
        stage_bytes = max(L.staging_bytes(W), 256) if resident_grads else 0
        # ring_bytes > 0 (timing only): the views do not all fit, so bucket after bucket takes the next piece of a
        # ring of that size and later buckets reuse the memory of earlier ones; contents are then meaningless
        self._ring_off = None
        if resident_grads and ring_bytes:
            self._ring_off, cur = [], 0
            for b in range(L.num_buckets):
                need = (L.staging_view(W, b, W - 1) - L.staging_view(W, b, 0)) + self.buckets[b][1] * wl.grad_bytes
                need = (need + (2 << 20) - 1) // (2 << 20) * (2 << 20)
                assert need <= ring_bytes, "ring smaller than one bucket's views"
                if cur + need > ring_bytes:
                    cur = 0
                self._ring_off.append(cur)
                cur += need
            stage_bytes = ring_bytes
        if placement is None:
            placement = "auto" if advised_placement else "packed"
        self.mem = Memory(L, clip and not refold, stage_bytes, snapshot_set, placement, "cuda:0", offsets)
        self.placement = self.mem.placement
        self.p, self.m, self.v, self.r = self.mem.p, self.mem.m, self.mem.v, self.mem.r
        self._stage = self.mem.stage
        self.snap = self.mem.snap
        self.m.zero_()
        self.v.zero_()
        if init_from is None:
            for (off, n, _), ls in zip(self.buckets, self.logical_start):
                inputs.fill_param_dev(self.p[off:off + n], ls)
        else:
            self.p.copy_(init_from[0]); self.m.copy_(init_from[1]); self.v.copy_(init_from[2])
        gdt = torch.int16 if wl.grad_dtype == "bf16" else torch.float32
        self.gdt = gdt
        self.hp = sh.HParams(lr=wl.lr, beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps, weight_decay=wl.weight_decay,
                             max_grad_norm=wl.max_grad_norm, num_workers=W,
                             grad_dtype=sh.GRAD_BF16 if wl.grad_dtype == "bf16" else sh.GRAD_F32,
                             reduce_op=sh.REDUCE_MEAN if mean else sh.REDUCE_SUM, num_streams=num_streams,
                             optimizer=OPTIMIZERS[optimizer], batch_bytes=batch_bytes)
        if launch is not None:
            self.hp.launch = launch
        self.optimizer = optimizer
        self._tstreams = [torch.cuda.Stream(device=self.dev) for _ in range(num_streams)] if torch_streams else None
        torch.cuda.synchronize()
        self.ctx = sh.Shadow(L, self.hp, self.p.data_ptr(), self.m.data_ptr(), None if optimizer == "sgd" else self.v.data_ptr(),
                             self.r.data_ptr() if self.r is not None else None, start_step,
                             [s.cuda_stream for s in self._tstreams] if self._tstreams else None)
        if self.snap is not None and attach_snapshot_set:
            self.ctx.snapshot_attach(self.snap[0].data_ptr(), self.snap[1].data_ptr(),
                                     None if optimizer == "sgd" else self.snap[2].data_ptr())
        self._views = None
        if resident_grads:
            self._views = [self.ctx.views_array([self.view(b, w).data_ptr() for w in range(W)])
                           for b in range(len(self.buckets))]

    def view(self, b: int, w: int) -> torch.Tensor:
        """Worker w's gradient view of bucket b inside the staging buffer."""
        n = self.buckets[b][1]
        W = self.wl.num_workers
        off = self.layout.staging_view(W, b, w)
        if self._ring_off is not None:
            off = self._ring_off[b] + off - self.layout.staging_view(W, b, 0)
        return self._stage[off:off + n * self.wl.grad_bytes].view(self.gdt)

    def fill_grads(self, step: int, buckets: Optional[Sequence[int]] = None) -> None:
        for b in (range(len(self.buckets)) if buckets is None else buckets):
            for w in range(self.wl.num_workers):
                self.inputs.fill_grad_dev(self.view(b, w), step, w, self.logical_start[b])
        torch.cuda.synchronize()

    def apply_step(self, step: int, order: Optional[Sequence[int]] = None) -> None:
        for b in (range(len(self.buckets)) if order is None else order):
            self.ctx.apply_bucket(b, self._views[b], step)

    def run_step(self, step: int, order: Optional[Sequence[int]] = None) -> None:
        self.fill_grads(step)
        self.apply_step(step, order)
        self.ctx.sync()

    def bucket_state(self, b: int):
        off, n, _ = self.buckets[b]
        self.ctx.sync()
        return tuple(x[off:off + n].cpu().numpy() for x in (self.p, self.m, self.v))

    def close(self) -> None:
        self.ctx.destroy()
